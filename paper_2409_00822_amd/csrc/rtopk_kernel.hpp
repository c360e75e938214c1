// Row-wise top-k selection kernels for gfx950 (MI355X): one 64-lane wavefront per row, the row held
// in VGPRs from the first load to the last store.
//
// Method: RTop-K (arXiv 2409.00822), Section 3.1.  Algorithm 1 with epsilon = 0 (exact mode) and
// Algorithm 2 (early stopping).  Per row: min / max, then a binary search over a threshold with
// cnt = #{v >= thres} per step, then the k chosen (value, column) pairs are emitted in ascending
// column order.  The paper's own kernel (Section 3.2) keeps the row in shared memory and reduces
// counts with shuffles; here the row never leaves registers, a compare writes the 64-lane mask
// straight to scalar registers, and the count is a scalar popcount.
//
// Data layout inside a wavefront.  A lane owns NG groups of G consecutive columns:
//   element e = g*G + c  (0 <= g < NG, 0 <= c < G)  <->  column (g*64 + lane)*G + c
// so that every load instruction of a wavefront covers 64*G*4 contiguous bytes (1 KiB for G = 4).
// Column order is therefore (g, lane, c), which is the order the ranking below follows.
//
// A wavefront handles R consecutive rows.  It issues all R rows' loads before the first search, and
// stages the R*k selected pairs in LDS so that the final stores are whole 128-bit, fully coalesced
// writes of R*k contiguous outputs.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rtopk_dispatch.hpp"

namespace rtopk {

constexpr int kWave = 64;

// ---- cross-lane helpers ---------------------------------------------------------------------------

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float keep, float src) {
  return __int_as_float(
      __builtin_amdgcn_update_dpp(__float_as_int(keep), __float_as_int(src), CTRL, ROW_MASK, 0xf, false));
}

// v_min_f32 / v_max_f32 on finite data; written as asm so that no NaN-quieting canonicalisation is
// added around values that come straight from memory.
__device__ __forceinline__ float vmin(float a, float b) {
  float r;
  asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float vmax(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Butterfly inside each row of 16 lanes, then two row broadcasts; lane 63 ends up with the result.
template <bool IS_MAX>
__device__ __forceinline__ float wave_reduce(float v) {
  auto op = [](float a, float b) { return IS_MAX ? vmax(a, b) : vmin(a, b); };
  v = op(v, dpp_move<0xB1, 0xf>(v, v));   // quad_perm [1,0,3,2]
  v = op(v, dpp_move<0x4E, 0xf>(v, v));   // quad_perm [2,3,0,1]
  v = op(v, dpp_move<0x141, 0xf>(v, v));  // row_half_mirror
  v = op(v, dpp_move<0x140, 0xf>(v, v));  // row_mirror
  v = op(v, dpp_move<0x142, 0xa>(v, v));  // row_bcast:15 into rows 1 and 3
  v = op(v, dpp_move<0x143, 0xc>(v, v));  // row_bcast:31 into rows 2 and 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask, uint32_t add) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, add));
}

// ---- one row ----------------------------------------------------------------------------------------

// cnt = #{e, lane : x[e] >= t}.  The compare writes a 64-lane mask to scalar registers; the count is
// a scalar popcount, so no cross-lane reduction is needed.
template <int E>
__device__ __forceinline__ int count_ge(const float (&x)[E], float t) {
  int cnt = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) cnt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(x[e] >= t));
  return cnt;
}

// Selecting stage.  An element is a candidate of class A when x >= ta, of class B when tb <= x < ta.
// All of A is wanted first (cut at `limit`, in column order), then the first `need_b` members of B in
// column order.  The chosen pairs are written to stage[0 .. ) in ascending column order
// (g, lane, c).  With need_b == 0 this is the one-pass selection "first `limit` of x >= ta".
template <int G, int NG, bool TWO_LEVEL>
__device__ __forceinline__ void compact_row(const float (&x)[G * NG], int lane, float ta, float tb, int limit,
                                            int need_b, uint2* stage) {
  uint32_t base = 0;    // wave-uniform: chosen elements in earlier groups
  uint32_t base_b = 0;  // wave-uniform: class-B elements in earlier groups
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    bool p[G];
    if constexpr (TWO_LEVEL) {
      bool b[G];
      uint64_t mb[G];
      uint32_t pos_b = base_b;
#pragma unroll
      for (int c = 0; c < G; ++c) {
        const float v = x[g * G + c];
        p[c] = v >= ta;
        b[c] = (v >= tb) && !p[c];
        mb[c] = __builtin_amdgcn_ballot_w64(b[c]);
        pos_b = lanes_below(mb[c], pos_b);
      }
#pragma unroll
      for (int c = 0; c < G; ++c) {
        p[c] = p[c] || (b[c] && pos_b < (uint32_t)need_b);
        pos_b += b[c] ? 1u : 0u;
        base_b += (uint32_t)__builtin_popcountll(mb[c]);
      }
    } else {
#pragma unroll
      for (int c = 0; c < G; ++c) p[c] = x[g * G + c] >= ta;
    }
    uint32_t pos = base;
    uint64_t mk[G];
#pragma unroll
    for (int c = 0; c < G; ++c) {
      mk[c] = __builtin_amdgcn_ballot_w64(p[c]);
      pos = lanes_below(mk[c], pos);
    }
#pragma unroll
    for (int c = 0; c < G; ++c) {
      if (p[c] && pos < (uint32_t)limit) {
        stage[pos] = make_uint2(__float_as_uint(x[g * G + c]), (uint32_t)((g * kWave + lane) * G + c));
      }
      pos += p[c] ? 1u : 0u;
    }
#pragma unroll
    for (int c = 0; c < G; ++c) base += (uint32_t)__builtin_popcountll(mk[c]);
  }
}

// Search and selection for one row held as x[E] (columns past M hold -inf and are never chosen).
//   EXACT: Algorithm 1 at epsilon = 0; otherwise Algorithm 2 with max_iter steps.
template <int G, int NG, bool FULL, bool EXACT>
__device__ __forceinline__ void select_row(const float (&x)[G * NG], int lane, int M, int k, int max_iter,
                                           uint2* stage) {
  constexpr int E = G * NG;
  const float kInf = __builtin_inff();

  // Alg. 1 / Alg. 2, first two steps: row minimum and maximum.
  float mx = x[0];
  float mn = (FULL || lane * G < M) ? x[0] : kInf;
#pragma unroll
  for (int e = 1; e < E; ++e) {
    mx = vmax(mx, x[e]);
    const bool valid = FULL || ((e / G) * kWave + lane) * G < M;
    mn = vmin(mn, valid ? x[e] : kInf);
  }
  float lo = wave_reduce<false>(mn);
  float hi = wave_reduce<true>(mx);

  if constexpr (EXACT) {
    // The loop ends on cnt == k, or when the fp32 midpoint is no longer strictly inside (lo, hi):
    // then no representable threshold separates the remaining candidates.
    float thres = lo;
    bool hit = false;
    for (;;) {
      thres = (lo + hi) * 0.5f;
      if (!(thres > lo && thres < hi)) break;
      const int cnt = count_ge<E>(x, thres);
      if (cnt == k) {
        hit = true;
        break;
      }
      if (cnt < k) {
        hi = thres;
      } else {
        lo = thres;
      }
    }
    if (hit) {
      compact_row<G, NG, false>(x, lane, thres, thres, k, 0, stage);
    } else {
      // Everything >= hi is in the answer (fewer than k of them unless hi is still the row maximum,
      // in which case they are all equal); the rest comes from [lo, hi) by ascending column.
      const int na = count_ge<E>(x, hi);
      compact_row<G, NG, true>(x, lane, hi, lo, k, k - (na < k ? na : k), stage);
    }
  } else {
    for (int it = 0; it < max_iter; ++it) {
      const float thres = (lo + hi) * 0.5f;
      const int cnt = count_ge<E>(x, thres);
      if (cnt < k) {
        hi = thres;
      } else {
        lo = thres;
        // cnt == k: lo can from now on only move to thresholds that still count exactly k, so the
        // selection is already final.
        if (cnt == k) break;
      }
    }
    compact_row<G, NG, false>(x, lane, lo, lo, k, 0, stage);
  }
}

// ---- kernel -----------------------------------------------------------------------------------------

template <int G>
struct VecOf;
template <>
struct VecOf<1> {
  using type = float;
};
template <>
struct VecOf<2> {
  using type = float2;
};
template <>
struct VecOf<4> {
  using type = float4;
};

template <int G, int NG, int R, bool FULL, bool EXACT, typename IdxT>
__global__ void __launch_bounds__(256)
    rtopk_wave_kernel(const float* __restrict__ in, int64_t N, int M, int k, int max_iter,
                      float* __restrict__ out_vals, IdxT* __restrict__ out_idx, int vec_store) {
  constexpr int E = G * NG;
  extern __shared__ uint2 stage_all[];  // [waves per block][R * k] (value bits, column)

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int waves_per_block = (int)(blockDim.x >> 6);
  const int64_t r0 = ((int64_t)blockIdx.x * waves_per_block + wave) * R;
  if (r0 >= N) return;
  const int nrows = (N - r0 < R) ? (int)(N - r0) : R;
  uint2* stage = stage_all + (size_t)wave * R * k;

  // Loading stage: all R rows' loads are issued before any is consumed.
  float x[R][E];
  using V = typename VecOf<G>::type;
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    const float* row = in + (r0 + (rr < nrows ? rr : 0)) * (int64_t)M;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int col0 = (g * kWave + lane) * G;
      if (FULL || col0 < M) {
        const V v = *reinterpret_cast<const V*>(row + col0);
        if constexpr (G == 1) {
          x[rr][g] = v;
        } else if constexpr (G == 2) {
          x[rr][g * 2 + 0] = v.x;
          x[rr][g * 2 + 1] = v.y;
        } else {
          x[rr][g * 4 + 0] = v.x;
          x[rr][g * 4 + 1] = v.y;
          x[rr][g * 4 + 2] = v.z;
          x[rr][g * 4 + 3] = v.w;
        }
      } else {
#pragma unroll
        for (int c = 0; c < G; ++c) x[rr][g * G + c] = -__builtin_inff();
      }
    }
  }

  // Searching and selecting stages, row by row.
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    if (rr < nrows) select_row<G, NG, FULL, EXACT>(x[rr], lane, M, k, max_iter, stage + (size_t)rr * k);
  }

  // Dump: the wavefront's nrows*k staged pairs are contiguous in both output arrays.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const int total = nrows * k;
  float* ov = out_vals + r0 * (int64_t)k;
  IdxT* oi = out_idx + r0 * (int64_t)k;
  if (vec_store) {
    for (int q = lane; q < (total >> 2); q += kWave) {
      const uint4 a = *reinterpret_cast<const uint4*>(stage + 4 * q);
      const uint4 b = *reinterpret_cast<const uint4*>(stage + 4 * q + 2);
      reinterpret_cast<uint4*>(ov)[q] = make_uint4(a.x, a.z, b.x, b.z);
      if constexpr (sizeof(IdxT) == 4) {
        reinterpret_cast<uint4*>(oi)[q] = make_uint4(a.y, a.w, b.y, b.w);
      } else {
        reinterpret_cast<uint32_t*>(oi)[q] = a.y | (a.w << 8) | (b.y << 16) | (b.w << 24);
      }
    }
  } else {
    for (int q = lane; q < total; q += kWave) {
      const uint2 a = stage[q];
      ov[q] = __uint_as_float(a.x);
      oi[q] = (IdxT)a.y;
    }
  }
}

// ---- host-side launcher -------------------------------------------------------------------------------

template <int G, int NG, int R, bool FULL, bool EXACT, typename IdxT>
hipError_t launch(const LaunchArgs& a) {
  // LDS per wavefront: R*k staged pairs of 8 bytes; at most 64 KiB per block.
  const size_t per_wave = (size_t)R * (size_t)a.k * sizeof(uint2);
  int waves = 4;
  while (waves > 1 && per_wave * waves > 65536) waves >>= 1;
  const int64_t batches = (a.N + R - 1) / R;
  const int64_t blocks = (batches + waves - 1) / waves;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  hipLaunchKernelGGL((rtopk_wave_kernel<G, NG, R, FULL, EXACT, IdxT>), dim3((unsigned)blocks), dim3(waves * kWave),
                     per_wave * waves, a.stream, a.in, a.N, a.M, a.k, a.max_iter, a.out_vals,
                     static_cast<IdxT*>(a.out_idx), a.vec_store);
  return hipGetLastError();
}

// Rows per wavefront for E = G*NG registers per row: keep R*E at about 32 VGPRs.
constexpr int rows_per_wave(int E) { return E <= 4 ? 8 : (E <= 8 ? 4 : (E <= 16 ? 2 : 1)); }

}  // namespace rtopk
