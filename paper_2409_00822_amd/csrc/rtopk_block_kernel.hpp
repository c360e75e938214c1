// Row-wise top-k for rows wider than one wavefront's registers can hold (8192 < M <= 65536): one
// workgroup of W wavefronts per row.  Same method as rtopk_kernel.hpp (RTop-K, arXiv 2409.00822,
// Section 3.1, Algorithms 1 and 2); the paper's own kernel stops at M = 8192 (Appendix B), the width its
// shared-memory row buffer allows.  Here every wavefront keeps its slice of the row in VGPRs, and what
// the wavefronts exchange through LDS is small: the slice minima and maxima once, one count per
// wavefront per search step, and one table of per-group candidate counts for the final ranking.
//
// Layout.  Wavefront w, lane l owns NG groups of G consecutive columns:
//   element e = g*G + c  <->  column ((g*W + w)*64 + l)*G + c
// so every load instruction of a wavefront still covers 64*G*4 contiguous bytes, the W wavefronts of a
// group step cover W KiB contiguous, and column order is (g, w, lane, c).  W is 4, 8 or 16, chosen so
// that a lane holds up to 64 values: fewer, fatter wavefronts spread the per-step fixed cost (two
// cross-lane sums, the LDS round trip, the barrier) over more compares, and narrower workgroups leave
// room for more rows per compute unit, whose load and search phases then overlap.
//
// Every wavefront evaluates the same thresholds on the same totals, so all of them take the same
// branches and reach the same barriers; the trip count of the search is uniform over the workgroup.
//
// Template parameters beyond the layout, all with the meaning they have in rtopk_kernel.hpp:
//   MODE (kEarly / kExact / kEps), NEG (the k smallest), DT (fp32, half or bfloat16 rows),
//   DENSE (chosen values in place and zero elsewhere instead of (value, column) pairs; fp32 only).
#pragma once

#include "rtopk_kernel.hpp"

// Share of a lane's E values counted per lane rather than by mask popcount (see count_ge_wide): all of
// them here -- the few wavefronts that share a SIMD run in lock step between barriers, so nothing hides
// the compare -> scalar popcount latency (8192 x 32768: 397 -> 380 us).
#ifndef RTOPK_BLOCK_ACC_OF
#define RTOPK_BLOCK_ACC_OF(E) (E)
#endif

namespace rtopk {

// Inclusive prefix sum over the 64 lanes of a wavefront (not on the hot path: used once per row).
__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int t = __shfl_up(v, d, kWave);
    if (lane >= d) v += t;
  }
  return v;
}

// In the lanes whose bit is set in `mask` (a subset of the active lanes): the 32-bit (or, for 16-bit
// rows, the narrowed 16-bit) value goes to vals + off_v bytes and the column to cols + off_c bytes.  Both
// bases are wave-uniform.  The set of active lanes is saved and put back.
template <int DT>
__device__ __forceinline__ void store_pair_masked(uint64_t mask, void* vals, uint32_t off_v, uint32_t value_bits,
                                                  int32_t* cols, uint32_t off_c, int32_t col) {
  uint64_t saved;
  if constexpr (DT == kF32) {
    asm volatile(
        "s_and_saveexec_b64 %0, %1\n\t"
        "global_store_dword %2, %3, %4\n\t"
        "global_store_dword %5, %6, %7\n\t"
        "s_mov_b64 exec, %0"
        : "=&s"(saved)
        : "s"(mask), "v"(off_v), "v"(value_bits), "s"(vals), "v"(off_c), "v"(col), "s"(cols)
        : "memory", "scc");
  } else {
    asm volatile(
        "s_and_saveexec_b64 %0, %1\n\t"
        "global_store_short %2, %3, %4\n\t"
        "global_store_dword %5, %6, %7\n\t"
        "s_mov_b64 exec, %0"
        : "=&s"(saved)
        : "s"(mask), "v"(off_v), "v"(value_bits), "s"(vals), "v"(off_c), "v"(col), "s"(cols)
        : "memory", "scc");
  }
}

template <int G, int NG, int W, int MODE, bool NEG, int DT, bool DENSE>
__global__ void __launch_bounds__(W * kWave)
    rtopk_block_kernel(const void* __restrict__ in, int64_t N, int M, int k, int max_iter, float eps_rel,
                       void* __restrict__ out_vals, int32_t* __restrict__ out_idx, int32_t* __restrict__ out_iters) {
  static_assert(!DENSE || DT == kF32, "the dense form is built for fp32 rows");
  constexpr int E = G * NG;
  constexpr int T = NG * W;  // (group, wavefront) cells of a row, in column order
  constexpr int CPL = (T + kWave - 1) / kWave;  // cells per lane when one wavefront scans the table
  using ElemT = typename std::conditional<DT == kF32, float, uint16_t>::type;
  __shared__ float s_hi[W], s_nlo[W];  // per-wavefront maximum and negated minimum
  __shared__ int s_cnt[2][W];          // per-wavefront counts of a search step, double buffered
  __shared__ int s_tab[2][T];          // candidates per cell of class A / class B, then their exclusive prefixes
  // narrowing of Algorithm 1's search (see gather_band): per-wavefront gather areas, the whole row's
  // band, its size, and what wavefront 0 hands back after finishing the search alone
  __shared__ float s_gather[W][kBandRegs * kWave];
  __shared__ float s_band[kBandRegs * kWave];
  __shared__ int s_tot[2];  // band members / elements at or above hi, summed over the wavefronts
  __shared__ float s_res[3];
  __shared__ int s_resi[2];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t r = blockIdx.x;
  if (r >= N) return;
  const ElemT* row = static_cast<const ElemT*>(in) + r * (int64_t)M;

  // Loading stage.  Lanes past M load the row's first columns (in bounds, cannot change min or max).
  float x[E];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int col0 = ((g * W + wave) * kWave + lane) * G;
    float v[G];
    load_group<DT, G>(row, col0 < M ? col0 : 0, v);
#pragma unroll
    for (int c = 0; c < G; ++c) x[g * G + c] = v[c];
  }

  // Row minimum and maximum: per lane, per wavefront, then over the W wavefronts through LDS.
  float hi, lo;
  {
    float mx, nm, wmax, wmin;
    lane_max_and_negmin<E>(x, mx, nm);
    wave_max_and_negmin(mx, nm, wmax, wmin);
    if (lane == 0) {
      s_hi[wave] = wmax;
      s_nlo[wave] = -wmin;
    }
    if (threadIdx.x == 0) {
      s_tot[0] = 0;
      s_tot[1] = 0;
    }
    __syncthreads();
    float a = s_hi[0], b = s_nlo[0];
#pragma unroll
    for (int w = 1; w < W; ++w) {
      a = vmax(a, s_hi[w]);
      b = vmax(b, s_nlo[w]);
    }
    // every lane holds the same two values; saying so lets the search loop branch on scalar conditions
    const float row_max = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a)));
    const float row_min = -__int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(b)));
    // bounds of the keys (negated values for the k smallest)
    hi = NEG ? -row_min : row_max;
    lo = NEG ? -row_max : row_min;
  }

  // From here on columns past M must never be counted or chosen: their key is -inf.
  if (M != kWave * G * NG * W) {  // uniform: full-width rows skip the masking
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int col0 = (((e / G) * W + wave) * kWave + lane) * G;
      x[e] = col0 < M ? x[e] : (NEG ? __builtin_inff() : -__builtin_inff());
    }
  }

  // cnt = #{row elements with key >= t}: this wavefront's share, then the sum over the workgroup.
  // `step` selects the half of s_cnt that is written; one barrier per step is enough because a half is
  // not written again before every wavefront has passed the next barrier.
  constexpr int ACC = E <= 8 ? 0 : RTOPK_BLOCK_ACC_OF(E);
  int step = 0;
  auto count = [&](float t) -> int {
    const int mine = count_ge_wide<E, ACC, NEG>(x, t);
    const int p = step & 1;
    ++step;
    if (lane == 0) s_cnt[p][wave] = mine;
    __syncthreads();
    return wave_sum(lane < W ? s_cnt[p][lane] : 0);
  };

  // The selection is described by two classes of elements and a limit for each:
  //   class A: key >= tA, the first limA of them in column order are chosen;
  //   class B: tB <= key < tA, the first limB of them are chosen (only after a converged search).
  float tA, tB = 0.0f;
  int limA = k, limB = 0;
  if constexpr (MODE == kExact || MODE == kEps) {
    // Algorithm 1; termination, collection and iteration numbering as in select_row.  The full-width
    // steps track cnt_lo = #{key >= lo} and a lower bound cnt_hi of #{key >= hi}; once the band
    // [lo, hi) of the whole row fits kBandRegs registers per lane of ONE wavefront, it is gathered
    // there and wavefront 0 finishes the search alone, with no further barriers.
    bool hit = false, narrow = false;
    float thres = lo;
    int steps = 0, cnt_lo = M, cnt_hi = 0;
    const float eps = MODE == kEps ? eps_rel * __builtin_fabsf(hi) : 0.0f;
    auto fits = [&](int cnt) -> bool {  // after move_bound with this count
      cnt_lo = cnt < k ? cnt_lo : cnt;
      cnt_hi = cnt < k ? cnt : cnt_hi;
      return cnt_lo - cnt_hi <= kBandRegs * kWave;
    };
    if constexpr (MODE == kExact) {
      float seen = lo;
      for (;;) {
        thres = midpoint_exact<DT>(lo, hi);
        if (!(thres < seen || thres > seen)) break;
        seen = thres;
        int cnt = count(thres);
        if (cnt == k) {
          hit = true;
          break;
        }
        move_bound(lo, hi, thres, cnt, k);
        if (fits(cnt)) {
          narrow = true;
          break;
        }
        thres = midpoint_exact<DT>(lo, hi);
        cnt = count(thres);
        if (cnt == k) {
          hit = true;
          break;
        }
        move_bound(lo, hi, thres, cnt, k);
        if (fits(cnt)) {
          narrow = true;
          break;
        }
      }
    } else {
      while (hi - lo > eps) {
        const float mid = (lo + hi) * 0.5f;
        if (!(mid > lo && mid < hi)) break;
        thres = mid;
        ++steps;
        const int cnt = count(thres);
        if (cnt == k) {
          hit = true;
          break;
        }
        move_bound(lo, hi, thres, cnt, k);
        if (fits(cnt)) {
          narrow = true;
          break;
        }
      }
    }
    if (narrow) {  // uniform over the workgroup
      // every wavefront gathers its own band members, then appends them to the row's band
      float band[kBandRegs];
      uint32_t nb;
      const int above = gather_band<E, NEG, true>(x, lo, hi, lane, (uint32_t)(uintptr_t)s_gather[wave], band, nb);
      // a place in the row's band for this wavefront's members (any order will do)
      uint32_t off = 0;
      if (lane == 0) {
        off = (uint32_t)atomicAdd(&s_tot[0], (int)nb);
        atomicAdd(&s_tot[1], above);
      }
      off = (uint32_t)__builtin_amdgcn_readfirstlane((int)off);
      const uint32_t dst = (uint32_t)(uintptr_t)s_band;
#pragma unroll
      for (int j = 0; j < kBandRegs; ++j) {
        const uint32_t i = (uint32_t)lane + 64u * j;
        lds_store_masked(__builtin_amdgcn_ballot_w64(i < nb), dst + (off + i) * 4u, band[j]);
      }
      __syncthreads();
      if (wave == 0) {
        float all[kBandRegs];
        const uint32_t total = (uint32_t)__builtin_amdgcn_readfirstlane(s_tot[0]);
        const int above_all = __builtin_amdgcn_readfirstlane(s_tot[1]);
        load_band<NEG, kBandRegs>(dst, lane, total, all);
        search_band<MODE, NEG, DT, kBandRegs>(all, above_all, k, eps, lo, hi, thres, hit, steps);
        if (lane == 0) {
          s_res[0] = lo;
          s_res[1] = hi;
          s_res[2] = thres;
          s_resi[0] = hit ? 1 : 0;
          s_resi[1] = steps;
        }
      }
      __syncthreads();
      lo = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s_res[0])));
      hi = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s_res[1])));
      thres = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s_res[2])));
      hit = __builtin_amdgcn_readfirstlane(s_resi[0]) != 0;
      steps = __builtin_amdgcn_readfirstlane(s_resi[1]);
    }
    if constexpr (MODE == kEps) {
      if (out_iters != nullptr && threadIdx.x == 0) out_iters[r] = hit ? steps : steps + 1;
    }
    if (hit) {
      tA = thres;
    } else {
      const int na = count(hi);
      tA = hi;
      tB = lo;
      limA = na < k ? na : k;
      limB = k - limA;
    }
  } else {
    // Algorithm 2: max_iter steps (fewer once a step counts exactly k), then the first k of key >= lo.
    for (int it = 0; it < max_iter; ++it) {
      const float thres = (lo + hi) * 0.5f;
      const int cnt = count(thres);
      move_bound(lo, hi, thres, cnt, k);
      if (cnt == k) break;
    }
    tA = lo;
  }
  const bool has_b = limB > 0;  // uniform over the workgroup

  // Ranking, part 1: candidates per (group, wavefront) cell, written in column order.
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    int nA = 0, nB = 0;
#pragma unroll
    for (int c = 0; c < G; ++c) {
      const float v = keyof<NEG>(x[g * G + c]);
      nA += __builtin_popcountll(__builtin_amdgcn_ballot_w64(v >= tA));
      if (has_b) nB += __builtin_popcountll(__builtin_amdgcn_ballot_w64(v >= tB && !(v >= tA)));
    }
    if (lane == 0) {
      s_tab[0][g * W + wave] = nA;
      s_tab[1][g * W + wave] = nB;
    }
    if constexpr (NG > 4) __builtin_amdgcn_sched_barrier(0);  // keep the groups' masks from piling up
  }
  __syncthreads();
  // Part 2: exclusive prefix over the cells (wavefront 0 scans class A, wavefront 1 class B).
  if (wave < 2) {
    int* tab = s_tab[wave];
    int v[CPL], sum = 0;
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
      const int f = lane * CPL + j;
      v[j] = f < T ? tab[f] : 0;
      sum += v[j];
    }
    int before = wave_inclusive_scan(sum, lane) - sum;
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
      const int f = lane * CPL + j;
      if (f < T) tab[f] = before;
      before += v[j];
    }
  }
  __syncthreads();

  // Part 3: every wavefront ranks its own elements.  Pairs go straight to the outputs at 4 (or 2) bytes
  // times their rank (k can be far larger than LDS could stage; consecutive ranks fall on consecutive
  // lanes, so the stores are still mostly coalesced); the dense form keeps or zeroes each element in
  // place and stores the row with the accesses it was loaded with.
  using OutT = typename std::conditional<DT == kF32, uint32_t, uint16_t>::type;  // value bits as stored
  OutT* ov = static_cast<OutT*>(out_vals) + r * (int64_t)(DENSE ? M : k);
  int32_t* oi = DENSE ? nullptr : out_idx + r * (int64_t)k;
  if (!has_b) {
    // One class: rank = cell prefix + chosen elements in lower lanes + own earlier elements.
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      int ln = lane;  // opaque per group: keeps the column numbers of all groups from being hoisted
      if constexpr (NG > 4) asm volatile("" : "+v"(ln));
      uint64_t m[G];
      uint32_t pos = (uint32_t)__builtin_amdgcn_readfirstlane(s_tab[0][g * W + wave]);
#pragma unroll
      for (int c = 0; c < G; ++c) {
        m[c] = __builtin_amdgcn_ballot_w64(keyof<NEG>(x[g * G + c]) >= tA);
        pos = lanes_below(m[c], pos);
      }
      const int col0 = ((g * W + wave) * kWave + ln) * G;
      float y[G];
#pragma unroll
      for (int c = 0; c < G; ++c) {
        const uint64_t mk = m[c] & __builtin_amdgcn_ballot_w64(pos < (uint32_t)limA);
        if constexpr (DENSE) {
          y[c] = keep_where(x[g * G + c], mk);
        } else {
          const uint32_t fb = __float_as_uint(x[g * G + c]);
          uint32_t bits = fb;
          if constexpr (DT != kF32) bits = narrow_bits<DT>(fb);
          // most masks are empty when k is a small part of the row: skip their store instructions
          if (mk != 0) store_pair_masked<DT>(mk, ov, pos * (uint32_t)sizeof(OutT), bits, oi, pos * 4u, col0 + c);
        }
        if (c + 1 < G) pos = add_mask_bit(pos, m[c]);
      }
      if constexpr (DENSE) {
        if (col0 < M) store_group<G>(reinterpret_cast<float*>(ov) + col0, y);
      }
      if constexpr (NG > 4) __builtin_amdgcn_sched_barrier(0);
    }
    return;
  }
  // Two classes (a search that converged on a value tied across the k-th place): rare, kept plain.
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    uint32_t posA = (uint32_t)s_tab[0][g * W + wave];
    uint32_t posB = (uint32_t)s_tab[1][g * W + wave];
    bool a[G], b[G];
#pragma unroll
    for (int c = 0; c < G; ++c) {
      const float v = keyof<NEG>(x[g * G + c]);
      a[c] = v >= tA;
      b[c] = v >= tB && !a[c];
      posA = lanes_below(__builtin_amdgcn_ballot_w64(a[c]), posA);
      posB = lanes_below(__builtin_amdgcn_ballot_w64(b[c]), posB);
    }
    const int col0 = ((g * W + wave) * kWave + lane) * G;
    float y[G];
#pragma unroll
    for (int c = 0; c < G; ++c) {
      const uint32_t selA = posA < (uint32_t)limA ? posA : (uint32_t)limA;  // chosen A's before this element
      const uint32_t selB = posB < (uint32_t)limB ? posB : (uint32_t)limB;
      const bool chosen = (a[c] && posA < (uint32_t)limA) || (b[c] && posB < (uint32_t)limB);
      if constexpr (DENSE) {
        y[c] = chosen ? x[g * G + c] : 0.0f;
      } else {
        if (chosen) {
          const uint32_t pos = selA + selB;
          const uint32_t fb = __float_as_uint(x[g * G + c]);
          uint32_t bits = fb;
          if constexpr (DT != kF32) bits = narrow_bits<DT>(fb);
          ov[pos] = (OutT)bits;
          oi[pos] = col0 + c;
        }
      }
      posA += a[c] ? 1u : 0u;
      posB += b[c] ? 1u : 0u;
    }
    if constexpr (DENSE) {
      if (col0 < M) store_group<G>(reinterpret_cast<float*>(ov) + col0, y);
    }
    if constexpr (NG > 4) __builtin_amdgcn_sched_barrier(0);
  }
}

template <int G, int NG, int W, int MODE, bool NEG = false, int DT = kF32, bool DENSE = false>
hipError_t launch_block(const LaunchArgs& a) {
  if (a.N > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  return launch_kernel(rtopk_block_kernel<G, NG, W, MODE, NEG, DT, DENSE>, dim3((unsigned)a.N), dim3(W * kWave), 0,
                       a.stream, a.in, a.N, a.M, a.k, a.max_iter, a.eps_rel, a.out_vals,
                       static_cast<int32_t*>(a.out_idx), a.out_iters);
}

}  // namespace rtopk
