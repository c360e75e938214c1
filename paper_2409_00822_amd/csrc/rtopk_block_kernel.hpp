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
#pragma once

#include "rtopk_kernel.hpp"

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

template <int G, int NG, int W, int MODE>
__global__ void __launch_bounds__(W * kWave)
    rtopk_block_kernel(const float* __restrict__ in, int64_t N, int M, int k, int max_iter,
                       float* __restrict__ out_vals, int32_t* __restrict__ out_idx) {
  constexpr int E = G * NG;
  constexpr int T = NG * W;  // (group, wavefront) cells of a row, in column order
  constexpr int CPL = (T + kWave - 1) / kWave;  // cells per lane when one wavefront scans the table
  __shared__ float s_hi[W], s_nlo[W];  // per-wavefront maximum and negated minimum
  __shared__ int s_cnt[2][W];          // per-wavefront counts of a search step, double buffered
  __shared__ int s_tab[2][T];          // candidates per cell of class A / class B, then their exclusive prefixes

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t r = blockIdx.x;
  if (r >= N) return;
  const float* row = in + r * (int64_t)M;

  // Loading stage.  Lanes past M load the row's first columns (in bounds, cannot change min or max).
  float x[E];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int col0 = ((g * W + wave) * kWave + lane) * G;
    float v[G];
    load_group<kF32, G>(row, col0 < M ? col0 : 0, v);
#pragma unroll
    for (int c = 0; c < G; ++c) x[g * G + c] = v[c];
  }

  // Row minimum and maximum: per lane, per wavefront, then over the W wavefronts through LDS.
  float mx = x[0], nm = -x[0];
#pragma unroll
  for (int e = 1; e < E; ++e) {
    mx = vmax(mx, x[e]);
    nm = vmax_an(nm, x[e]);
  }
  float hi, lo;
  wave_max_and_negmin(mx, nm, hi, lo);
  if (lane == 0) {
    s_hi[wave] = hi;
    s_nlo[wave] = -lo;
  }
  __syncthreads();
  {
    float a = s_hi[0], b = s_nlo[0];
#pragma unroll
    for (int w = 1; w < W; ++w) {
      a = vmax(a, s_hi[w]);
      b = vmax(b, s_nlo[w]);
    }
    // every lane holds the same two values; saying so lets the search loop branch on scalar conditions
    hi = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a)));
    lo = -__int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(b)));
  }

  // From here on columns past M must never be counted or chosen.
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int col0 = (((e / G) * W + wave) * kWave + lane) * G;
    x[e] = col0 < M ? x[e] : -__builtin_inff();
  }

  // cnt = #{row elements >= t}: this wavefront's share, then the sum over the workgroup.  `step`
  // selects the half of s_cnt that is written; one barrier per step is enough because a half is not
  // written again before every wavefront has passed the next barrier.
  constexpr int ACC = E <= 8 ? 0 : (E - 3) / 3;
  int step = 0;
  auto count = [&](float t) -> int {
    const int mine = count_ge_wide<E, ACC, false>(x, t);
    const int p = step & 1;
    ++step;
    if (lane == 0) s_cnt[p][wave] = mine;
    __syncthreads();
    return wave_sum(lane < W ? s_cnt[p][lane] : 0);
  };

  // The selection is described by two classes of elements and a limit for each:
  //   class A: x >= tA, the first limA of them in column order are chosen;
  //   class B: tB <= x < tA, the first limB of them are chosen (only after a converged search).
  float tA, tB = 0.0f;
  int limA = k, limB = 0;
  if constexpr (MODE == kExact) {
    // Algorithm 1 at epsilon = 0; termination and collection as in select_row.
    bool hit = false;
    float thres = lo, seen = lo;
    for (;;) {
      thres = (lo + hi) * 0.5f;
      if (!(thres < seen || thres > seen)) break;
      seen = thres;
      int cnt = count(thres);
      if (cnt == k) {
        hit = true;
        break;
      }
      move_bound(lo, hi, thres, cnt, k);
      thres = (lo + hi) * 0.5f;
      cnt = count(thres);
      if (cnt == k) {
        hit = true;
        break;
      }
      move_bound(lo, hi, thres, cnt, k);
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
    // Algorithm 2: max_iter steps (fewer once a step counts exactly k), then the first k of x >= lo.
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
      const float v = x[g * G + c];
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
  // Part 3: every wavefront ranks its own elements and writes the chosen pairs straight to the
  // outputs (k can be far larger than LDS could stage; consecutive ranks fall on consecutive lanes,
  // so the stores are still mostly coalesced).
  float* ov = out_vals + r * (int64_t)k;
  int32_t* oi = out_idx + r * (int64_t)k;
  if (!has_b) {
    // One class: rank = cell prefix + chosen elements in lower lanes + own earlier elements; the pair
    // goes to byte offset 4*rank of both outputs under EXEC = (candidate and rank < limA).  The
    // kernel's control flow is uniform over the wavefront, so EXEC is all ones here and is restored so.
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      int ln = lane;  // opaque per group: keeps the column numbers of all groups from being hoisted
      if constexpr (NG > 4) asm volatile("" : "+v"(ln));
      uint64_t m[G];
      uint32_t pos = (uint32_t)__builtin_amdgcn_readfirstlane(s_tab[0][g * W + wave]);
#pragma unroll
      for (int c = 0; c < G; ++c) {
        m[c] = __builtin_amdgcn_ballot_w64(x[g * G + c] >= tA);
        pos = lanes_below(m[c], pos);
      }
#pragma unroll
      for (int c = 0; c < G; ++c) {
        const uint64_t mk = m[c] & __builtin_amdgcn_ballot_w64(pos < (uint32_t)limA);
        const uint32_t off = pos * 4u;
        const int32_t col = ((g * W + wave) * kWave + ln) * G + c;
        asm volatile(
            "s_mov_b64 exec, %0\n\t"
            "global_store_dword %1, %2, %3\n\t"
            "global_store_dword %1, %4, %5\n\t"
            "s_mov_b64 exec, -1"
            :
            : "s"(mk), "v"(off), "v"(x[g * G + c]), "s"(ov), "v"(col), "s"(oi)
            : "memory");
        if (c + 1 < G) pos = add_mask_bit(pos, m[c]);
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
      const float v = x[g * G + c];
      a[c] = v >= tA;
      b[c] = v >= tB && !a[c];
      posA = lanes_below(__builtin_amdgcn_ballot_w64(a[c]), posA);
      posB = lanes_below(__builtin_amdgcn_ballot_w64(b[c]), posB);
    }
#pragma unroll
    for (int c = 0; c < G; ++c) {
      const uint32_t selA = posA < (uint32_t)limA ? posA : (uint32_t)limA;  // chosen A's before this element
      const uint32_t selB = posB < (uint32_t)limB ? posB : (uint32_t)limB;
      if ((a[c] && posA < (uint32_t)limA) || (b[c] && posB < (uint32_t)limB)) {
        const uint32_t pos = selA + selB;
        ov[pos] = x[g * G + c];
        oi[pos] = ((g * W + wave) * kWave + lane) * G + c;
      }
      posA += a[c] ? 1u : 0u;
      posB += b[c] ? 1u : 0u;
    }
    if constexpr (NG > 4) __builtin_amdgcn_sched_barrier(0);
  }
}

template <int G, int NG, int W, int MODE>
hipError_t launch_block(const LaunchArgs& a) {
  if (a.N > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  hipLaunchKernelGGL((rtopk_block_kernel<G, NG, W, MODE>), dim3((unsigned)a.N), dim3(W * kWave), 0, a.stream,
                     static_cast<const float*>(a.in), a.N, a.M, a.k, a.max_iter, static_cast<float*>(a.out_vals),
                     static_cast<int32_t*>(a.out_idx));
  return hipGetLastError();
}

}  // namespace rtopk
