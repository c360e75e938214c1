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
// cross-lane sums, the LDS round trip, the barrier) over more elements, and narrower workgroups leave
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

// Sum over each row of 16 lanes; every lane of a row ends up with its row's total.
__device__ __forceinline__ uint32_t row16_sum(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, false);  // row_half_mirror
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, false);  // row_mirror
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

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order.
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// The lane's candidate bits against t: lane_below_packs' layout, set when key >= t.  The same sign-bit
// test as the search's counts, so the set bits of a lane number exactly the keys not counted as below t.
template <int E, bool NEG>
__device__ __forceinline__ void lane_bits_at_or_above(const float (&x)[E], float t, uint32_t (&w)[(E + 31) / 32]) {
  lane_below_packs<E, NEG>(x, t, w);
#pragma unroll
  for (int g = 0; g < (E + 31) / 32; ++g) w[g] = ~w[g] & pack_valid<E>(g);
}

// The G bits of elements g*G .. g*G + G - 1 out of lane_bits_at_or_above's words; element g*G is the
// highest of them.  G divides 32, so a group never straddles two words.
template <int E, int G>
__device__ __forceinline__ uint32_t group_bits(const uint32_t (&w)[(E + 31) / 32], int g) {
  static_assert(32 % G == 0, "a group must not straddle two words");
  const int e0 = g * G, word = e0 / 32;
  const int filled = (word == (E + 31) / 32 - 1 && E % 32 != 0) ? E % 32 : 32;
  return __builtin_amdgcn_ubfe(w[word], (uint32_t)(filled - (e0 % 32) - G), (uint32_t)G);
}

// In the lanes where pos < limit (unsigned; a lane that must not store passes pos = 0xffffffff): the value
// goes to slot pos of vals and col0 + C to slot pos of cols.  The compare leaves its mask in VCC; when
// no lane stores -- the usual case when k is a small part of the row -- one branch skips everything,
// and otherwise the mask becomes the set of active lanes for the address arithmetic and the two
// stores, with no work on the scalar unit beyond saving and restoring that set.
template <int DT, int C>
__device__ __forceinline__ void store_pair_if_below(uint32_t pos, uint32_t limit, void* vals, uint32_t value_bits,
                                                    int32_t* cols, int32_t col0) {
  uint64_t saved;
  uint32_t t1, t2;
  if constexpr (DT == kF32) {
    asm volatile(
        "v_cmp_gt_u32 vcc, %[lim], %[pos]\n\t"
        "s_cbranch_vccz 1f\n\t"
        "s_and_saveexec_b64 %[sv], vcc\n\t"
        "v_lshlrev_b32 %[t1], 2, %[pos]\n\t"
        "v_add_u32 %[t2], %[c], %[col0]\n\t"
        "global_store_dword %[t1], %[val], %[vals]\n\t"
        "global_store_dword %[t1], %[t2], %[cols]\n\t"
        "s_mov_b64 exec, %[sv]\n"
        "1:"
        : [sv] "=&s"(saved), [t1] "=&v"(t1), [t2] "=&v"(t2)
        : [lim] "s"(limit), [pos] "v"(pos), [c] "n"(C), [col0] "v"(col0), [val] "v"(value_bits), [vals] "s"(vals),
          [cols] "s"(cols)
        : "memory", "scc", "vcc");
  } else {
    uint32_t t3;
    asm volatile(
        "v_cmp_gt_u32 vcc, %[lim], %[pos]\n\t"
        "s_cbranch_vccz 1f\n\t"
        "s_and_saveexec_b64 %[sv], vcc\n\t"
        "v_lshlrev_b32 %[t1], 2, %[pos]\n\t"
        "v_lshlrev_b32 %[t3], 1, %[pos]\n\t"
        "v_add_u32 %[t2], %[c], %[col0]\n\t"
        "global_store_short %[t3], %[val], %[vals]\n\t"
        "global_store_dword %[t1], %[t2], %[cols]\n\t"
        "s_mov_b64 exec, %[sv]\n"
        "1:"
        : [sv] "=&s"(saved), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3)
        : [lim] "s"(limit), [pos] "v"(pos), [c] "n"(C), [col0] "v"(col0), [val] "v"(value_bits), [vals] "s"(vals),
          [cols] "s"(cols)
        : "memory", "scc", "vcc");
  }
}

// Register budget: a row of 64 values per lane compiles to 83 registers, i.e. 5 wavefronts per SIMD and,
// at 8 wavefronts per workgroup, two rows per compute unit.  Forcing 80 registers (a third row per
// compute unit, at the price of 5 spilled registers) measured no faster in exact mode and 7-15 % slower
// with early stopping, so the allocation is left to the compiler.
// Groups of a row that a workgroup loads ahead, during the ranking of its previous row (16-wavefront
// shape only: the others are launched with one workgroup per row): RTOPK_BLOCK_AHEAD values per lane,
// half of the row, which is what the register budget of four wavefronts per SIMD leaves free (not the
// scalar-load fallback, whose ranking by lane masks needs those registers).
#ifndef RTOPK_BLOCK_AHEAD
#define RTOPK_BLOCK_AHEAD 32
#endif
// (Measured on 1 GiB inputs: 4096 x 65536 exact 357 us with a workgroup per row, 347 us looping, 319 us with
// 32 values loaded ahead, 324 us with 24, 361 us with 40, which spills.  The narrower shapes, which have two
// to four workgroups on a compute unit whose phases overlap anyway, lose: 8192 x 32768 247 -> 278 us,
// 16384 x 16384 249 -> 299 us when each resident workgroup walks a fixed share of the rows.
// Loading the other half as well, each group of the next row into the registers of the group the ranking
// has just finished with, costs no register on paper but 23 spilled ones in practice: 319 -> 415 us.)
#ifndef RTOPK_BLOCK_PERSIST_MIN_W
#define RTOPK_BLOCK_PERSIST_MIN_W 16
#endif
constexpr bool block_persistent(int W) { return W >= RTOPK_BLOCK_PERSIST_MIN_W; }
constexpr int block_groups_ahead(int W, int G) { return block_persistent(W) && G > 1 ? RTOPK_BLOCK_AHEAD / G : 0; }

// One row, by the whole workgroup.  Every wavefront leaves through the same return statement.
template <int G, int NG, int W, int MODE, bool NEG, int DT, bool DENSE>
__device__ __forceinline__ void block_row(int64_t r, const void* __restrict__ in, int64_t N, int M, int k, int max_iter,
                                          float eps_rel, void* __restrict__ out_vals, int32_t* __restrict__ out_idx,
                                          int32_t* __restrict__ out_iters, int64_t r_next, bool& have_ahead,
                                          float (&ahead)[block_groups_ahead(W, G) * G + 1]) {
  static_assert(!DENSE || DT == kF32, "the dense form is built for fp32 rows");
  constexpr int E = G * NG;
  constexpr int T = NG * W;  // (group, wavefront) cells of a row, in column order
  constexpr int CPL = (T + kWave - 1) / kWave;  // cells per lane when one wavefront scans the table
  using ElemT = typename std::conditional<DT == kF32, float, uint16_t>::type;
  __shared__ float s_hi[W], s_nlo[W];  // per-wavefront maximum and negated minimum
  __shared__ int s_cnt[2][W];          // per-wavefront counts of a search step, double buffered
  __shared__ int s_tab[2][T];          // candidates per cell of class A / class B, then their exclusive prefixes
  // narrowing of Algorithm 1's search (see gather_band): the whole row's band, its size, and what
  // wavefront 0 hands back after finishing the search alone
  __shared__ float s_band[kBandRegs * kWave + W * kWave];  // the row's band, then one dummy word per lane of the workgroup
  __shared__ int s_tot[2];  // band members / elements at or above hi, summed over the wavefronts
  __shared__ float s_res[3];
  __shared__ int s_resi[2];

  int lane = threadIdx.x & (kWave - 1);
  asm volatile("" : "+v"(lane));  // opaque per row: nothing derived from it is carried around the loop over rows
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const ElemT* row = static_cast<const ElemT*>(in) + r * (int64_t)M;

  // Loading stage.  Lanes past M load the row's first columns (in bounds, cannot change min or max).
  // The first groups may have been loaded already, while the workgroup's previous row was ranked.
  constexpr int AHEAD = block_groups_ahead(W, G) < NG ? block_groups_ahead(W, G) : NG;
  float x[E];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int col0 = ((g * W + wave) * kWave + lane) * G;
    float v[G];
    if (g < AHEAD && have_ahead) {  // uniform
#pragma unroll
      for (int c = 0; c < G; ++c) v[c] = ahead[g * G + c];
    } else {
      load_group<DT, G>(row, col0 < M ? col0 : 0, v);
    }
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

  // cnt = #{row elements with key >= t}.  Every lane counts its keys below t, the wavefront sums them,
  // lane 0 posts the sum, and after the barrier every wavefront adds up the W posted sums itself (they sit
  // in one row of 16 lanes).  `step` selects the half of s_cnt that is written; one barrier per step is
  // enough because a half is not written again before every wavefront has passed the next barrier.
  // (Adding the lanes' counts to one LDS word with atomics instead, which saves the second reduction,
  // measured slower: 8192 x 32768 at eight steps 252 -> 266 us.)
  int step = 0;
  constexpr int kPackWords = (E + 31) / 32;
  uint32_t last[kPackWords];  // this lane's sign-bit words of the latest count
  auto count = [&](float t) -> int {
    lane_below_packs<E, NEG>(x, t, last);
    uint32_t below_lane = 0;
#pragma unroll
    for (int g = 0; g < kPackWords; ++g) below_lane += (uint32_t)__builtin_popcount(last[g]);
    const int mine = wave_sum((int)below_lane);
    const int p = step & 1;
    ++step;
    if (lane == 0) s_cnt[p][wave] = mine;
    __syncthreads();
    const int below = __builtin_amdgcn_readfirstlane((int)row16_sum(lane < W ? (uint32_t)s_cnt[p][lane] : 0u));
    return W * kWave * E - below;  // padded columns hold a key of -inf and are among the `below`
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
    // (Narrowing as soon as the band fits stays the fastest: never narrowing costs 3 % on Laplace rows --
    // 12.3 full-width steps on average at 32768 columns -- and starting only after 8 to 14 steps 7-12 %.
    // Narrowing three to four steps earlier, onto kBandRegs registers per lane of EVERY wavefront with the
    // remaining steps still going through the barrier, measured slower as well: 8192 x 32768 249 -> 263 us,
    // 4096 x 65536 319 -> 350 us; a step on one wavefront's registers costs a tenth of a step that all
    // wavefronts have to meet for.)
    // the sign-bit words of the steps that set the current lo and hi: the gather needs no compare of its own
    uint32_t below_lo[kPackWords], below_hi[kPackWords];
    bool lo_moved = false, hi_moved = false;
    auto fits = [&](int cnt) -> bool {  // after move_bound with this count
      if (cnt < k) {  // uniform
        hi_moved = true;
#pragma unroll
        for (int g = 0; g < kPackWords; ++g) below_hi[g] = last[g];
      } else {
        lo_moved = true;
#pragma unroll
        for (int g = 0; g < kPackWords; ++g) below_lo[g] = last[g];
      }
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
      // every wavefront appends its band members to the row's band (any order will do)
      const uint32_t dst = (uint32_t)(uintptr_t)s_band;
      if (!lo_moved) lane_below_packs<E, NEG>(x, lo, below_lo);  // a bound still at the row's minimum or maximum
      if (!hi_moved) lane_below_packs<E, NEG>(x, hi, below_hi);
      scatter_band_members<E, NEG>(x, below_lo, below_hi, lane, dst + (uint32_t)((kBandRegs + wave) * kWave) * 4u,
                                   [&](uint32_t n, uint32_t above) -> uint32_t {
                                     uint32_t off = 0;
                                     if (lane == 0) {
                                       off = (uint32_t)atomicAdd(&s_tot[0], (int)n);
                                       atomicAdd(&s_tot[1], (int)above);
                                     }
                                     off = (uint32_t)__builtin_amdgcn_readfirstlane((int)off);
                                     return off + n <= (uint32_t)(kBandRegs * kWave) ? dst + off * 4u : kNoRoom;
                                   });
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
    // (Counting the midpoint and both midpoints that can follow it in one pass -- two levels per barrier,
    // three counts per element -- gives the same bounds but measured slower, 250 -> 276 us at eight steps on
    // 8192 x 32768: a step is bound by its counting work, not by the barrier.)
#pragma nounroll
    for (int it = 0; it < max_iter; ++it) {
      const float thres = (lo + hi) * 0.5f;
      const int cnt = count(thres);
      move_bound(lo, hi, thres, cnt, k);
      if (cnt == k) break;
    }
    tA = lo;
  }
  // The search is over; what follows needs few registers besides the row.  A workgroup that has another
  // row to do starts that row's first loads now, so that they fly while this row is ranked and stored.
  have_ahead = false;
  if constexpr (AHEAD > 0) {
    if (r_next < N) {
      const ElemT* next = static_cast<const ElemT*>(in) + r_next * (int64_t)M;
#pragma unroll
      for (int g = 0; g < AHEAD; ++g) {
        const int col0 = ((g * W + wave) * kWave + lane) * G;
        float v[G];
        load_group<DT, G>(next, col0 < M ? col0 : 0, v);
#pragma unroll
        for (int c = 0; c < G; ++c) ahead[g * G + c] = v[c];
      }
      have_ahead = true;
    }
  }
  const bool has_b = limB > 0;  // uniform over the workgroup

  // Ranking, part 1: candidates per (group, wavefront) cell, written in column order.
  //
  // One class (every search that ended on a count of k, and Algorithm 2): all per lane.  Each lane takes
  // its elements' candidate bits from the sign of key - tA, counts them per group, and the counts of up to
  // three groups share one word (10 bits each: a wavefront holds at most 64 * 8 candidates of a group)
  // through one prefix scan over the lanes.  The scan's last lane holds the cell totals, every lane keeps
  // the candidates in lower lanes for part 3.  Against one mask, one scalar popcount and one scalar add per
  // ELEMENT this leaves the scalar unit, which the 16 wavefronts of two rows share, nearly idle.
  constexpr bool kLaneRank = G > 1;      // the scalar-load fallback (G = 1) keeps the mask form
  constexpr int kScanWords = (NG + 2) / 3;
  uint32_t cand[(E + 31) / 32];          // candidate bits of this lane
  uint32_t lower[kScanWords];            // per group, 10 bits each: candidates of the cell in lower lanes
  uint32_t cell_total[kScanWords];       // the same fields for the whole wavefront (uniform)
  if (kLaneRank && !has_b) {
    lane_bits_at_or_above<E, NEG>(x, tA, cand);
    uint32_t own[kScanWords];
#pragma unroll
    for (int j = 0; j < kScanWords; ++j) own[j] = 0;
#pragma unroll
    for (int g = 0; g < NG; ++g)
      own[g / 3] |= (uint32_t)__builtin_popcount(group_bits<E, G>(cand, g)) << (10 * (g % 3));
#pragma unroll
    for (int j = 0; j < kScanWords; ++j) {
      const uint32_t incl = wave_inclusive_scan_dpp(own[j]);
      lower[j] = incl - own[j];  // field by field: no field borrows, incl >= own in each
      cell_total[j] = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    }
    if (lane < NG) {
      // lane g posts cell g (the totals are uniform; the shift is per lane)
      uint32_t word = cell_total[0];
#pragma unroll
      for (int j = 1; j < kScanWords; ++j) word = lane / 3 == j ? cell_total[j] : word;
      s_tab[0][lane * W + wave] = (int)((word >> (10 * (lane % 3))) & 0x3ffu);
    }
  } else {
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
  if (kLaneRank && !has_b) {
    // One class, per lane: rank = cell prefix + candidates of the cell in lower lanes + own earlier
    // candidates in the group.  A lane's non-candidates get rank 0xffffffff, so that the one compare against
    // limA (which also keeps every store inside the row's k slots whatever the input held) decides who
    // stores.  Cells without a candidate are skipped as a whole.
    // (opaque copies: otherwise the group fields extracted in part 1 are kept in 16 registers for reuse here)
#pragma unroll
    for (int i = 0; i < (E + 31) / 32; ++i) asm volatile("" : "+v"(cand[i]));
    // lane g fetches the prefix of cell g: one LDS round trip for all the wavefront's cells
    const int my_cell = s_tab[0][(lane < NG ? lane : 0) * W + wave];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      if constexpr (!DENSE) {
        if (((cell_total[g / 3] >> (10 * (g % 3))) & 0x3ffu) == 0) continue;  // uniform
      }
      int ln = lane;  // opaque per group: keeps the column numbers of all groups from being hoisted
      if constexpr (NG > 4) asm volatile("" : "+v"(ln));
      const uint32_t bits = group_bits<E, G>(cand, g);
      const uint32_t before = (uint32_t)__builtin_amdgcn_readlane(my_cell, g) +
                              __builtin_amdgcn_ubfe(lower[g / 3], (uint32_t)(10 * (g % 3)), 10u);
      const int col0 = ((g * W + wave) * kWave + ln) * G;
      float y[G];
      auto one = [&](auto cc) {
        constexpr int c = decltype(cc)::value;
        const uint32_t pos = before + (c == 0 ? 0u : (uint32_t)__builtin_popcount(bits >> (G - c)));
        const uint32_t is_cand = (uint32_t)__builtin_amdgcn_sbfe(bits, (uint32_t)(G - 1 - c), 1u);  // all ones or zero
        const uint32_t rank = pos | ~is_cand;
        if constexpr (DENSE) {
          y[c] = rank < (uint32_t)limA ? x[g * G + c] : 0.0f;
        } else {
          const uint32_t fb = __float_as_uint(x[g * G + c]);
          uint32_t vb = fb;
          if constexpr (DT != kF32) vb = narrow_bits<DT>(fb);
          store_pair_if_below<DT, c>(rank, (uint32_t)limA, ov, vb, oi, col0);
        }
      };
      static_for<G>(one);
      if constexpr (DENSE) {
        if (col0 < M) store_group<G>(reinterpret_cast<float*>(ov) + col0, y);
      }
      if constexpr (NG > 4) __builtin_amdgcn_sched_barrier(0);
    }
    return;
  }
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

// Workgroup b takes rows b, b + gridDim.x, ...: with as many workgroups as rows each takes one; the widest
// shape (16 wavefronts, one workgroup to a compute unit) is launched with one workgroup per compute unit
// instead, which saves the dispatch of a new 1024-thread workgroup between a unit's rows.
template <int G, int NG, int W, int MODE, bool NEG, int DT, bool DENSE>
__global__ void __launch_bounds__(W * kWave) __attribute__((amdgpu_waves_per_eu(block_persistent(W) ? 4 : 1)))
    rtopk_block_kernel(const void* __restrict__ in, int64_t N, int M, int k, int max_iter, float eps_rel,
                       void* __restrict__ out_vals, int32_t* __restrict__ out_idx, int32_t* __restrict__ out_iters) {
  bool have_ahead = false;
  float ahead[block_groups_ahead(W, G) * G + 1];
  if constexpr (block_persistent(W)) {
    for (int64_t r = blockIdx.x; r < N; r += gridDim.x) {
      block_row<G, NG, W, MODE, NEG, DT, DENSE>(r, in, N, M, k, max_iter, eps_rel, out_vals, out_idx, out_iters,
                                                r + gridDim.x, have_ahead, ahead);
      __syncthreads();  // the next row reuses the shared tables
    }
  } else {
    const int64_t r = blockIdx.x;  // launched with one workgroup per row
    if (r < N)
      block_row<G, NG, W, MODE, NEG, DT, DENSE>(r, in, N, M, k, max_iter, eps_rel, out_vals, out_idx, out_iters, N,
                                                have_ahead, ahead);
  }
}

// Compute units of the current device (asked once per device; concurrent first calls store the same value).
inline int compute_units() {
  static int units[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  if (units[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    units[dev] = n;
  }
  return units[dev];
}

#ifndef RTOPK_BLOCK_PERSIST
#define RTOPK_BLOCK_PERSIST 1
#endif
template <int G, int NG, int W, int MODE, bool NEG = false, int DT = kF32, bool DENSE = false>
hipError_t launch_block(const LaunchArgs& a) {
  if (a.N > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  int64_t grid = a.N;
  if (RTOPK_BLOCK_PERSIST && block_persistent(W)) {
    const int64_t resident = (int64_t)compute_units() * (16 / W);  // workgroups that run at the same time
    if (resident > 0 && grid > resident) grid = resident;
  }
  return launch_kernel(rtopk_block_kernel<G, NG, W, MODE, NEG, DT, DENSE>, dim3((unsigned)grid), dim3(W * kWave), 0,
                       a.stream, a.in, a.N, a.M, a.k, a.max_iter, a.eps_rel, a.out_vals,
                       static_cast<int32_t*>(a.out_idx), a.out_iters);
}

}  // namespace rtopk
