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

#include <type_traits>
#include <utility>

#include "rtopk_dispatch.hpp"

namespace rtopk {

constexpr int kWave = 64;

// Wavefronts per workgroup.  The wavefronts of a workgroup share nothing, so the workgroup is only a
// unit of dispatch; one wavefront each spreads the rows most evenly over the compute units.  Against
// 4 per workgroup: equal at the headline shape (1.3 GB per launch), 3-10 % faster where a launch
// touches more memory or holds more registers (2.4M x 256: 530 -> 512 us, 2^20 x 1024: 900 -> 868 us,
// 65536 x 4096: 207 -> 199 us).
#ifndef RTOPK_WAVES_PER_BLOCK
#define RTOPK_WAVES_PER_BLOCK 1
#endif

// Host side: enqueue `kernel` and return the status of THIS launch.  The runtime's per-thread "last error"
// is neither read nor cleared, so an error left behind by the caller's own earlier HIP calls is not
// reported as a failure of the library, and stays visible to the caller.
template <typename T>
struct same_type {
  using type = T;
};
template <typename... KArgs>
hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream,
                         typename same_type<KArgs>::type... args) {
  void* ptrs[] = {static_cast<void*>(&args)...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, stream);
}

// ---- cross-lane helpers ---------------------------------------------------------------------------

// v_max_f32 with optional source negation, written as asm so that no NaN-quieting canonicalisation
// is added around values that come straight from memory.
__device__ __forceinline__ float vmax(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float vmax_an(float a, float b) {  // max(a, -b)
  float r;
  asm("v_max_f32_e64 %0, %1, -%2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float vmax_nn(float a, float b) {  // max(-a, -b) = -min(a, b)
  float r;
  asm("v_max_f32_e64 %0, -%1, -%2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

__device__ __forceinline__ float vmax3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float vmax3_nnn(float a, float b, float c) {  // max(-a, -b, -c)
  float r;
  asm("v_max3_f32 %0, -%1, -%2, -%3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float vmax3_ann(float a, float b, float c) {  // max(a, -b, -c)
  float r;
  asm("v_max3_f32 %0, %1, -%2, -%3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Row maximum and minimum in one reduction.  On entry every lane holds mx = max of its elements and
// nm = max of its negated elements.  The two halves of the wavefront are swapped so that lanes 0..31
// reduce the maxima and lanes 32..63 the negated minima with the same five DPP steps.
__device__ __forceinline__ void wave_max_and_negmin(float mx, float nm, float& hi, float& lo) {
  asm("s_nop 1\n\t"
      "v_permlane32_swap_b32 %0, %1\n\t"
      "s_nop 1\n\t"
      "v_max_f32 %0, %0, %1\n\t"
      "s_nop 1\n\t"
      "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\t"
      "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\t"
      "v_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\t"
      "v_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\t"
      "v_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(mx), "+v"(nm));
  hi = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx), 31));
  lo = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx), 63) ^ (int)0x80000000);
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask, uint32_t add) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, add));
}

// The search key of a value: the value itself when the k largest are wanted, its negation when the
// k smallest are (Section 3 states the problem for either end of the order and develops the largest).
// The negation folds into the source modifiers of the compares, so the smallest-k variant costs nothing
// extra.
template <bool NEG>
__device__ __forceinline__ float keyof(float v) {
  return NEG ? -v : v;
}

// p + (bit `lane` of mask): one add-with-carry whose carry-in is the lane mask.
__device__ __forceinline__ uint32_t add_mask_bit(uint32_t p, uint64_t mask) {
  uint32_t r;
  asm("v_addc_co_u32_e64 %0, vcc, %1, 0, %2" : "=v"(r) : "v"(p), "s"(mask) : "vcc");
  return r;
}

// In the lanes whose bit is set in `mask`: LDS[addr] = a, LDS[addr + 4] = b.  `mask` must be a subset of
// the lanes active at the call (every mask here comes from a ballot, which is); the set of active lanes
// is saved and put back, so the block is also correct under divergent control flow.
__device__ __forceinline__ void lds_store_pair_masked(uint64_t mask, uint32_t addr, uint32_t a, uint32_t b) {
  uint64_t saved;
  asm volatile(
      "s_and_saveexec_b64 %0, %1\n\t"
      "ds_write2_b32 %2, %3, %4 offset1:1\n\t"
      "s_mov_b64 exec, %0"
      : "=&s"(saved)
      : "s"(mask), "v"(addr), "v"(a), "v"(b)
      : "memory", "scc");
}

// The same for four elements at once (the active lanes are saved and restored once for the four).
__device__ __forceinline__ void lds_store_pairs_masked4(const uint64_t (&mk)[4], const uint32_t (&addr)[4],
                                                        const float (&a)[4], const uint32_t (&b)[4]) {
  uint64_t saved;
  asm volatile(
      "s_and_saveexec_b64 %[sv], %[m0]\n\t"
      "ds_write2_b32 %[a0], %[v0], %[c0] offset1:1\n\t"
      "s_mov_b64 exec, %[m1]\n\t"
      "ds_write2_b32 %[a1], %[v1], %[c1] offset1:1\n\t"
      "s_mov_b64 exec, %[m2]\n\t"
      "ds_write2_b32 %[a2], %[v2], %[c2] offset1:1\n\t"
      "s_mov_b64 exec, %[m3]\n\t"
      "ds_write2_b32 %[a3], %[v3], %[c3] offset1:1\n\t"
      "s_mov_b64 exec, %[sv]"
      : [sv] "=&s"(saved)
      : [m0] "s"(mk[0]), [m1] "s"(mk[1]), [m2] "s"(mk[2]), [m3] "s"(mk[3]), [a0] "v"(addr[0]), [a1] "v"(addr[1]),
        [a2] "v"(addr[2]), [a3] "v"(addr[3]), [v0] "v"(a[0]), [v1] "v"(a[1]), [v2] "v"(a[2]), [v3] "v"(a[3]),
        [c0] "v"(b[0]), [c1] "v"(b[1]), [c2] "v"(b[2]), [c3] "v"(b[3])
      : "memory", "scc");
}

// if (cnt < k) hi = t; else lo = t;   (all operands wave-uniform)
__device__ __forceinline__ void move_bound(float& lo, float& hi, float t, int cnt, int k) {
  const bool less = cnt < k;
  hi = less ? t : hi;
  lo = less ? lo : t;
}

// ---- one row ----------------------------------------------------------------------------------------

// cnt = #{e, lane : x[e] >= t}.  The compare writes a 64-lane mask to scalar registers; the count is
// a scalar popcount, so no cross-lane reduction is needed.  m[e] keeps the masks.
template <int E, bool NEG>
__device__ __forceinline__ int count_ge(const float (&x)[E], float t, uint64_t (&m)[E]) {
  int cnt = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    m[e] = __builtin_amdgcn_ballot_w64(keyof<NEG>(x[e]) >= t);
    cnt += __builtin_popcountll(m[e]);
  }
  return cnt;
}

// Sum of a per-lane integer over the wavefront (result wave-uniform).
__device__ __forceinline__ int wave_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false);  // row_half_mirror
  v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, false);  // row_mirror
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
  return __builtin_amdgcn_readlane(v, 63);
}

// The same count for wide rows, without keeping masks.  Two ways to count, per element:
//   by mask popcount: one compare that writes the 64-lane mask to scalar registers, then a scalar popcount
//     and add.  Measured issue cost on MI355X (all wavefronts of a SIMD busy): ~4.4 cycles of the vector
//     unit per compare (a vector instruction that writes a lane mask runs at about half rate) plus two
//     scalar instructions at ~4.8 cycles each per SIMD (the compute unit's scalar unit serves its four SIMDs
//     in turn) -- the scalar side is the limit.
//   per lane: d = key - t (one full-rate subtraction, ~2.5 cycles), whose sign bit says key < t, and one
//     v_alignbit that shifts that bit into a per-lane bit pack (~2.5 cycles); every 32 elements one
//     v_bcnt adds the pack's population to a per-lane counter, and the counters are summed over the
//     wavefront once per step.  ~5 cycles per element and no scalar work, against ~8.4 for a compare plus
//     an add-with-carry (both of which go through VCC and run at half rate).
// ACC of the E elements are counted per lane, the rest by popcount.  Below 32 elements per lane the fixed
// cost of the bit-pack form (the zero test, the final subtraction) outweighs its gain and a compare plus
// add-with-carry per element is kept (M = 1024: 232 us against 243 us per 2^18 rows); from 32 on the
// bit pack wins (M = 8192: 222 -> 213 us exact, 218 -> 203 us at eight steps; one workgroup per row,
// M = 32768: 337 -> 317 us and 279 -> 252 us).
//
// The sign test is exact: with denormals kept, key - t is zero only when key == t, and rounding never
// changes its sign otherwise.  Zero needs care: (-0) - (+0) = -0 would count a key of -0 as below a
// threshold of +0, so a zero threshold is taken as -0 (then key - t = key + 0, which is +0 for either zero).
template <int E, int ACC, bool NEG>
__device__ __forceinline__ int count_ge_wide(const float (&x)[E], float t) {
  int cnt = 0;
#pragma unroll
  for (int e = ACC; e < E; ++e) cnt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(keyof<NEG>(x[e]) >= t));
  if constexpr (ACC >= 32) {
    const float tz = (t == 0.0f) ? -0.0f : t;
    uint32_t below = 0, pack = 0;
#pragma unroll
    for (int e = 0; e < ACC; ++e) {
      const float d = keyof<NEG>(x[e]) - tz;
      pack = __builtin_amdgcn_alignbit(pack, __float_as_uint(d), 31);  // (pack << 1) | sign(d)
      if ((e & 31) == 31 || e + 1 == ACC) {
        below += (uint32_t)__builtin_popcount(pack);
        pack = 0;
      }
    }
    cnt += ACC * kWave - wave_sum((int)below);
  } else if constexpr (ACC > 0) {
    int acc = 0;
#pragma unroll
    for (int e = 0; e < ACC; ++e) acc += (keyof<NEG>(x[e]) >= t) ? 1 : 0;
    cnt += wave_sum(acc);
  }
  return cnt;
}

// Selecting stage, one level: the candidates are the set bits of m[] (element e of lane l is bit l
// of m[e]); the first `limit` of them in column order (g, lane, c) are written as (value, column)
// pairs to stage[0 ..).  CUT = false promises that there are at most `limit` candidates.
// LAZY: the masks are not passed in but formed here, group by group, as x >= t, where t is `t_hi`
// for columns above `split_col` and `t_lo` for columns up to it (a plain threshold has t_lo == t_hi).
template <int G, int NG, bool CUT, bool LAZY, bool NEG>
__device__ __forceinline__ void compact_masks(const float (&x)[G * NG], const uint64_t* mm, float t_hi, float t_lo,
                                              int split_col, int lane, int limit, uint32_t stage_addr) {
  uint32_t base = 0;  // wave-uniform: candidates in earlier groups
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    // An opaque copy of the lane id per group: otherwise the column numbers of all groups, shared by
    // every call site, are computed up front and stay live through the whole search.
    int ln = lane;
    if constexpr (NG > 4) asm volatile("" : "+v"(ln));
    if constexpr (CUT && NG > 1) {
      if (base >= (uint32_t)limit) break;  // the first `limit` candidates are all in earlier groups
    }
    uint64_t m[G];
#pragma unroll
    for (int c = 0; c < G; ++c) {
      if constexpr (LAZY) {
        const int col = (g * kWave + ln) * G + c;
        m[c] = __builtin_amdgcn_ballot_w64(keyof<NEG>(x[g * G + c]) >= (col <= split_col ? t_lo : t_hi));
      } else {
        m[c] = mm[g * G + c];
      }
    }
    uint32_t pos = base;
#pragma unroll
    for (int c = 0; c < G; ++c) pos = lanes_below(m[c], pos);
    if constexpr (G % 4 == 0) {
      // four elements at a time: one EXEC restore per four staged pairs
#pragma unroll
      for (int h = 0; h < G / 4; ++h) {
        uint64_t mk[4];
        uint32_t addr[4], col[4];
        float val[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int cc = h * 4 + c;
          mk[c] = m[cc];
          if constexpr (CUT) mk[c] &= __builtin_amdgcn_ballot_w64(pos < (uint32_t)limit);
          addr[c] = stage_addr + pos * 8u;
          val[c] = x[g * G + cc];
          col[c] = (uint32_t)((g * kWave + ln) * G + cc);
          if (cc + 1 < G) pos = add_mask_bit(pos, m[cc]);
        }
        lds_store_pairs_masked4(mk, addr, val, col);
      }
    } else {
#pragma unroll
      for (int c = 0; c < G; ++c) {
        uint64_t mk = m[c];
        if constexpr (CUT) mk &= __builtin_amdgcn_ballot_w64(pos < (uint32_t)limit);
        lds_store_pair_masked(mk, stage_addr + pos * 8u, __float_as_uint(x[g * G + c]),
                              (uint32_t)((g * kWave + ln) * G + c));
        if (c + 1 < G) pos = add_mask_bit(pos, m[c]);
      }
    }
    if (g + 1 < NG) {
#pragma unroll
      for (int c = 0; c < G; ++c) base += (uint32_t)__builtin_popcountll(m[c]);
    }
    // keep the groups in program order: hoisting every group's compares would hold all masks live
    if constexpr (NG > 4) __builtin_amdgcn_sched_barrier(0);
  }
}

// Column of the `want`-th (1-based) element, in column order, among those with tb <= x < ta;
// -1 when want == 0.  Used only after the exact search has converged without cnt == k.
template <int G, int NG, bool NEG>
__device__ __forceinline__ int nth_column_in_band(const float (&x)[G * NG], int lane, float ta, float tb, int want) {
  uint32_t base = 0;  // wave-uniform: band members in earlier groups
  int mine = -1;      // per lane: the wanted column if this lane owns it
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    int ln = lane;  // opaque per group, see compact_masks
    if constexpr (NG > 4) asm volatile("" : "+v"(ln));
    uint32_t pos = base;
    bool b[G];
#pragma unroll
    for (int c = 0; c < G; ++c) {
      const float v = keyof<NEG>(x[g * G + c]);
      b[c] = (v >= tb) && !(v >= ta);
      const uint64_t mb = __builtin_amdgcn_ballot_w64(b[c]);
      pos = lanes_below(mb, pos);
      base += (uint32_t)__builtin_popcountll(mb);
    }
#pragma unroll
    for (int c = 0; c < G; ++c) {
      if (b[c] && pos + 1u == (uint32_t)want) mine = (g * kWave + ln) * G + c;
      pos += b[c] ? 1u : 0u;
    }
    if constexpr (NG > 4) __builtin_amdgcn_sched_barrier(0);
  }
  // exactly one lane (or none) holds a column >= 0: a wavefront maximum returns it
  int v = mine;
  v = max(v, __builtin_amdgcn_update_dpp(-1, v, 0xB1, 0xf, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(-1, v, 0x4E, 0xf, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(-1, v, 0x141, 0xf, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(-1, v, 0x140, 0xf, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(-1, v, 0x142, 0xa, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(-1, v, 0x143, 0xc, 0xf, false));
  return __builtin_amdgcn_readlane(v, 63);
}

// x where bit `lane` of mask is set, +0 elsewhere: one v_cndmask with the lane mask as its condition.
__device__ __forceinline__ float keep_where(float x, uint64_t mask) {
  float r;
  asm("v_cndmask_b32_e64 %0, 0, %1, %2" : "=v"(r) : "v"(x), "s"(mask));
  return r;
}

// Selecting stage in dense form (the MaxK non-linearity as MaxK-GNN applies it before aggregation,
// Section 1 / Fig. 1): y[e] = x[e] for the chosen elements and +0 for all others, in the row's own
// register layout, so that the result goes back to memory with the same coalesced accesses the row
// came in with.  Same candidates, order and cut as compact_masks.
template <int G, int NG, bool CUT, bool LAZY, bool NEG>
__device__ __forceinline__ void mask_dense(const float (&x)[G * NG], const uint64_t* mm, float t_hi, float t_lo,
                                           int split_col, int lane, int limit, float (&y)[G * NG]) {
  uint32_t base = 0;  // wave-uniform: candidates in earlier groups
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    int ln = lane;  // opaque per group, see compact_masks
    if constexpr (NG > 4) asm volatile("" : "+v"(ln));
    uint64_t m[G];
#pragma unroll
    for (int c = 0; c < G; ++c) {
      if constexpr (LAZY) {
        const int col = (g * kWave + ln) * G + c;
        m[c] = __builtin_amdgcn_ballot_w64(keyof<NEG>(x[g * G + c]) >= (col <= split_col ? t_lo : t_hi));
      } else {
        m[c] = mm[g * G + c];
      }
    }
    if constexpr (CUT) {
      uint32_t pos = base;
#pragma unroll
      for (int c = 0; c < G; ++c) pos = lanes_below(m[c], pos);
#pragma unroll
      for (int c = 0; c < G; ++c) {
        y[g * G + c] = keep_where(x[g * G + c], m[c] & __builtin_amdgcn_ballot_w64(pos < (uint32_t)limit));
        if (c + 1 < G) pos = add_mask_bit(pos, m[c]);
      }
      if (g + 1 < NG) {
#pragma unroll
        for (int c = 0; c < G; ++c) base += (uint32_t)__builtin_popcountll(m[c]);
      }
    } else {
#pragma unroll
      for (int c = 0; c < G; ++c) y[g * G + c] = keep_where(x[g * G + c], m[c]);
    }
    if constexpr (NG > 4) __builtin_amdgcn_sched_barrier(0);
  }
}

// The selection in the form the kernel wants: (value, column) pairs staged in LDS, or the dense row.
template <int G, int NG, bool CUT, bool LAZY, bool NEG, bool DENSE>
__device__ __forceinline__ void emit_selection(const float (&x)[G * NG], const uint64_t* mm, float t_hi, float t_lo,
                                               int split_col, int lane, int limit, uint32_t stage_addr,
                                               float (&y)[G * NG]) {
  if constexpr (DENSE) {
    mask_dense<G, NG, CUT, LAZY, NEG>(x, mm, t_hi, t_lo, split_col, lane, limit, y);
  } else {
    compact_masks<G, NG, CUT, LAZY, NEG>(x, mm, t_hi, t_lo, split_col, lane, limit, stage_addr);
  }
}

// Hand-scheduled search loops for 2, 4 and 8 values per lane: search_exact_asm / search_early_asm
// (generated by gen_search_loops.py; same steps as the generic loops in select_row).
#include "rtopk_search_loops.inc"

// Per-lane part of the row minimum and maximum: mx = max of the lane's elements, nm = max of their
// negations.  (Lanes past M hold copies of the row's first columns here, which changes neither.)
template <int E>
__device__ __forceinline__ void lane_max_and_negmin(const float (&xin)[E], float& mx, float& nm) {
  if constexpr (E == 1) {
    mx = xin[0];
    nm = -xin[0];
  } else if constexpr (E == 2) {
    mx = vmax(xin[0], xin[1]);
    nm = vmax_nn(xin[0], xin[1]);
  } else {
    mx = vmax3(xin[0], xin[1], xin[2]);
    nm = vmax3_nnn(xin[0], xin[1], xin[2]);
    int e = 3;
#pragma unroll
    for (; e + 1 < E; e += 2) {
      mx = vmax3(mx, xin[e], xin[e + 1]);
      nm = vmax3_ann(nm, xin[e], xin[e + 1]);
    }
    if (e < E) {
      mx = vmax(mx, xin[e]);
      nm = vmax_an(nm, xin[e]);
    }
  }
}

// Maximum and minimum of each of the R rows a wavefront holds (wave-uniform results).  Two or more rows
// are reduced together (wave_max_and_negmin_rows: about 4 vector instructions per row instead of 9).
template <int R, int E>
__device__ __forceinline__ void rows_max_and_min(const float (&x)[R][E], float (&hi)[R], float (&lo)[R]) {
  if constexpr (R == 1) {
    float mx, nm;
    lane_max_and_negmin<E>(x[0], mx, nm);
    wave_max_and_negmin(mx, nm, hi[0], lo[0]);
  } else if constexpr (R <= 8) {
    float mx[R], nm[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) lane_max_and_negmin<E>(x[rr], mx[rr], nm[rr]);
    wave_max_and_negmin_rows(mx, nm, hi, lo);
  } else {
    // eight rows at a time: the same instruction count as one wider reduction, half the registers
    static_assert(R % 8 == 0, "rows per wavefront: 1, 2, 4, 8 or a multiple of 8");
#pragma unroll
    for (int b = 0; b < R; b += 8) {
      float mx[8], nm[8], h[8], l[8];
#pragma unroll
      for (int rr = 0; rr < 8; ++rr) lane_max_and_negmin<E>(x[b + rr], mx[rr], nm[rr]);
      wave_max_and_negmin_rows(mx, nm, h, l);
#pragma unroll
      for (int rr = 0; rr < 8; ++rr) {
        hi[b + rr] = h[rr];
        lo[b + rr] = l[rr];
      }
    }
  }
}

// Exact mode on rows stored in 16 bits: the midpoint with the fp32 bits below the row type's precision
// cleared (see gen_search_loops.py for why this ends the search early and is still exact).
template <int DT>
__device__ __forceinline__ float midpoint_exact(float lo, float hi) {
  const float t = (lo + hi) * 0.5f;
  if constexpr (DT == kF32) {
    return t;
  } else {
    return __uint_as_float(__float_as_uint(t) & (DT == kBF16 ? 0xffff0000u : 0xffffe000u));
  }
}

// In the lanes whose bit is set in `mask` (a subset of the active lanes): LDS[addr] = v.
__device__ __forceinline__ void lds_store_masked(uint64_t mask, uint32_t addr, float v) {
  uint64_t saved;
  asm volatile(
      "s_and_saveexec_b64 %0, %1\n\t"
      "ds_write_b32 %2, %3\n\t"
      "s_mov_b64 exec, %0"
      : "=&s"(saved)
      : "s"(mask), "v"(addr), "v"(v)
      : "memory", "scc");
}

// Narrowing of a wide row's search.  A threshold between lo and hi separates only the elements whose
// key lies in [lo, hi); everything at or above hi is counted by every later threshold and everything
// below lo by none.  On the rows this method is meant for that band empties fast -- the bisection is
// over the value range, and after three to five steps it holds a few hundred of thousands of elements
// (median 161 of 4096 after three steps and 68 after four on Laplace rows, 277 of 8192 after four on
// normal ones) -- so once at most 256 (or 512) elements are left they are gathered, in any order, into
// four (or eight) registers per lane and the remaining steps compare those instead of the whole row:
//   #{key >= t} = #{key >= hi} + #{band members with key >= t}    for every lo <= t < hi.
// Thresholds, counts and therefore the result are exactly those of the full-width search.
constexpr int kBandRegs = 4;
// Registers per lane the band is gathered into, by row width: eight for rows of 128 values per lane
// (M = 8192: 4 % faster than four, one full-width step fewer), four otherwise (M = 4096: 4 % faster
// than eight; the workgroup-per-row kernel likewise).
constexpr int band_regs(int E) { return E >= 128 ? 8 : kBandRegs; }
// Which kernels narrow: those for rows of 24 or more values per lane, which are the widths that go one
// row to a wavefront, so that the row's staging area is still unused while it is searched.
constexpr bool narrows(int E, int /*mode*/) { return E >= 24; }

// The sign bits of key - t for this lane's E keys, 32 to a word: element e is bit (filled - 1 - e % 32) of
// word e / 32 (filled = elements in that word; the bits above them stay zero), set when key < t.  Two
// full-rate vector instructions per element and no scalar work (see count_ge_wide).
template <int E, bool NEG>
__device__ __forceinline__ void lane_below_packs(const float (&x)[E], float t, uint32_t (&p)[(E + 31) / 32]) {
  const float tz = (t == 0.0f) ? -0.0f : t;
  uint32_t pack = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const float d = keyof<NEG>(x[e]) - tz;
    pack = __builtin_amdgcn_alignbit(pack, __float_as_uint(d), 31);  // (pack << 1) | sign(d)
    if ((e & 31) == 31 || e + 1 == E) {
      p[e / 32] = pack;
      pack = 0;
    }
  }
}

// All ones in the bits of word `word` that lane_below_packs fills.
template <int E>
constexpr uint32_t pack_valid(int word) {
  return (word == (E + 31) / 32 - 1 && E % 32 != 0) ? ((1u << (E % 32)) - 1u) : 0xffffffffu;
}

// Inclusive prefix sum over the 64 lanes with six DPP steps (a lane without a source keeps 0 added).
__device__ __forceinline__ uint32_t wave_inclusive_scan_dpp(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);  // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);  // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);  // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);  // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
  return v;
}

typedef __attribute__((address_space(3))) float lds_float;

// (a & mask) | (b & ~mask) in one instruction.
__device__ __forceinline__ uint32_t select_bits(uint32_t mask, uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "v"(mask), "v"(a), "v"(b));
  return r;
}

constexpr uint32_t kNoRoom = 0xffffffffu;

// The wavefront's members of the band lo <= key < hi go to consecutive 4-byte slots of LDS, in any order.
// below_lo and below_hi are the lane's sign-bit words against the two bounds (lane_below_packs); the
// search has them already, from the steps that set the bounds.  The lanes' member counts are scanned,
// `reserve(n, above)` returns the byte address of n free slots, or kNoRoom (and is told how many keys are
// at or above hi); then each lane walks its elements once and stores every one of them -- members to the
// lane's next slot, the others to a per-lane dummy word at `dummy` -- so that no lane mask or branch is
// needed.
template <int E, bool NEG, typename Reserve>
__device__ __forceinline__ void scatter_band_members(const float (&x)[E], const uint32_t (&below_lo)[(E + 31) / 32],
                                                     const uint32_t (&below_hi)[(E + 31) / 32], int lane,
                                                     uint32_t dummy, Reserve reserve) {
  constexpr int GROUPS = (E + 31) / 32;
  uint32_t member[GROUPS];
  uint32_t n_lane = 0, above_lane = 0;
#pragma unroll
  for (int g = 0; g < GROUPS; ++g) {
    member[g] = ~below_lo[g] & below_hi[g];
    n_lane += (uint32_t)__builtin_popcount(member[g]);
    above_lane += (uint32_t)__builtin_popcount(~below_hi[g] & pack_valid<E>(g));
  }
  const uint32_t incl = wave_inclusive_scan_dpp(n_lane);
  const uint32_t n_wave = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
  const uint32_t above = (uint32_t)wave_sum((int)above_lane);
  const uint32_t base = reserve(n_wave, above);  // wave-uniform LDS byte address, or kNoRoom
  if (base == kNoRoom) {
    // cannot happen on finite input (the caller has bounded the band by its counts); with NaN or
    // infinite keys the sign bits need not agree with those counts, and then nothing is stored
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) member[g] = 0;
  }
  // the lane's slots are filled from its last one downwards
  uint32_t addr = base + (incl - 1u) * 4u;
  const uint32_t trash = dummy + (uint32_t)lane * 4u;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int filled = (e / 32 == GROUPS - 1 && E % 32 != 0) ? E % 32 : 32;
    const int bit = filled - 1 - (e & 31);
    // three vector instructions per element, written out because the compiler otherwise rebuilds the
    // select from a compare and a conditional move and the address from a running count (seven)
    const uint32_t m = (uint32_t)__builtin_amdgcn_sbfe(member[e / 32], (uint32_t)bit, 1u);  // all ones for a member
    *reinterpret_cast<lds_float*>(select_bits(m, addr, trash)) = x[e];
    asm("v_lshl_add_u32 %0, %1, 2, %0" : "+v"(addr) : "v"(m));  // one slot down after a member
  }
}

// y[j] = the (lane + 64 j)-th of the nb floats at LDS address `scratch`, or a key of -inf beyond them.
// The LDS queue of a wavefront is served in order, so the reads see the wavefront's earlier writes; the
// wait is written out because the compiler does not track LDS operations inside asm blocks.
template <bool NEG, int BR>
__device__ __forceinline__ void load_band(uint32_t scratch, int lane, uint32_t nb, float (&y)[BR]) {
  static_assert(BR == 4 || BR == 8, "four or eight values per lane");
  const float none = NEG ? __builtin_inff() : -__builtin_inff();
  float v[8];
  asm volatile(
      "ds_read_b32 %0, %4\n\t"
      "ds_read_b32 %1, %4 offset:256\n\t"
      "ds_read_b32 %2, %4 offset:512\n\t"
      "ds_read_b32 %3, %4 offset:768\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
      : "v"(scratch + (uint32_t)lane * 4u)
      : "memory");
  if constexpr (BR == 8) {
    asm volatile(
        "ds_read_b32 %0, %4 offset:1024\n\t"
        "ds_read_b32 %1, %4 offset:1280\n\t"
        "ds_read_b32 %2, %4 offset:1536\n\t"
        "ds_read_b32 %3, %4 offset:1792\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
        : "v"(scratch + (uint32_t)lane * 4u)
        : "memory");
  }
#pragma unroll
  for (int j = 0; j < BR; ++j) y[j] = (uint32_t)lane + 64u * j < nb ? v[j] : none;
}

// Gathers the row's band members through `scratch` (BR*64 floats of LDS) into y[]; lanes beyond
// the band hold a key of -inf.  Returns #{key >= hi}.  The caller guarantees the band fits.
// SPARSE: most of the lane masks are expected to be empty (a workgroup's band is spread over all its
// wavefronts), so each is tested before it is ranked and stored.
template <int E, bool NEG, bool SPARSE = false, int BR = kBandRegs>
__device__ __forceinline__ int gather_band(const float (&x)[E], float lo, float hi, int lane, uint32_t scratch,
                                           float (&y)[BR], uint32_t& nb) {
  int above = 0;
  nb = 0;  // wave-uniform: band members found so far
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const float key = keyof<NEG>(x[e]);
    const uint64_t a = __builtin_amdgcn_ballot_w64(key >= hi);
    const uint64_t b = __builtin_amdgcn_ballot_w64(key >= lo) & ~a;
    above += __builtin_popcountll(a);
    if (!SPARSE || b != 0) {
      lds_store_masked(b, scratch + lanes_below(b, nb) * 4u, x[e]);
      nb += (uint32_t)__builtin_popcountll(b);
    }
    if ((e & 3) == 3) __builtin_amdgcn_sched_barrier(0);  // keep the masks of later elements from piling up
  }
  load_band<NEG, BR>(scratch, lane, nb, y);
  return above;
}

// #{band members with key >= t}
template <bool NEG, int BR>
__device__ __forceinline__ int count_band(const float (&band)[BR], float t) {
  int cnt = 0;
#pragma unroll
  for (int j = 0; j < BR; ++j) cnt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(keyof<NEG>(band[j]) >= t));
  return cnt;
}

// The rest of Algorithm 1's loop on a gathered band (`above` = #{key >= hi} when it was gathered):
// exact mode until a step counts k or the midpoint is no longer strictly inside (lo, hi) -- the state
// the full-width loop detects, one or two steps later, by its midpoint repeating -- and the
// precision-bounded mode with its own guard and step count.
template <int MODE, bool NEG, int DT, int BR>
__device__ __forceinline__ void search_band(const float (&band)[BR], int above, int k, float eps, float& lo,
                                            float& hi, float& thres, bool& hit, int& steps) {
  for (;;) {
    if constexpr (MODE == kEps) {
      if (!(hi - lo > eps)) break;
    }
    const float mid = MODE == kEps ? (lo + hi) * 0.5f : midpoint_exact<DT>(lo, hi);
    if (!(mid > lo && mid < hi)) break;
    thres = mid;
    ++steps;
    const int cnt = above + count_band<NEG, BR>(band, thres);
    if (cnt == k) {
      hit = true;
      break;
    }
    move_bound(lo, hi, thres, cnt, k);
  }
}

// How many of a wide row's E values per lane are counted per lane (reduced over the wavefront once per
// step) rather than by mask popcount on the scalar unit (see count_ge_wide).  From sweeps on MI355X:
// a third up to 48 values per lane, two thirds at 64, all of them from 96 on -- the scalar unit is shared
// by the four SIMDs of a compute unit and is the first to saturate, and the more registers a wavefront
// holds the fewer wavefronts share a SIMD to hide the compare -> scalar popcount latency
// (M = 8192: 361 -> 276 us per 32768 rows, M = 6144: 284 -> 239 us, M = 4096: 214 -> 205 us).
#ifndef RTOPK_ACC_OF
#define RTOPK_ACC_OF(E) ((E) >= 96 ? (E) : ((E) >= 64 ? (2 * (E)) / 3 : ((E) - 3) / 3))
#endif
// Rows whose every element is counted per lane gather their band from the sign-bit words of the search
// (see select_row); the scatter needs one dummy word per lane behind the band's slots.
constexpr bool scatter_gathers(int E) { return E > 8 && narrows(E, 0) && RTOPK_ACC_OF(E) == (E); }
// Floats of LDS scratch per wavefront that the narrowing of a row of E values per lane uses (0: none).
constexpr int band_scratch_floats(int E) {
  return narrows(E, 0) ? band_regs(E) * kWave + (scatter_gathers(E) ? kWave : 0) : 0;
}

// Search and selection for one row held as xin[E] (lanes past column M hold duplicates of real
// elements on entry).
//   MODE: kExact = Algorithm 1 at epsilon = 0, kEarly = Algorithm 2 with max_iter steps,
//         kEps = Algorithm 1 with epsilon = eps_rel * |max|.
// Returns the exit iteration of the search loop (kEps only; 0 otherwise): the number of midpoints
// evaluated when one of them counted exactly k, one more when the loop ended through its guard.
//   DENSE: the result is y[] (chosen values in place, +0 elsewhere) instead of pairs staged at `stage`.
//   row_max, row_min: the row's maximum and minimum (Alg. 1 / Alg. 2, first two steps), wave-uniform.
template <int G, int NG, bool FULL, int MODE, bool NEG, int DT = kF32, bool DENSE = false>
__device__ __forceinline__ int select_row(const float (&xin)[G * NG], int lane, int M, int k, int max_iter,
                                          float eps_rel, uint2* stage, float (&y)[G * NG], float row_max,
                                          float row_min) {
  constexpr int E = G * NG;
  const uint32_t stage_addr = (uint32_t)(uintptr_t)stage;  // LDS byte address

  // lo, hi bound the keys: for the smallest-k variant the keys are the negated values, whose maximum
  // is the negated row minimum and vice versa, so the two reduction results just swap roles.
  float lo = NEG ? -row_max : row_min;
  float hi = NEG ? -row_min : row_max;

  // From here on columns past M must never be counted or chosen: a key of -inf is below every threshold.
  float x[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const bool valid = FULL || ((e / G) * kWave + lane) * G < M;
    x[e] = valid ? xin[e] : (NEG ? __builtin_inff() : -__builtin_inff());  // key -inf
  }

  constexpr bool ASM = (E == 2 || E == 4 || E == 8);  // hand-scheduled loops exist for these widths
  constexpr bool KEEP = E <= 8;                       // masks of the last step stay in scalar registers
  // wider rows: ACC of the E elements are counted per lane, the rest by mask popcount
  constexpr int ACC = KEEP ? 0 : RTOPK_ACC_OF(E);
  constexpr int BR = band_regs(E);  // registers per lane of a gathered band (see gather_band)
  uint64_t m[KEEP ? E : 1];
  // Rows counted entirely per lane keep the sign-bit words of the steps that set lo and hi; the band is
  // then gathered from those words (scatter_band_members) instead of with two compares per element.
  constexpr bool PACKS = scatter_gathers(E);
  constexpr int PW = (E + 31) / 32;
  uint32_t last[PW], below_lo[PW], below_hi[PW];
  bool lo_moved = false, hi_moved = false;
  auto count = [&](float t) -> int {
    if constexpr (KEEP) {
      return count_ge<E, NEG>(x, t, m);
    } else if constexpr (PACKS) {
      lane_below_packs<E, NEG>(x, t, last);
      uint32_t below = 0;
#pragma unroll
      for (int g = 0; g < PW; ++g) below += (uint32_t)__builtin_popcount(last[g]);
      return E * kWave - wave_sum((int)below);
    } else {
      return count_ge_wide<E, ACC, NEG>(x, t);
    }
  };
  auto note_bound = [&](int cnt) {  // after move_bound with the latest count
    if constexpr (PACKS) {
      if (cnt < k) {  // uniform
        hi_moved = true;
#pragma unroll
        for (int g = 0; g < PW; ++g) below_hi[g] = last[g];
      } else {
        lo_moved = true;
#pragma unroll
        for (int g = 0; g < PW; ++g) below_lo[g] = last[g];
      }
    }
  };
  auto gather = [&](float (&band)[BR]) -> int {  // the band [lo, hi) into band[]; returns #{key >= hi}
    if constexpr (PACKS) {
      if (!lo_moved) lane_below_packs<E, NEG>(x, lo, below_lo);  // a bound still at the row's minimum or maximum
      if (!hi_moved) lane_below_packs<E, NEG>(x, hi, below_hi);
      int above = 0;
      uint32_t members = 0;
      scatter_band_members<E, NEG>(x, below_lo, below_hi, lane, stage_addr + (uint32_t)(BR * kWave) * 4u,
                                   [&](uint32_t n, uint32_t ab) -> uint32_t {
                                     above = (int)ab;
                                     members = n <= (uint32_t)(BR * kWave) ? n : 0u;
                                     return n <= (uint32_t)(BR * kWave) ? stage_addr : kNoRoom;
                                   });
      load_band<NEG, BR>(stage_addr, lane, members, band);
      return above;
    } else {
      uint32_t nb;
      return gather_band<E, NEG, false, BR>(x, lo, hi, lane, stage_addr, band, nb);
    }
  };
  if constexpr (MODE == kExact) {
    // The loop ends on cnt == k, or once the fp32 midpoint stops changing: then no representable
    // threshold lies strictly inside (lo, hi).  The latter is tested every second step against the
    // previous midpoint (a converged search repeats its midpoint for ever, a live one never returns to
    // an earlier midpoint); the extra steps leave lo and hi untouched.
    bool hit = false;
    float thres = lo;
    if constexpr (ASM) {
      hit = search_exact_asm(x, lo, hi, k, m, std::integral_constant<bool, NEG>(), std::integral_constant<int, DT>());
    } else {
      // cnt_lo = #{key >= lo} and a lower bound cnt_hi of #{key >= hi} bound the band [lo, hi) from
      // above; once it fits BR registers per lane the search narrows to it (see gather_band).
      constexpr bool NARROW = narrows(E, MODE);
      int cnt_lo = M, cnt_hi = 0;
      bool narrow = false;
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
        if constexpr (NARROW) {
          note_bound(cnt);
          cnt_lo = cnt < k ? cnt_lo : cnt;
          cnt_hi = cnt < k ? cnt : cnt_hi;
          if (cnt_lo - cnt_hi <= BR * kWave) {
            narrow = true;
            break;
          }
        }
        thres = midpoint_exact<DT>(lo, hi);
        cnt = count(thres);
        if (cnt == k) {
          hit = true;
          break;
        }
        move_bound(lo, hi, thres, cnt, k);
        if constexpr (NARROW) {
          note_bound(cnt);
          cnt_lo = cnt < k ? cnt_lo : cnt;
          cnt_hi = cnt < k ? cnt : cnt_hi;
          if (cnt_lo - cnt_hi <= BR * kWave) {
            narrow = true;
            break;
          }
        }
      }
      if constexpr (NARROW) {
        if (narrow) {
          float band[BR];
          const int above = gather(band);
          int unused_steps = 0;
          search_band<kExact, NEG, DT, BR>(band, above, k, 0.0f, lo, hi, thres, hit, unused_steps);
        }
      }
    }
    if (hit) {
      emit_selection<G, NG, false, !KEEP, NEG, DENSE>(x, m, thres, thres, -1, lane, k, stage_addr, y);
    } else {
      // Everything >= hi is taken first (cut at k by column when hi is still the row maximum and k
      // or more tie there); the first k - na members of [lo, hi) follow: all columns up to the
      // (k - na)-th member's column select against lo, the others against hi.
      const int na = count(hi);
      const int split = nth_column_in_band<G, NG, NEG>(x, lane, hi, lo, k - (na < k ? na : k));
      emit_selection<G, NG, true, true, NEG, DENSE>(x, nullptr, hi, lo, split, lane, k, stage_addr, y);
    }
    return 0;
  } else if constexpr (MODE == kEps) {
    // Algorithm 1 as printed, with epsilon = eps_rel * |max| and the same two readings as the exact
    // mode: the loop also ends when the midpoint is not strictly inside (lo, hi), and the selection
    // after a guard exit takes everything >= hi, then the first columns of [lo, hi).
    const float eps = eps_rel * __builtin_fabsf(hi);
    bool hit = false;
    float thres = lo;
    int steps = 0;
    // narrowing as in the exact mode: same thresholds and counts, hence the same exit iteration
    constexpr bool NARROW = narrows(E, MODE);
    int cnt_lo = M, cnt_hi = 0, above = 0;
    bool narrow = false;
    float band[BR];
    while (hi - lo > eps) {
      const float mid = (lo + hi) * 0.5f;
      if (!(mid > lo && mid < hi)) break;
      thres = mid;
      ++steps;
      int cnt;
      if (NARROW && narrow) {
        cnt = above + count_band<NEG, BR>(band, thres);
      } else {
        cnt = count(thres);
      }
      if (cnt == k) {
        hit = true;
        break;
      }
      move_bound(lo, hi, thres, cnt, k);
      if constexpr (NARROW) {
        if (!narrow) {
          note_bound(cnt);
          cnt_lo = cnt < k ? cnt_lo : cnt;
          cnt_hi = cnt < k ? cnt : cnt_hi;
          if (cnt_lo - cnt_hi <= BR * kWave) {
            above = gather(band);
            narrow = true;
          }
        }
      }
    }
    if (hit) {
      emit_selection<G, NG, false, !KEEP, NEG, DENSE>(x, m, thres, thres, -1, lane, k, stage_addr, y);
      return steps;
    }
    const int na = count(hi);
    const int split = nth_column_in_band<G, NG, NEG>(x, lane, hi, lo, k - (na < k ? na : k));
    emit_selection<G, NG, true, true, NEG, DENSE>(x, nullptr, hi, lo, split, lane, k, stage_addr, y);
    return steps + 1;
  } else {
    int cnt = -1;
    if constexpr (ASM) {
      cnt = search_early_asm(x, lo, hi, k, max_iter, m, std::integral_constant<bool, NEG>());
    } else {
      // narrowing as in Algorithm 1: every midpoint lies in [lo, hi], so the identity behind it holds
      constexpr bool NARROW = narrows(E, MODE);
      int cnt_lo = M, cnt_hi = 0, above = 0;
      bool narrow = false;
      float band[BR];
      for (int it = 0; it < max_iter; ++it) {
        const float thres = (lo + hi) * 0.5f;
        if (NARROW && narrow) {
          cnt = above + count_band<NEG, BR>(band, thres);
        } else {
          cnt = count(thres);
        }
        // cnt == k: from here on lo can only move to thresholds that still count exactly k, so the
        // selection is already final.
        move_bound(lo, hi, thres, cnt, k);
        if (cnt == k) break;
        if constexpr (NARROW) {
          if (!narrow) {
            note_bound(cnt);
            cnt_lo = cnt < k ? cnt_lo : cnt;
            cnt_hi = cnt < k ? cnt : cnt_hi;
            // the gather costs about as much as three full-width steps (one, from sign-bit words): only
            // when more remain
            if (cnt_lo - cnt_hi <= BR * kWave && it + (PACKS ? 2 : 6) < max_iter) {
              above = gather(band);
              narrow = true;
            }
          }
        }
      }
    }
    // The last step lowered hi (or none ran): the kept masks are not those of lo, so they are formed
    // again.  Wide rows keep no masks and rank against lo directly; only when the last step counted
    // exactly k can they skip the cut.
    if constexpr (KEEP) {
      if (cnt < k) cnt = count(lo);
    }
    if (cnt == k) {
      emit_selection<G, NG, false, !KEEP, NEG, DENSE>(x, m, lo, lo, -1, lane, k, stage_addr, y);
    } else {
      emit_selection<G, NG, true, !KEEP, NEG, DENSE>(x, m, lo, lo, -1, lane, k, stage_addr, y);
    }
    return 0;
  }
}

// ---- kernel -----------------------------------------------------------------------------------------

// Element types of the input matrix.  Rows stored in 16 bits are widened exactly to fp32 as they are
// loaded; the whole method (Section 3.1) then runs in fp32, as the paper defines it, and the values
// written out are narrowed back, which is exact because they are copies of inputs.
template <int DT>
__device__ __forceinline__ float widen_half(uint32_t w, int upper) {  // one of the two 16-bit halves of w
  if constexpr (DT == kBF16) {
    return __uint_as_float(upper ? (w & 0xffff0000u) : (w << 16));
  } else {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(upper ? (w >> 16) : (w & 0xffffu)));
  }
}
template <int DT>
__device__ __forceinline__ uint32_t narrow_bits(uint32_t fbits) {  // fp32 bits -> the 16-bit pattern it came from
  if constexpr (DT == kBF16) {
    return fbits >> 16;
  } else {
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)__uint_as_float(fbits));
  }
}

// One load of G consecutive elements starting at element `col` of the row at `row` (G*4 bytes for
// fp32, G*2 bytes for 16-bit types; the address is aligned to that size), with the non-temporal
// hint: every input byte is read exactly once, and keeping it out of the caches' retention policy
// measurably raises the streaming rate.
template <int DT, int G>
__device__ __forceinline__ void load_group(const typename std::conditional<DT == kF32, float, uint16_t>::type* row,
                                           int col, float (&dst)[G]) {
  typedef uint32_t u2 __attribute__((ext_vector_type(2)));
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  if constexpr (DT == kF32) {
    const float* p = row + col;
    if constexpr (G == 1) {
      dst[0] = __builtin_nontemporal_load(p);
    } else if constexpr (G == 2) {
      typedef float f2 __attribute__((ext_vector_type(2)));
      const f2 v = __builtin_nontemporal_load(reinterpret_cast<const f2*>(p));
      dst[0] = v.x;
      dst[1] = v.y;
    } else {
      static_assert(G == 4, "fp32 rows load 1, 2 or 4 values at a time");
      typedef float f4 __attribute__((ext_vector_type(4)));
      const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
      dst[0] = v.x;
      dst[1] = v.y;
      dst[2] = v.z;
      dst[3] = v.w;
    }
  } else {
    const uint16_t* p = row + col;
    if constexpr (G == 1) {
      dst[0] = widen_half<DT>((uint32_t)__builtin_nontemporal_load(p), 0);
    } else if constexpr (G == 2) {
      const uint32_t w = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
      dst[0] = widen_half<DT>(w, 0);
      dst[1] = widen_half<DT>(w, 1);
    } else if constexpr (G == 4) {
      const u2 w = __builtin_nontemporal_load(reinterpret_cast<const u2*>(p));
      dst[0] = widen_half<DT>(w.x, 0);
      dst[1] = widen_half<DT>(w.x, 1);
      dst[2] = widen_half<DT>(w.y, 0);
      dst[3] = widen_half<DT>(w.y, 1);
    } else {
      static_assert(G == 8, "16-bit rows load 1, 2, 4 or 8 values at a time");
      const u4 w = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
      dst[0] = widen_half<DT>(w.x, 0);
      dst[1] = widen_half<DT>(w.x, 1);
      dst[2] = widen_half<DT>(w.y, 0);
      dst[3] = widen_half<DT>(w.y, 1);
      dst[4] = widen_half<DT>(w.z, 0);
      dst[5] = widen_half<DT>(w.z, 1);
      dst[6] = widen_half<DT>(w.w, 0);
      dst[7] = widen_half<DT>(w.w, 1);
    }
  }
}

// Cache-policy bits of the output stores: non-temporal.  What decides is whether a launch's outputs were
// written before.  Timed over buffers that are rewritten in place launch after launch, and only while
// those outputs fit the 256 MB last-level cache, cached ("sc1", "sc0 sc1") stores look best (2^20 x 256,
// k = 32: 204 us against 216 us), because part of the write traffic is absorbed by that cache and never
// reaches HBM; rotating the launches over distinct output buffers -- what a caller inside a larger
// program sees -- takes that away (229 us), while non-temporal stores run the same either way (221 us).
// Over distinct buffers "nt" is the fastest or within 0.5 % of it on every workload measured (k = 16:
// 186 against 196 us; k = 64: 256 against 266 us; 2.4M x 256 with byte columns: 452 against 454 us; the
// dense form: 344 against 349 us); no policy bit at all is 1-6 % slower than either.
#ifndef RTOPK_STORE_POLICY
#define RTOPK_STORE_POLICY "nt"
#endif

// 128-bit, 64-bit and 32-bit output stores with that policy: the outputs are written once and never read
// back by this kernel.
__device__ __forceinline__ void store_streaming(uint4* p, uint4 v) {
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  const u4 d = {v.x, v.y, v.z, v.w};
  // A store of more than 64 bits reads its data registers late: a vector instruction that overwrites
  // them within the next two issue slots would corrupt the stored value.  The compiler pads its own
  // stores for this but cannot see inside an asm block, so the padding is written out here.
  asm volatile("global_store_dwordx4 %0, %1, off " RTOPK_STORE_POLICY "\n\ts_nop 1" : : "v"(p), "v"(d) : "memory");
}
__device__ __forceinline__ void store_streaming(uint2* p, uint2 v) {
  typedef uint32_t u2 __attribute__((ext_vector_type(2)));
  const u2 d = {v.x, v.y};
  asm volatile("global_store_dwordx2 %0, %1, off " RTOPK_STORE_POLICY : : "v"(p), "v"(d) : "memory");
}
__device__ __forceinline__ void store_streaming(uint32_t* p, uint32_t v) {
  asm volatile("global_store_dword %0, %1, off " RTOPK_STORE_POLICY : : "v"(p), "v"(v) : "memory");
}

// (Rows of 128 values per lane are held to three wavefronts per SIMD and rows of 96 to four: the ragged-width variants would
// otherwise take a few registers more than that allows and run two.)
template <int G, int NG, int R, bool FULL, int MODE, bool NEG, typename IdxT, int DT>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(G * NG >= 128 ? 3 : (G * NG >= 96 ? 4 : 1))))
    rtopk_wave_kernel(const void* __restrict__ in, int64_t N, int M, int k, int max_iter, float eps_rel,
                      void* __restrict__ out_vals, IdxT* __restrict__ out_idx, int32_t* __restrict__ out_iters,
                      int vec_store) {
  constexpr int E = G * NG;
  using ElemT = typename std::conditional<DT == kF32, float, uint16_t>::type;
  extern __shared__ uint2 stage_all[];  // [waves per block][R * k] (value bits, column)

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int waves_per_block = (int)(blockDim.x >> 6);
  const int64_t r0 = ((int64_t)blockIdx.x * waves_per_block + wave) * R;
  if (r0 >= N) return;
  const int nrows = (N - r0 < R) ? (int)(N - r0) : R;
  // per wavefront: R*k pairs, and at least the band scratch where the exact search of a wide row uses it
  static_assert(!narrows(E, MODE) || R == 1, "the band scratch reuses the staging area of the wavefront's only row");
  constexpr int kMinPairs = band_scratch_floats(E) / 2;
  const int pairs_per_wave = R * k > kMinPairs ? R * k : kMinPairs;
  uint2* stage = stage_all + (size_t)wave * pairs_per_wave;

  // Loading stage: all R rows' loads are issued before any is consumed.
  float x[R][E];
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    const ElemT* row = static_cast<const ElemT*>(in) + (r0 + (rr < nrows ? rr : 0)) * (int64_t)M;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      // Lanes whose columns lie past M load the row's first columns instead (in bounds, no branch, so
      // all loads of the wavefront stay in flight together).  Duplicates of real elements cannot
      // change the row's minimum or maximum; select_row turns them into -inf before it counts.
      const int col0 = (g * kWave + lane) * G;
      const bool valid = FULL || col0 < M;
      float v[G];
      load_group<DT, G>(row, valid ? col0 : 0, v);
#pragma unroll
      for (int c = 0; c < G; ++c) x[rr][g * G + c] = v[c];
    }
  }
  // Row minima and maxima of all R rows, then the searching and selecting stages row by row.
  float row_max[R], row_min[R];
  rows_max_and_min<R, E>(x, row_max, row_min);
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    if (rr < nrows) {
      float unused[E];
      const int it = select_row<G, NG, FULL, MODE, NEG, DT, false>(x[rr], lane, M, k, max_iter, eps_rel,
                                                                    stage + (size_t)rr * k, unused, row_max[rr],
                                                                    row_min[rr]);
      if constexpr (MODE == kEps) {
        if (out_iters != nullptr && lane == 0) out_iters[r0 + rr] = it;
      }
    }
  }

  // Dump: the wavefront's nrows*k staged pairs are contiguous in both output arrays.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const int total = nrows * k;
  using OutT = typename std::conditional<DT == kF32, uint32_t, uint16_t>::type;  // value bits as stored
  OutT* ov = static_cast<OutT*>(out_vals) + r0 * (int64_t)k;
  IdxT* oi = out_idx + r0 * (int64_t)k;
  if (vec_store) {
#pragma unroll 1
    for (int q = lane; q < (total >> 2); q += kWave) {
      const uint4 a = *reinterpret_cast<const uint4*>(stage + 4 * q);
      const uint4 b = *reinterpret_cast<const uint4*>(stage + 4 * q + 2);
      if constexpr (DT == kF32) {
        store_streaming(reinterpret_cast<uint4*>(ov) + q, make_uint4(a.x, a.z, b.x, b.z));
      } else {
        store_streaming(reinterpret_cast<uint2*>(ov) + q,
                        make_uint2(narrow_bits<DT>(a.x) | (narrow_bits<DT>(a.z) << 16),
                                   narrow_bits<DT>(b.x) | (narrow_bits<DT>(b.z) << 16)));
      }
      if constexpr (sizeof(IdxT) == 4) {
        store_streaming(reinterpret_cast<uint4*>(oi) + q, make_uint4(a.y, a.w, b.y, b.w));
      } else {
        store_streaming(reinterpret_cast<uint32_t*>(oi) + q, a.y | (a.w << 8) | (b.y << 16) | (b.w << 24));
      }
    }
  } else {
#pragma unroll 1
    for (int q = lane; q < total; q += kWave) {
      const uint2 a = stage[q];
      if constexpr (DT == kF32) {
        ov[q] = a.x;
      } else {
        ov[q] = (uint16_t)narrow_bits<DT>(a.x);
      }
      oi[q] = (IdxT)a.y;
    }
  }
}

// ---- dense-output kernel -------------------------------------------------------------------------------

// 128-bit / 64-bit / 32-bit store of G consecutive row elements.
template <int G>
__device__ __forceinline__ void store_group(float* p, const float* v) {
  if constexpr (G == 4) {
    store_streaming(reinterpret_cast<uint4*>(p),
                    make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])));
  } else if constexpr (G == 2) {
    store_streaming(reinterpret_cast<uint2*>(p), make_uint2(__float_as_uint(v[0]), __float_as_uint(v[1])));
  } else {
    store_streaming(reinterpret_cast<uint32_t*>(p), __float_as_uint(v[0]));
  }
}

// MaxK non-linearity, dense form: out[r][c] = in[r][c] where column c is among the k selected for
// row r (Algorithm 1 at epsilon = 0, or Algorithm 2), +0 elsewhere.  Same loading, min/max and
// search as rtopk_wave_kernel; the selection is a register-to-register mask, so nothing passes
// through LDS and each row leaves in the layout it arrived in.
template <int G, int NG, int R, bool FULL, int MODE>
__global__ void __launch_bounds__(256)
    rtopk_dense_kernel(const float* __restrict__ in, int64_t N, int M, int k, int max_iter, float* __restrict__ out) {
  constexpr int E = G * NG;
  extern __shared__ uint2 band_scratch[];  // [waves per block][band_regs(E) * 64 floats], wide rows only
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int waves_per_block = (int)(blockDim.x >> 6);
  const int64_t r0 = ((int64_t)blockIdx.x * waves_per_block + wave) * R;
  if (r0 >= N) return;
  const int nrows = (N - r0 < R) ? (int)(N - r0) : R;
  uint2* scratch = band_scratch + (size_t)wave * (band_scratch_floats(E) / 2);

  float x[R][E];
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    const float* row = in + (r0 + (rr < nrows ? rr : 0)) * (int64_t)M;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int col0 = (g * kWave + lane) * G;  // lanes past M: see rtopk_wave_kernel
      const bool valid = FULL || col0 < M;
      float v[G];
      load_group<kF32, G>(row, valid ? col0 : 0, v);
#pragma unroll
      for (int c = 0; c < G; ++c) x[rr][g * G + c] = v[c];
    }
  }
  float row_max[R], row_min[R];
  rows_max_and_min<R, E>(x, row_max, row_min);
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    if (rr < nrows) {
      float y[E];
      select_row<G, NG, FULL, MODE, false, kF32, true>(x[rr], lane, M, k, max_iter, 0.0f, scratch, y, row_max[rr],
                                                       row_min[rr]);
      float* orow = out + (r0 + rr) * (int64_t)M;
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int col0 = (g * kWave + lane) * G;
        if (FULL || col0 < M) store_group<G>(orow + col0, &y[g * G]);
      }
    }
  }
}

template <int G, int NG, int R, bool FULL, int MODE>
hipError_t launch_dense(const LaunchArgs& a) {
  const int waves = RTOPK_WAVES_PER_BLOCK;
  const int64_t batches = (a.N + R - 1) / R;
  const int64_t blocks = (batches + waves - 1) / waves;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  const size_t lds = (size_t)waves * band_scratch_floats(G * NG) * sizeof(float);
  return launch_kernel(rtopk_dense_kernel<G, NG, R, FULL, MODE>, dim3((unsigned)blocks), dim3(waves * kWave), lds,
                       a.stream, static_cast<const float*>(a.in), a.N, a.M, a.k, a.max_iter,
                       static_cast<float*>(a.out_vals));
}

// ---- host-side launcher -------------------------------------------------------------------------------

template <int G, int NG, int R, bool FULL, int MODE, typename IdxT, bool NEG = false, int DT = kF32>
hipError_t launch(const LaunchArgs& a) {
  // LDS per wavefront: R*k staged pairs of 8 bytes; at most 64 KiB per block.
  size_t per_wave = (size_t)R * (size_t)a.k * sizeof(uint2);
  // the exact search of wide rows gathers its band through the (not yet used) staging area
  if (per_wave < band_scratch_floats(G * NG) * sizeof(float)) per_wave = band_scratch_floats(G * NG) * sizeof(float);
  // one wavefront per workgroup, except where a wavefront stages 8 KiB or more of pairs: there four
  // per workgroup measured 7 % faster (2^20 x 256, k = 128: 387 -> 360 us), while at 4 KiB and below
  // one per workgroup is the faster by 3-11 %
  int waves = per_wave >= 8192 ? 4 : RTOPK_WAVES_PER_BLOCK;
  while (waves > 1 && per_wave * waves > 65536) waves >>= 1;
  const int64_t batches = (a.N + R - 1) / R;
  const int64_t blocks = (batches + waves - 1) / waves;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  return launch_kernel(rtopk_wave_kernel<G, NG, R, FULL, MODE, NEG, IdxT, DT>, dim3((unsigned)blocks),
                       dim3(waves * kWave), per_wave * waves, a.stream, a.in, a.N, a.M, a.k, a.max_iter, a.eps_rel,
                       a.out_vals, static_cast<IdxT*>(a.out_idx), a.out_iters, a.vec_store);
}

// Rows per wavefront for E = G*NG registers per row, from sweeps at 2^20 rows: 16 for M <= 128,
// 8 for M = 256, 2 for M = 512..1024 (M = 512 runs 10 % slower with 4), 1 beyond.
constexpr int rows_per_wave(int E) { return E <= 2 ? 16 : (E <= 4 ? 8 : (E <= 16 ? 2 : 1)); }
// fp32 rows of 129..256 columns with int32 columns (and their dense form) take 4 instead: with
// non-temporal output stores the smaller per-wavefront footprint streams better (2^20 x 256: k = 32
// 221 -> 215 us, k = 64 254 -> 247 us, k = 128 356 -> 345 us, dense 346 -> 339 us; with no search steps at
// all, 2 rows per wavefront reach 200 us but the search then costs 47 us more).  The variants that are
// bound by instruction issue rather than by memory keep 8, which amortises the per-wavefront work over
// more rows: rows stored in 16 bits (192 against 202 us) and byte-wide columns (2.4M rows: 475 against 483 us).
constexpr int kRowsPerWaveFp32M256 = 4;

// Few rows: with 8 or 16 rows per wavefront a launch of less than ~32768 rows does not even put two
// wavefronts on every SIMD, and each of them walks its rows one after the other.  Two rows per wavefront
// then spread the same work over more wavefronts (M = 256: 4096 rows 10.5 -> 6.6 us, 16384 rows
// 11.8 -> 9.4 us; no difference from 65536 rows on).
constexpr int64_t kFewRows = 32768;
constexpr int kRowsPerWaveFew = 2;

}  // namespace rtopk
