// Row-wise top-k for rows that no longer fit a workgroup's registers (65536 < M <= 2^24): one workgroup
// per row, the row streamed from memory -- once in the usual case.
//
// Same method and same results as the other kernels (RTop-K, arXiv 2409.00822, Section 3.1, Algorithms 1
// and 2).  Appendix B of the paper observes that for very wide rows a search that pays one pass over the
// row per bisection step loses to radix-style selection.  Two remedies here keep the paper's thresholds.
//
// First: the algorithms look at a count only to compare it with k.  The pass that finds the row's minimum
// and maximum (needed before the first threshold) therefore also keeps, in LDS, every key at or above a
// floor that it raises as it goes, chosen so that more than k keys stay at or above it.  Counts over those
// keys decide every step exactly as counts over the row would, so the whole search runs on them, and the
// k pairs are written from them: one pass over the row.
//
// Second, for rows whose kept keys do not fit (k in the thousands, or the winners crowded into one part
// of the row) or whose search stops so early that its last threshold lies below the floor: kLevels = 8
// bisection steps per pass instead of one.  All 255 midpoints that the next eight steps can possibly visit
// are fixed by (lo, hi) alone -- they form a binary tree, each node the fp32 midpoint of its interval
// exactly as the algorithms compute it -- so one pass sorts every element of the band [lo, hi) into the 256
// leaf intervals of that tree (an arithmetic guess corrected against a table in LDS, one LDS atomic), and
// the suffix sums of that histogram are the counts cnt(t) of all 255 thresholds at once.  The eight steps
// are then replayed on the counts, with the algorithms' own guards (cnt == k, the iteration limit,
// epsilon, the midpoint no longer strictly inside), bit for bit as the one-step-per-pass loop would have
// run them.  In effect: a radix-256 select over the value range whose digit boundaries are the paper's
// midpoints.  The last such pass again leaves the keys that can still be selected in LDS for the final
// write; only if those lists overflow as well is the row read once more to rank and write.
//
// Layout: wavefront w of 16 walks the w-th sixteenth of the row, lane l owning G consecutive columns of
// each 64*G-column load (G = 4: 128-bit loads), so that a wavefront meets its columns in ascending order.
// Loads are ordinary cached loads: the row is read again by the next pass.
//
// Nothing but registers and LDS is used; the library still allocates nothing.  One workgroup per row
// means that a launch of fewer rows than the GPU has compute units leaves the rest idle.
#pragma once

#include "rtopk_block_kernel.hpp"

namespace rtopk {

constexpr int kStreamWaves = 16;
constexpr int kStreamThreads = kStreamWaves * kWave;
constexpr int kLevels = 8;
constexpr int kLeaves = 1 << kLevels;
#ifndef RTOPK_STREAM_WAVES_PER_SIMD
#define RTOPK_STREAM_WAVES_PER_SIMD 8
#endif
#ifndef RTOPK_STREAM_AHEAD
#define RTOPK_STREAM_AHEAD 3
#endif
constexpr int kKeptPerWave = 256;  // at least one load of a wavefront (the first, which nothing filters yet)

template <int G>
__device__ __forceinline__ void stream_load(const float* p, float (&v)[G]) {
  if constexpr (G == 4) {
    const float4 q = *reinterpret_cast<const float4*>(p);
    v[0] = q.x;
    v[1] = q.y;
    v[2] = q.z;
    v[3] = q.w;
  } else {
    v[0] = *p;
  }
}

template <int G, int MODE, bool NEG>
__global__ void __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(RTOPK_STREAM_WAVES_PER_SIMD)))
    rtopk_stream_kernel(const float* __restrict__ in, int64_t N, int M, int k, int max_iter, float eps_rel,
                        float* __restrict__ out_vals, int32_t* __restrict__ out_idx, int32_t* __restrict__ out_iters) {
  __shared__ float s_tab[kLeaves];               // thresholds of the tree's nodes 1..255 (heap order; [0] unused)
  __shared__ float s_bnd[kLeaves + 1];           // the same thresholds in value order, with lo and hi at the ends
  __shared__ int s_hist[kStreamWaves][kLeaves];  // per-wavefront leaf histograms
  __shared__ int s_suffix[kLeaves + 1];          // suffix[j] = band members in leaves j..255
  __shared__ float s_hi[kStreamWaves], s_nlo[kStreamWaves];
  __shared__ int s_above[kStreamWaves];
  __shared__ __attribute__((aligned(16))) int s_parts[3][kLeaves];  // pass 0: kept keys per part of [floor, largest key seen)
  __shared__ float s_top[2][kStreamWaves];  // pass 0: per-wavefront largest key seen, exchanged by a raise for the next one
  __shared__ int s_void[kStreamWaves];    // per wavefront: its list of pass 0 ran full
  __shared__ int s_cnt[2][kStreamWaves];  // per-wavefront counts of a search step on the lists, double buffered
  __shared__ int s_pre[2][kStreamWaves];  // per-wavefront candidate counts of a chunk (A in the low half, B in the high), double buffered
  __shared__ uint2 s_kept[kStreamWaves][kKeptPerWave];  // per wavefront, in column order: (value bits, column) of the keys at or above the floor of pass 0, later at or above bstar of a search pass

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t r = blockIdx.x;
  if (r >= N) return;
  const float* row = in + r * (int64_t)M;
  constexpr int kChunk = kStreamThreads * G;

  // Suffix sums over the 256 leaves: thread j < 256 passes the population h of leaf j and gets the sum over
  // leaves j..255 (a DPP prefix scan per wavefront, the four wavefront totals through LDS).  Called by
  // every thread of the workgroup (it contains a barrier); threads 256.. pass 0 and ignore the result.
  auto suffix_of = [&](int h) -> int {
    const uint32_t incl = wave_inclusive_scan_dpp((uint32_t)h);
    if (lane == kWave - 1 && wave < kLeaves / kWave) s_pre[1][wave] = (int)incl;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kLeaves / kWave; ++w) {
      const uint32_t t = (uint32_t)s_pre[1][w];
      before += w < wave ? t : 0u;
      total += t;
    }
    return (int)(total - (before + incl) + (uint32_t)h);
  };

  constexpr int kUnit = kWave * G;  // columns a wavefront covers per load
  const int units = (M + kUnit - 1) / kUnit;
  const int u0 = (int)((int64_t)units * wave / kStreamWaves), u1 = (int)((int64_t)units * (wave + 1) / kStreamWaves);
  const int trips = (units + kStreamWaves - 1) / kStreamWaves;  // no wavefront has more loads than this
  // A wavefront keeps kAhead loads in flight in a ring of registers: a slot is worked on, then loaded again
  // with the wavefront's load kAhead further on (with one load at a time a pass is bound by memory latency).
  constexpr int kAhead = RTOPK_STREAM_AHEAD;
  auto load_slot = [&](int i, float (&slot)[G]) {  // the wavefront's i-th load
    // (no branch: past the wavefront's share or the row's end the row's first columns are loaded and not
    // looked at; a conditional load would make the compiler wait for all loads in flight at every use)
    const int u = u0 + i;
    const int c0 = u * kUnit + lane * G;
    stream_load<G>(row + ((u < u1 && c0 < M) ? c0 : 0), slot);
  };
  // The same with the non-temporal hint, for pass 0: as a rule the row is not read again, and streaming
  // loads that do not displace each other's lines from the caches run faster (see rtopk_kernel.hpp).
  auto load_slot_once = [&](int i, float (&slot)[G]) {
    const int u = u0 + i;
    const int c0 = u * kUnit + lane * G;
    load_group<kF32, G>(row, (u < u1 && c0 < M) ? c0 : 0, slot);
  };
  uint2* kept = &s_kept[wave][0];
  if (tid < 2 * kLeaves) s_parts[tid >> kLevels][tid & (kLeaves - 1)] = 0;  // the third is cleared by the first raise
  __syncthreads();

  // ---- pass 0: row minimum and maximum, and the keys that can still be among the k winners -------------
  // The algorithms need the row's minimum and maximum before their first threshold, which costs a pass.
  // That pass already does most of the selecting: it keeps, per wavefront and in column order, every key at
  // or above a floor T0 that rises as the pass goes on -- after 1, 2, 4, 8, ... loads per wavefront the kept
  // keys of the whole workgroup are counted into 256 equal parts of [T0, largest key seen), and the lower
  // end of the highest part with more than k (and a margin) kept keys at or above it becomes the new T0,
  // whereupon every wavefront drops what fell below.  More than k keys of the row are then at
  // or above T0, so #{key >= t} > k for every t <= T0 and the lists give that count exactly for every t > T0:
  // the whole search can run on the lists (a count over them is > k exactly when the true count is, equals k
  // exactly when the true count does, and is the true count whenever it is below k), and the k pairs can
  // be written from them, provided the lowest threshold of the selection ends at or above T0.  Only if a
  // list overflows, or that last condition fails, are the search passes below needed.
  float lo, hi;
  float T0 = -__builtin_inff();
  uint32_t n0 = 0;         // entries of this wavefront's list
  bool void0 = false;      // the list ran full: no selection from lists for this row
  {
    float mx = -__builtin_inff(), nm = -__builtin_inff();
    auto take = [&](const float (&v)[G], int u) {  // one load of the wavefront, already in registers
      // No branch before the one that skips the list: every branch between a load's issue and its use
      // makes the compiler wait for all loads in flight instead of this one.
      const int c0 = u * kUnit + lane * G;
      const bool valid = u < u1 && c0 < M;
      bool keep[G], any_keep = false;
#pragma unroll
      for (int c = 0; c < G; ++c) {
        mx = vmax(mx, valid ? v[c] : -__builtin_inff());
        nm = vmax_an(nm, valid ? v[c] : __builtin_inff());
        keep[c] = valid && keyof<NEG>(v[c]) >= T0;
        any_keep = any_keep || keep[c];
      }
      if (void0 || __builtin_amdgcn_ballot_w64(any_keep) == 0) return;
      uint64_t m[G];
      uint32_t pos = n0, total = 0;
#pragma unroll
      for (int c = 0; c < G; ++c) {
        m[c] = __builtin_amdgcn_ballot_w64(keep[c]);
        pos = lanes_below(m[c], pos);
        total += (uint32_t)__builtin_popcountll(m[c]);
      }
      if (n0 + total > (uint32_t)kKeptPerWave) {
        void0 = true;
        return;
      }
#pragma unroll
      for (int c = 0; c < G; ++c) {
        if (keep[c]) kept[pos] = make_uint2(__float_as_uint(v[c]), (uint32_t)(c0 + c));
        pos += keep[c] ? 1u : 0u;
      }
      n0 += total;
    };
    // Raising the floor.  The kept keys of the whole workgroup are counted into 256 equal parts of
    // [lower, upper) -- lower the current floor (the smallest key seen, the first time), upper the largest key
    // seen up to the previous raise (larger keys fall into the top part, which has no upper end) -- each key
    // into the part whose ends, computed as lower + j * width, enclose it: the arithmetic guess is corrected
    // against those very ends, so the suffix sums of the parts are exact counts of key >= lower + j * width.
    // The new floor is the lower end of the highest part with more than k + margin keys at or above it; the
    // margin leaves room below the k-th key for a search that stops early (its last threshold must not end
    // below the floor if the lists are to be used).  One histogram for the workgroup, three of them in turn:
    // a raise counts into one, clears the next, and the third may still be read by a wavefront that is late
    // leaving the previous raise; so a raise needs one barrier (two the first time, for the bounds).
    float upper = 0.0f;
    int raises = 0;
    const int wanted = k + (k / 2 > 64 ? k / 2 : 64);
    auto raise_floor = [&]() {  // called by the whole workgroup
      float lower = T0;
      if (raises == 0) {  // uniform
        float wmax, wmin;
        wave_max_and_negmin(mx, nm, wmax, wmin);
        if (lane == 0) {
          s_hi[wave] = wmax;
          s_nlo[wave] = -wmin;
        }
        __syncthreads();
        float a = s_hi[0], b = s_nlo[0];
#pragma unroll
        for (int w = 1; w < kStreamWaves; ++w) {
          a = vmax(a, s_hi[w]);
          b = vmax(b, s_nlo[w]);
        }
        const float seen_max = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a)));
        const float seen_min = -__int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(b)));
        upper = NEG ? -seen_min : seen_max;  // largest and smallest key seen
        lower = NEG ? -seen_max : seen_min;
      }
      int* parts = s_parts[raises % 3];
      if (tid < kLeaves) s_parts[(raises + 1) % 3][tid] = 0;
      {
        // the largest key seen so far, for the next raise (exchanged through this raise's barrier)
        float wmax, wmin;
        wave_max_and_negmin(mx, nm, wmax, wmin);
        if (lane == 0) s_top[raises & 1][wave] = NEG ? -wmin : wmax;
      }
      const int turn = raises & 1;
      ++raises;
      const float width = (upper - lower) * (1.0f / kLeaves);
      const float scale = (float)kLeaves / (upper - lower);
      const bool usable = upper > lower && width > 0.0f && width < __builtin_inff() && scale < __builtin_inff();  // false for NaN as well
      const uint32_t n_own = void0 ? 0u : n0;
      if (usable) {
        for (uint32_t j0 = 0; j0 < n_own; j0 += kWave) {
          const uint32_t j = j0 + (uint32_t)lane;
          if (j < n_own) {
            const float key = keyof<NEG>(__uint_as_float(kept[j].x));
            int part = (int)((key - lower) * scale);
            part = part < 0 ? 0 : (part > kLeaves - 1 ? kLeaves - 1 : part);
            while (part > 0 && key < lower + (float)part * width) --part;
            while (part < kLeaves - 1 && key >= lower + (float)(part + 1) * width) ++part;
            atomicAdd(&parts[part], 1);
          }
        }
      }
      __syncthreads();
      {
        float a = s_top[turn][0];
#pragma unroll
        for (int w = 1; w < kStreamWaves; ++w) a = vmax(a, s_top[turn][w]);
        upper = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a)));  // not used before the next raise
      }
      // every wavefront sums the parts from the top for itself: lane l holds parts 4l .. 4l + 3
      const int4 h = *reinterpret_cast<const int4*>(&parts[lane * 4]);
      const uint32_t own = (uint32_t)(h.x + h.y + h.z + h.w);
      const uint32_t incl = wave_inclusive_scan_dpp(own);
      const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
      const int s3 = (int)(total - incl) + h.w, s2 = s3 + h.z, s1 = s2 + h.y, s0 = s1 + h.x;  // keys at or above the lower end of part 4l + i
      const int enough = __builtin_popcountll(__builtin_amdgcn_ballot_w64(s0 > wanted)) +
                         __builtin_popcountll(__builtin_amdgcn_ballot_w64(s1 > wanted)) +
                         __builtin_popcountll(__builtin_amdgcn_ballot_w64(s2 > wanted)) +
                         __builtin_popcountll(__builtin_amdgcn_ballot_w64(s3 > wanted));  // a prefix of the parts: the sums never increase
      const int part = enough - 1;
      const float floor_new = lower + (float)part * width;
      if (usable && part > 0 && floor_new > T0) {  // uniform over the workgroup
        T0 = floor_new;
        uint32_t n_new = 0;  // drop what fell below; an entry never moves up, and a round only writes below what the next reads
        for (uint32_t j0 = 0; j0 < n_own; j0 += kWave) {
          const uint32_t j = j0 + (uint32_t)lane;
          const uint2 e = j < n_own ? kept[j] : make_uint2(0u, 0u);
          const bool stay = j < n_own && keyof<NEG>(__uint_as_float(e.x)) >= T0;
          const uint64_t m = __builtin_amdgcn_ballot_w64(stay);
          if (stay) kept[lanes_below(m, n_new)] = e;
          n_new += (uint32_t)__builtin_popcountll(m);
        }
        if (!void0) n0 = n_new;
      }
    };
    // The floor is raised after 1, 2, 4, 8, ... loads per wavefront: after the first (nothing filters that
    // load, so the list is full of it), and so on; i, j, trips and next_raise are uniform over the workgroup.
    int next_raise = 2;
    float ring[kAhead][G];
#pragma unroll
    for (int j = 0; j < kAhead; ++j) load_slot_once(j, ring[j]);
    for (int i = 0; i < trips; i += kAhead) {
#pragma unroll
      for (int j = 0; j < kAhead; ++j) {
        take(ring[j], u0 + i + j);
        load_slot_once(i + j + kAhead, ring[j]);
        const int done = i + j + 1;
        if (done < trips && (done == 1 || done == next_raise)) {
          if (done > 1) next_raise *= 2;
          raise_floor();
        }
      }
    }
    float wmax, wmin;
    wave_max_and_negmin(mx, nm, wmax, wmin);
    if (lane == 0) {
      s_hi[wave] = wmax;
      s_nlo[wave] = -wmin;
      s_void[wave] = void0 ? 1 : 0;
    }
    __syncthreads();
    float a = s_hi[0], b = s_nlo[0];
    int any_void = s_void[0];
#pragma unroll
    for (int w = 1; w < kStreamWaves; ++w) {
      a = vmax(a, s_hi[w]);
      b = vmax(b, s_nlo[w]);
      any_void |= s_void[w];
    }
    const float row_max = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a)));
    const float row_min = -__int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(b)));
    hi = NEG ? -row_min : row_max;  // bounds of the keys (negated values for the k smallest)
    lo = NEG ? -row_max : row_min;
    void0 = __builtin_amdgcn_readfirstlane(any_void) != 0;  // from here on uniform over the workgroup
  }

  // #{keys >= t} by one plain pass over the row (used only where no histogram pass has run).
  auto count_pass = [&](float t) -> int {
    int mine = 0;
#pragma unroll 4
    for (int c0 = tid * G; c0 < M; c0 += kChunk) {
      float v[G];
      stream_load<G>(row + c0, v);
#pragma unroll
      for (int c = 0; c < G; ++c) mine += keyof<NEG>(v[c]) >= t ? 1 : 0;
    }
    mine = wave_sum(mine);
    __syncthreads();  // s_above may still be read from an earlier use
    if (lane == 0) s_above[wave] = mine;
    __syncthreads();
    return __builtin_amdgcn_readfirstlane((int)row16_sum(lane < kStreamWaves ? (uint32_t)s_above[lane] : 0u));
  };

  // ---- search: eight steps per pass ---------------------------------------------------------------------
  // All of lo, hi, thres, steps, hit, na are uniform over the workgroup: every thread replays the same
  // steps on the same counts.
  bool hit = false;
  float thres = lo;
  int steps = 0;   // midpoints evaluated (Algorithm 1's iteration numbering; Algorithm 2's trip count)
  int na = -1;     // #{key >= hi} once known
  const float eps = MODE == kEps ? eps_rel * __builtin_fabsf(hi) : 0.0f;
  // ---- search on the lists of pass 0 ---------------------------------------------------------------------
  // Algorithm 1 / Algorithm 2 step by step, each count taken over the lists (see pass 0 for why that is
  // enough), with the guards of the replay further down.
  bool searched = false;
  if (!void0) {  // uniform over the workgroup
    searched = true;
    float lk[kKeptPerWave / kWave];  // this wavefront's kept keys, lane + 64 i; a key of -inf beyond the list
#pragma unroll
    for (int i = 0; i < kKeptPerWave / kWave; ++i) {
      const uint32_t j = (uint32_t)(i * kWave + lane);
      lk[i] = j < n0 ? keyof<NEG>(__uint_as_float(kept[j].x)) : -__builtin_inff();
    }
    int turn = 0;
    auto count_lists = [&](float t) -> int {  // one barrier; the halves of s_cnt alternate as in rtopk_block_kernel
      int mine = 0;
#pragma unroll
      for (int i = 0; i < kKeptPerWave / kWave; ++i) mine += __builtin_popcountll(__builtin_amdgcn_ballot_w64(lk[i] >= t));
      const int p = turn & 1;
      ++turn;
      if (lane == 0) s_cnt[p][wave] = mine;
      __syncthreads();
      return __builtin_amdgcn_readfirstlane((int)row16_sum(lane < kStreamWaves ? (uint32_t)s_cnt[p][lane] : 0u));
    };
    for (;;) {
      if (MODE == kEarly && steps >= max_iter) break;
      if (MODE == kEps && !(hi - lo > eps)) break;
      const float mid = (lo + hi) * 0.5f;
      if (!(mid > lo && mid < hi)) {
        // no fp32 value strictly inside (lo, hi): see the same test in the loop over passes below
        if (MODE == kEarly && mid == hi && hi > lo) {
          if (na < 0) na = count_lists(hi);
          if (na >= k) lo = hi;
        }
        break;
      }
      const int cnt = count_lists(mid);
      thres = mid;
      ++steps;
      if (cnt == k) {
        hit = true;
        if (MODE == kEarly) lo = mid;  // Algorithm 2 moves min here; later steps cannot change the selection
        break;
      }
      if (cnt < k) {
        hi = mid;
        na = cnt;
      } else {
        lo = mid;
      }
    }
    if (MODE != kEarly && !hit && na < 0) na = count_lists(hi);  // hi is still the row's maximum, which is on a list
  }

  bool kept_valid = false;  // a search pass has run and left its lists
  float kept_bstar = lo;    // what the lists of the last pass were filtered by at its end (uniform)
  uint32_t kept_n = 0;      // this wavefront's list length (above kKeptPerWave: overflowed)
  while (!searched) {
    if (MODE == kEarly && steps >= max_iter) break;
    if (MODE == kEps && !(hi - lo > eps)) break;
    {
      const float mid = (lo + hi) * 0.5f;
      if (!(mid > lo && mid < hi)) {
        // No fp32 value strictly inside (lo, hi).  Algorithm 1 ends here.  Algorithm 2 has no such test, but
        // from here on its steps repeat one midpoint, equal to lo (a step that moves nothing) or to hi (which
        // moves lo up to hi when hi itself counts k or more, and nothing otherwise): one replay settles it.
        if (MODE == kEarly && mid == hi && hi > lo) {
          if (na < 0) na = count_pass(hi);
          if (na >= k) lo = hi;
        }
        break;
      }
    }
    // the tree of midpoints below (lo, hi): leaf j's path from the root, one node per level.  s_tab holds
    // the nodes in heap order (for the replay), s_bnd the same thresholds in value order: s_bnd[j] is the
    // lower end of leaf j, s_bnd[0] = lo, s_bnd[256] = hi; it never decreases, because a rounded midpoint
    // lies within its interval.
    if (tid < kLeaves) {
      float a = lo, b = hi;
#pragma unroll
      for (int l = 0; l < kLevels; ++l) {
        const float t = (a + b) * 0.5f;
        const int pos = tid >> (kLevels - l);  // position of the node within its level
        s_tab[(1 << l) + pos] = t;
        s_bnd[(2 * pos + 1) << (kLevels - 1 - l)] = t;
        if ((tid >> (kLevels - 1 - l)) & 1) a = t; else b = t;
      }
    }
    if (tid == 0) {
      s_bnd[0] = lo;
      s_bnd[kLeaves] = hi;
    }
    for (int i = lane; i < kLeaves; i += kWave) s_hist[wave][i] = 0;
    __syncthreads();
    // One pass: keys at or above hi are counted, band members are sorted into their leaf.  The leaf is
    // found from an arithmetic estimate (the leaves are 256 nearly equal parts of [lo, hi)) corrected by a
    // walk along s_bnd until s_bnd[j] <= key < s_bnd[j + 1] -- the leaf the descent through the tree would
    // reach, since both put the key into the one non-empty leaf interval that contains it.  The G elements
    // of a thread advance together, so their LDS reads overlap.
    //
    // Most elements need no histogram at all.  A threshold whose count is already above k among the
    // elements seen so far is decided (cnt > k), whatever the rest of the row holds; so after 1, 4, 16, ...
    // chunks the partial histogram is summed and the highest leaf boundary with more than k seen elements
    // at or above it becomes `bstar`: from then on only keys >= bstar are sorted into leaves -- for k << M a
    // few percent of the row -- and the others cost two compares.  The suffix sums below bstar are then
    // lower bounds instead of exact counts, but each of them contains the (complete) sum at bstar, which
    // exceeds k, so the replay takes the same branch as with the exact count.
    //
    // Every wavefront walks its own contiguous sixteenth of the row (so that what it meets, it meets in
    // column order), one load ahead.  Besides the histogram it keeps a list of every key at or above bstar,
    // value and column: the final selection is a subset of the last pass's lists (the final thresholds are
    // at or above that pass's bstar, which is checked), so the k pairs can be ranked and written from LDS
    // without another pass over the row.  When bstar rises a wavefront drops the list entries below it.
    const float scale = (float)kLeaves / (hi - lo);
    int above = 0, jstar = 0, next_sync = 4;
    float bstar = lo;
    uint32_t n_kept = 0;      // entries of this wavefront's list
    bool overflowed = false;  // the list once ran full: it no longer holds every key at or above bstar
    // The leaf of a band member: the arithmetic estimate, one correction step (the estimate is rarely off by
    // more than one leaf), and a walk for whatever is still outside its leaf (near float resolution the
    // estimate is useless and the walk does all the work).
    auto find_leaf = [&](float key, bool inb) -> int {
      const float f = (key - lo) * scale;  // garbage for a degenerate scale: clamped, then walked
      int j = (int)f;
      j = j < 0 ? 0 : (j > kLeaves - 1 ? kLeaves - 1 : j);
      j = inb ? j : 0;
      {
        const float b0 = s_bnd[j], b1 = s_bnd[j + 1];
        if (inb) j += (key >= b1 ? 1 : 0) - (key < b0 ? 1 : 0);
      }
      j = j < 0 ? 0 : (j > kLeaves - 1 ? kLeaves - 1 : j);
      bool more = inb;
      while (more) {
        const float b0 = s_bnd[j], b1 = s_bnd[j + 1];
        if (key < b0) {
          --j;
        } else if (key >= b1) {
          ++j;
        } else {
          more = false;
        }
      }
      return j;
    };
    // List entries [n_done, n_kept) have not been counted yet: one entry per lane, so that the leaf search
    // and the atomic run on full wavefronts instead of on the one or two members a single load holds.
    uint32_t n_done = 0;
    auto count_pending = [&]() {
      for (uint32_t j0 = n_done; j0 < n_kept; j0 += kWave) {
        const uint32_t j = j0 + (uint32_t)lane;
        const bool live = j < n_kept;
        const float key = keyof<NEG>(__uint_as_float(live ? kept[j].x : 0u));
        const bool inb = live && !(key >= hi);  // entries are at or above the bstar they were met under
        const int leaf = find_leaf(key, inb);
        if (inb) atomicAdd(&s_hist[wave][leaf], 1);
      }
      n_done = n_kept;
    };
    // After 1, 4, 16, ... loads per wavefront: raise bstar to the highest decided leaf boundary.
    auto raise_bstar = [&]() {  // called by the whole workgroup
      count_pending();
      __syncthreads();
      int h = 0;
      if (tid < kLeaves) {
#pragma unroll
        for (int w = 0; w < kStreamWaves; ++w) h += s_hist[w][tid];
      }
      const int sum = suffix_of(h);
      if (tid < kLeaves) {
        // the sums never increase with the leaf index: the decided leaves are a prefix, counted by ballot
        const uint64_t decided = __builtin_amdgcn_ballot_w64(sum > k);
        if (lane == 0) s_pre[0][wave] = __builtin_popcountll(decided);
      }
      __syncthreads();
      const int n_decided = s_pre[0][0] + s_pre[0][1] + s_pre[0][2] + s_pre[0][3];
      if (n_decided - 1 > jstar) {
        jstar = n_decided - 1;
        bstar = s_bnd[jstar];
        if (overflowed) {
          n_kept = 0;  // everything in the list has been counted, and the list selects nothing any more
          n_done = 0;
        } else {
          // drop what fell below the new bstar; an entry never moves up, and a round only writes below
          // what the next round reads
          uint32_t n_new = 0;
          for (uint32_t j0 = 0; j0 < n_kept; j0 += kWave) {
            const uint32_t j = j0 + (uint32_t)lane;
            const uint2 e = j < n_kept ? kept[j] : make_uint2(0u, 0u);
            const bool stay = j < n_kept && keyof<NEG>(__uint_as_float(e.x)) >= bstar;
            const uint64_t m = __builtin_amdgcn_ballot_w64(stay);
            if (stay) kept[lanes_below(m, n_new)] = e;
            n_new += (uint32_t)__builtin_popcountll(m);
          }
          n_kept = n_new;
          n_done = n_new;
        }
      }
    };
    // One load of the wavefront (64 * G columns from unit u on), already in registers.
    auto process = [&](const float (&v)[G], int u) {
      // (this early exit makes the compiler wait for all loads in flight here; leaving it out, as pass 0
      // does, costs this pass registers it does not have: 18 spill, 1024 x 262144 with k = 2000 700 -> 779 us)
      if (u >= u1) return;  // uniform over the wavefront
      const int c0 = u * kUnit + lane * G;
      const bool valid = c0 < M;
      bool keep[G];
      bool any_keep = false;
#pragma unroll
      for (int c = 0; c < G; ++c) {
        const float key = keyof<NEG>(v[c]);
        above += (valid && key >= hi) ? 1 : 0;
        keep[c] = valid && key >= bstar;
        any_keep = any_keep || keep[c];
      }
      // once bstar has risen most loads of a wavefront hold no such key at all: one scalar branch
      if (__builtin_amdgcn_ballot_w64(any_keep) == 0) return;
      uint64_t m[G];
      uint32_t pos = 0, total = 0;
#pragma unroll
      for (int c = 0; c < G; ++c) {
        m[c] = __builtin_amdgcn_ballot_w64(keep[c]);
        pos = lanes_below(m[c], pos);
        total += (uint32_t)__builtin_popcountll(m[c]);
      }
      if (n_kept + total > (uint32_t)kKeptPerWave) {
        // The list is full.  Its entries are counted and dropped, and from here on it only batches keys for
        // the histogram: the selection will have to come from another pass over the row.
        count_pending();
        n_kept = 0;
        n_done = 0;
        overflowed = true;
      }
      pos += n_kept;
#pragma unroll
      for (int c = 0; c < G; ++c) {
        if (keep[c]) kept[pos] = make_uint2(__float_as_uint(v[c]), (uint32_t)(c0 + c));
        pos += keep[c] ? 1u : 0u;
      }
      n_kept += total;
    };
    // bstar is raised after 1, 4, 16, ... loads per wavefront (after the first because nothing filters that
    // load, so the list is full of it); i, j, trips and next_sync are uniform over the workgroup.
    float ring[kAhead][G];
#pragma unroll
    for (int j = 0; j < kAhead; ++j) load_slot(j, ring[j]);
    for (int i = 0; i < trips; i += kAhead) {
#pragma unroll
      for (int j = 0; j < kAhead; ++j) {
        process(ring[j], u0 + i + j);
        load_slot(i + j + kAhead, ring[j]);
        const int done = i + j + 1;
        if (done < trips && (done == 1 || done == next_sync)) {
          if (done > 1) next_sync *= 4;
          raise_bstar();
        }
      }
    }
    count_pending();
    kept_valid = true;
    kept_bstar = bstar;
    kept_n = overflowed ? (uint32_t)kKeptPerWave + 1u : n_kept;
    above = wave_sum(above);
    if (lane == 0) s_above[wave] = above;
    __syncthreads();
    // leaf totals over the wavefronts, then their suffix sums
    {
      int h = 0;
      if (tid < kLeaves) {
#pragma unroll
        for (int w = 0; w < kStreamWaves; ++w) h += s_hist[w][tid];
      }
      const int sum = suffix_of(h);
      if (tid < kLeaves) s_suffix[tid] = sum;
      if (tid == kLeaves) s_suffix[kLeaves] = 0;
      __syncthreads();
    }
    const int above_all = __builtin_amdgcn_readfirstlane((int)row16_sum(lane < kStreamWaves ? (uint32_t)s_above[lane] : 0u));
    na = above_all;
    // replay up to eight steps of the algorithm on the counts
    int node = 1;
    bool stop = false;
    for (int l = 0; l < kLevels; ++l) {
      if (MODE == kEarly && steps >= max_iter) { stop = true; break; }
      if (MODE == kEps && !(hi - lo > eps)) { stop = true; break; }
      const float t = s_tab[node];  // == (lo + hi) * 0.5f by construction
      if (!(t > lo && t < hi)) break;  // handled at the top of the outer loop
      const int split = ((2 * node + 1) << (kLevels - 1 - l)) - kLeaves;  // first leaf at or above t
      const int cnt = above_all + s_suffix[split];
      thres = t;
      ++steps;
      if (cnt == k) {
        hit = true;
        if (MODE == kEarly) lo = t;  // Algorithm 2 moves min here; later steps cannot change the selection
        stop = true;
        break;
      }
      if (cnt < k) {
        hi = t;
        na = cnt;
        node = 2 * node;
      } else {
        lo = t;
        node = 2 * node + 1;
      }
    }
    __syncthreads();  // the table and the histograms are rebuilt by the next pass
    if (stop) break;
  }
  if constexpr (MODE == kEps) {
    if (out_iters != nullptr && tid == 0) out_iters[r] = hit ? steps : steps + 1;
  }

  // ---- the selection: two classes of elements and a limit for each (as in rtopk_block_kernel) -----------
  //   class A: key >= tA, the first limA in column order;  class B: tB <= key < tA, the first limB.
  float tA, tB = 0.0f;
  int limA = k, limB = 0;
  if (MODE == kEarly) {
    tA = lo;  // the first k of key >= min
  } else if (hit) {
    tA = thres;  // exactly k keys
  } else {
    if (na < 0) na = lo < hi ? count_pass(hi) : M;  // no pass has run: every key equals hi, or the guard ended the loop at once
    tA = hi;
    tB = lo;
    limA = na < k ? na : k;
    limB = k - limA;
  }

  // ---- last pass: rank in column order and write ----------------------------------------------------------
  float* ov = out_vals + r * (int64_t)k;
  int32_t* oi = out_idx + r * (int64_t)k;

  // The k pairs from per-wavefront lists in LDS.  Each list holds (value bits, column) in column order and
  // the lists follow each other in wavefront order; every candidate of the row is in one of them (the
  // caller's claim, `complete`), possibly among entries that are no candidates.  n is this wavefront's list
  // length, or more than `cap` for a list that overflowed.  Every wavefront counts its candidates of either
  // class, the counts are exchanged through one barrier, and if all lists are whole each wavefront ranks and
  // writes its own behind those before it.  Returns whether the pairs were written (uniform).
  auto write_from_lists = [&](const uint2* list, uint32_t n, uint32_t cap, bool complete) -> bool {
    const bool whole = n <= cap;
    auto classes = [&](uint32_t j, uint2& e, bool& isA, bool& isB) {
      const bool live = whole && j < n;
      e = live ? list[j] : make_uint2(0u, 0u);
      const float key = keyof<NEG>(__uint_as_float(e.x));
      isA = live && key >= tA;
      isB = live && limB > 0 && key >= tB && !isA;
    };
    uint32_t nA = 0, nB = 0;
    for (uint32_t j0 = 0; whole && j0 < n; j0 += kWave) {
      uint2 e;
      bool isA, isB;
      classes(j0 + (uint32_t)lane, e, isA, isB);
      nA += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(isA));
      nB += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(isB));
    }
    if (lane == 0) {
      s_pre[0][wave] = whole ? (int)nA : -1;
      s_pre[1][wave] = (int)nB;
    }
    __syncthreads();
    uint32_t beforeA = 0, beforeB = 0;
    bool ok = complete;
#pragma unroll
    for (int w = 0; w < kStreamWaves; ++w) {
      const int a = s_pre[0][w];
      ok = ok && a >= 0;
      beforeA += w < wave ? (uint32_t)a : 0u;
      beforeB += w < wave ? (uint32_t)s_pre[1][w] : 0u;
    }
    if (ok) {  // uniform over the workgroup
      for (uint32_t j0 = 0; j0 < n; j0 += kWave) {
        uint2 e;
        bool isA, isB;
        classes(j0 + (uint32_t)lane, e, isA, isB);
        const uint64_t mA = __builtin_amdgcn_ballot_w64(isA), mB = __builtin_amdgcn_ballot_w64(isB);
        const uint32_t posA = lanes_below(mA, beforeA), posB = lanes_below(mB, beforeB);
        if ((isA && posA < (uint32_t)limA) || (isB && posB < (uint32_t)limB)) {
          const uint32_t pos = (posA < (uint32_t)limA ? posA : (uint32_t)limA) + (posB < (uint32_t)limB ? posB : (uint32_t)limB);
          ov[pos] = __uint_as_float(e.x);
          oi[pos] = (int32_t)e.y;
        }
        beforeA += (uint32_t)__builtin_popcountll(mA);
        beforeB += (uint32_t)__builtin_popcountll(mB);
      }
    }
    __syncthreads();  // s_pre is used again by whatever follows
    return ok;
  };

  // First choice: the lists the last search pass left.  They hold every key at or above that pass's final
  // bstar; the selection's lowest threshold is at or above it whenever the replay ran the tree to its leaves
  // or stopped on a count of k (then cnt(threshold) = k < cnt(bstar)), but not, for one, when max_iter ended
  // the replay on a coarser level -- hence the test.  (A NaN threshold fails it as well.)
  if (searched) {
    const float t_min = limB > 0 ? tB : tA;
    if (write_from_lists(kept, n0, (uint32_t)kKeptPerWave, t_min >= T0)) return;
  } else if (kept_valid) {
    const float t_min = limB > 0 ? tB : tA;
    if (write_from_lists(kept, kept_n, (uint32_t)kKeptPerWave, t_min >= kept_bstar)) return;
  }

  // Second: one more pass, for the usual case of few candidates (k <= 2048 and no wavefront meeting more
  // than 128 of them): every wavefront scans its own contiguous sixteenth of the row with no barrier at
  // all, appending the candidates it meets -- in column order -- to a list of its own in LDS (the histogram's
  // memory, free by now).  If a list overflows, the general form below redoes the pass.
  constexpr int kListPerWave = kLeaves * (int)sizeof(int) / (int)sizeof(uint2);  // 128 pairs in a wavefront's histogram
  if (k <= kStreamWaves * kListPerWave) {
    uint2* list = reinterpret_cast<uint2*>(&s_hist[wave][0]);
    uint32_t wn = 0;  // candidates met by this wavefront
    float ring[kAhead][G];
#pragma unroll
    for (int j = 0; j < kAhead; ++j) load_slot(j, ring[j]);
    for (int i = 0; i < u1 - u0 && wn <= (uint32_t)kListPerWave; i += kAhead) {  // an overflowing list ends the attempt
#pragma unroll
      for (int j = 0; j < kAhead; ++j) {
        const int u = u0 + i + j;
        const int c0 = u * kUnit + lane * G;
        const bool valid = u < u1 && c0 < M;
        float v[G];
        bool cand[G], any = false;
#pragma unroll
        for (int c = 0; c < G; ++c) {
          v[c] = ring[j][c];
          const float key = keyof<NEG>(v[c]);
          cand[c] = valid && (key >= tA || (limB > 0 && key >= tB));
          any = any || cand[c];
        }
        load_slot(i + j + kAhead, ring[j]);
        if (__builtin_amdgcn_ballot_w64(any) != 0) {  // most loads of a wide row hold no candidate
          uint64_t m[G];
          uint32_t pos = wn;
#pragma unroll
          for (int c = 0; c < G; ++c) {
            m[c] = __builtin_amdgcn_ballot_w64(cand[c]);
            pos = lanes_below(m[c], pos);
          }
#pragma unroll
          for (int c = 0; c < G; ++c) {
            if (cand[c] && pos < (uint32_t)kListPerWave) list[pos] = make_uint2(__float_as_uint(v[c]), (uint32_t)(c0 + c));
            pos += cand[c] ? 1u : 0u;
            wn += (uint32_t)__builtin_popcountll(m[c]);
          }
        }
      }
    }
    if (write_from_lists(list, wn, (uint32_t)kListPerWave, true)) return;
  }

  // General form: chunk by chunk, the candidates' ranks through one barrier per chunk.
  uint32_t baseA = 0, baseB = 0;  // candidates of either class in earlier chunks (uniform)
  int parity = 0;
  float nv[G];  // loaded one chunk ahead
  if (tid * G < M) stream_load<G>(row + tid * G, nv);
  for (int cb = 0; cb < M; cb += kChunk) {
    const uint32_t selA0 = baseA < (uint32_t)limA ? baseA : (uint32_t)limA;
    const uint32_t selB0 = baseB < (uint32_t)limB ? baseB : (uint32_t)limB;
    if (selA0 + selB0 >= (uint32_t)k) break;  // all k pairs are written
    const int c0 = cb + tid * G;
    float v[G];
    bool a[G], b[G];
    uint32_t mine = 0;  // own candidates: A in the low half, B in the high half
    if (c0 < M) {
#pragma unroll
      for (int c = 0; c < G; ++c) v[c] = nv[c];
      if (c0 + kChunk < M) stream_load<G>(row + c0 + kChunk, nv);
#pragma unroll
      for (int c = 0; c < G; ++c) {
        const float key = keyof<NEG>(v[c]);
        a[c] = key >= tA;
        b[c] = limB > 0 && key >= tB && !a[c];
        mine += (a[c] ? 1u : 0u) + (b[c] ? 0x10000u : 0u);
      }
    } else {
#pragma unroll
      for (int c = 0; c < G; ++c) a[c] = b[c] = false;
    }
    const uint32_t incl = wave_inclusive_scan_dpp(mine);
    if (lane == kWave - 1) s_pre[parity][wave] = (int)incl;
    __syncthreads();
    uint32_t before = incl - mine;  // candidates in lower lanes of this wavefront
    uint32_t chunk_total = 0;
#pragma unroll
    for (int w = 0; w < kStreamWaves; ++w) {
      const uint32_t wt = (uint32_t)s_pre[parity][w];
      before += w < wave ? wt : 0u;
      chunk_total += wt;
    }
    parity ^= 1;
    uint32_t posA = baseA + (before & 0xffffu), posB = baseB + (before >> 16);
#pragma unroll
    for (int c = 0; c < G; ++c) {
      const bool chosen = (a[c] && posA < (uint32_t)limA) || (b[c] && posB < (uint32_t)limB);
      if (chosen) {
        const uint32_t pos = (posA < (uint32_t)limA ? posA : (uint32_t)limA) + (posB < (uint32_t)limB ? posB : (uint32_t)limB);
        ov[pos] = v[c];
        oi[pos] = c0 + c;
      }
      posA += a[c] ? 1u : 0u;
      posB += b[c] ? 1u : 0u;
    }
    baseA += chunk_total & 0xffffu;
    baseB += chunk_total >> 16;
  }
}

template <int G, int MODE, bool NEG>
hipError_t launch_stream(const LaunchArgs& a) {
  if (a.N > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  return launch_kernel(rtopk_stream_kernel<G, MODE, NEG>, dim3((unsigned)a.N), dim3(kStreamThreads), 0, a.stream,
                       static_cast<const float*>(a.in), a.N, a.M, a.k, a.max_iter, a.eps_rel,
                       static_cast<float*>(a.out_vals), static_cast<int32_t*>(a.out_idx), a.out_iters);
}

}  // namespace rtopk
