// Row-wise top-k for rows that no longer fit a workgroup's registers (65536 < M <= 2^24): one workgroup
// per row, the row streamed from memory several times.
//
// Same method and same results as the other kernels (RTop-K, arXiv 2409.00822, Section 3.1, Algorithms 1
// and 2).  Appendix B of the paper observes that for very wide rows a search that pays one pass over the
// row per bisection step loses to radix-style selection.  The remedy here keeps the paper's thresholds
// and takes kLevels = 8 bisection steps per pass instead of one: all 255 midpoints that the next eight
// steps can possibly visit are fixed by (lo, hi) alone -- they form a binary tree, each node the fp32
// midpoint of its interval exactly as the algorithms compute it -- so one pass sorts every element of
// the band [lo, hi) into the 256 leaf intervals of that tree (an arithmetic guess corrected against a table
// in LDS, one LDS atomic), and the suffix sums of that histogram are the counts cnt(t) of all 255
// thresholds at once.  The eight steps are then replayed on the counts, with the algorithms' own guards
// (cnt == k, the iteration limit, epsilon, the midpoint no longer strictly inside), bit for bit as the
// one-step-per-pass loop would have run them.  In effect: a radix-256 select over the value range whose
// digit boundaries are the paper's midpoints.  A row costs one pass for its minimum and maximum, one pass
// per eight search steps (one for Algorithm 2 with max_iter <= 8, two for a typical exact search), and
// one pass that ranks and writes the k pairs.
//
// Layout: thread t of 1024 owns columns c*1024*G + t*G .. +G-1 of chunk c (G = 4: 128-bit loads), so a
// chunk is 16 KiB contiguous and column order within a chunk is (thread, element).  Loads are ordinary
// cached loads: the row is read again by the next pass.
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
__global__ void __launch_bounds__(kStreamThreads)
    rtopk_stream_kernel(const float* __restrict__ in, int64_t N, int M, int k, int max_iter, float eps_rel,
                        float* __restrict__ out_vals, int32_t* __restrict__ out_idx, int32_t* __restrict__ out_iters) {
  __shared__ float s_tab[kLeaves];               // thresholds of the tree's nodes 1..255 (heap order; [0] unused)
  __shared__ float s_bnd[kLeaves + 1];           // the same thresholds in value order, with lo and hi at the ends
  __shared__ int s_hist[kStreamWaves][kLeaves];  // per-wavefront leaf histograms
  __shared__ int s_suffix[kLeaves + 1];          // suffix[j] = band members in leaves j..255
  __shared__ float s_hi[kStreamWaves], s_nlo[kStreamWaves];
  __shared__ int s_above[kStreamWaves];
  __shared__ int s_pre[2][kStreamWaves];  // per-wavefront candidate counts of a chunk (A in the low half, B in the high), double buffered

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t r = blockIdx.x;
  if (r >= N) return;
  const float* row = in + r * (int64_t)M;
  constexpr int kChunk = kStreamThreads * G;

  // ---- pass 0: row minimum and maximum -----------------------------------------------------------------
  float lo, hi;
  {
    float mx = -__builtin_inff(), nm = -__builtin_inff();
#pragma unroll 4
    for (int c0 = tid * G; c0 < M; c0 += kChunk) {
      float v[G];
      stream_load<G>(row + c0, v);
#pragma unroll
      for (int c = 0; c < G; ++c) {
        mx = vmax(mx, v[c]);
        nm = vmax_an(nm, v[c]);
      }
    }
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
    const float row_max = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a)));
    const float row_min = -__int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(b)));
    hi = NEG ? -row_min : row_max;  // bounds of the keys (negated values for the k smallest)
    lo = NEG ? -row_max : row_min;
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

  // ---- search: eight steps per pass ---------------------------------------------------------------------
  // All of lo, hi, thres, steps, hit, na are uniform over the workgroup: every thread replays the same
  // steps on the same counts.
  bool hit = false;
  float thres = lo;
  int steps = 0;   // midpoints evaluated (Algorithm 1's iteration numbering; Algorithm 2's trip count)
  int na = -1;     // #{key >= hi} once known
  const float eps = MODE == kEps ? eps_rel * __builtin_fabsf(hi) : 0.0f;
  for (;;) {
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
    const float scale = (float)kLeaves / (hi - lo);
    int above = 0, jstar = 0, next_sync = 1, chunk_i = 0;
    float bstar = lo;
    float nv[G];  // the thread's elements of the next chunk, loaded one chunk ahead
    if (tid * G < M) stream_load<G>(row + tid * G, nv);
    for (int cb = 0; cb < M; cb += kChunk, ++chunk_i) {
      if (chunk_i == next_sync) {  // uniform over the workgroup
        next_sync *= 4;
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
        }
      }
      const int c0 = cb + tid * G;
      if (c0 >= M) continue;
      float v[G];
#pragma unroll
      for (int c = 0; c < G; ++c) v[c] = nv[c];
      if (c0 + kChunk < M) stream_load<G>(row + c0 + kChunk, nv);
      float key[G];
      bool inb[G];
      bool mine = false;
#pragma unroll
      for (int c = 0; c < G; ++c) {
        key[c] = keyof<NEG>(v[c]);
        const bool ge_hi = key[c] >= hi;
        above += ge_hi ? 1 : 0;
        inb[c] = key[c] >= bstar && !ge_hi;
        mine = mine || inb[c];
      }
      // once bstar has risen most wavefronts hold no band member at all in a chunk: one scalar branch
      if (__builtin_amdgcn_ballot_w64(mine) != 0) {
        int leaf[G];
        bool more = false;
#pragma unroll
        for (int c = 0; c < G; ++c) {
          const float f = (key[c] - lo) * scale;  // garbage for keys outside the band or a degenerate scale: clamped, then walked
          int j = (int)f;
          j = j < 0 ? 0 : (j > kLeaves - 1 ? kLeaves - 1 : j);
          leaf[c] = inb[c] ? j : 0;
        }
        // one correction step for every element at once (the estimate is rarely off by more than one leaf) ...
#pragma unroll
        for (int c = 0; c < G; ++c) {
          const float b0 = s_bnd[leaf[c]], b1 = s_bnd[leaf[c] + 1];
          if (inb[c]) leaf[c] += (key[c] >= b1 ? 1 : 0) - (key[c] < b0 ? 1 : 0);
        }
#pragma unroll
        for (int c = 0; c < G; ++c) {
          const int j = leaf[c] < 0 ? 0 : (leaf[c] > kLeaves - 1 ? kLeaves - 1 : leaf[c]);
          leaf[c] = j;
          more = more || (inb[c] && (key[c] < s_bnd[j] || key[c] >= s_bnd[j + 1]));
        }
        // ... and the walk for whatever is still outside its leaf (near float resolution the estimate is useless)
        while (more) {
          more = false;
#pragma unroll
          for (int c = 0; c < G; ++c) {
            if (inb[c]) {
              const float b0 = s_bnd[leaf[c]], b1 = s_bnd[leaf[c] + 1];
              if (key[c] < b0) {
                --leaf[c];
                more = true;
              } else if (key[c] >= b1) {
                ++leaf[c];
                more = true;
              }
            }
          }
        }
#pragma unroll
        for (int c = 0; c < G; ++c) {
          if (__builtin_amdgcn_ballot_w64(inb[c]) != 0) {
            if (inb[c]) atomicAdd(&s_hist[wave][leaf[c]], 1);
          }
        }
      }
    }
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

  // Fast form, for the usual case of few candidates (k <= 2048 and no wavefront meeting more than 128 of
  // them): every wavefront scans its own contiguous sixteenth of the row with no barrier at all, appending
  // the candidates it meets -- in column order -- to a list of its own in LDS (the histogram's memory,
  // free by now); then one barrier, and every wavefront ranks and writes its list behind the candidates
  // of the wavefronts before it.  If a list overflows, the general form below redoes the pass.
  constexpr int kListPerWave = kLeaves * (int)sizeof(int) / (int)sizeof(uint2);  // 128 pairs in a wavefront's histogram
  bool listed = false;
  if (k <= kStreamWaves * kListPerWave) {
    uint2* list = reinterpret_cast<uint2*>(&s_hist[wave][0]);
    constexpr int kUnit = kWave * G;  // columns a wavefront covers per load
    const int units = (M + kUnit - 1) / kUnit;
    const int u0 = (int)((int64_t)units * wave / kStreamWaves), u1 = (int)((int64_t)units * (wave + 1) / kStreamWaves);
    uint32_t wn = 0, wnA = 0;  // candidates met by this wavefront, and those of class A among them
    float nv[G];
    if (u0 < u1 && u0 * kUnit + lane * G < M) stream_load<G>(row + u0 * kUnit + lane * G, nv);
    for (int u = u0; u < u1 && wn <= (uint32_t)kListPerWave; ++u) {  // an overflowing list ends the attempt
      const int c0 = u * kUnit + lane * G;
      float v[G];
      bool cand = false, a[G], b[G];
#pragma unroll
      for (int c = 0; c < G; ++c) v[c] = nv[c];
      if (u + 1 < u1 && c0 + kUnit < M) stream_load<G>(row + c0 + kUnit, nv);
#pragma unroll
      for (int c = 0; c < G; ++c) {
        const float key = keyof<NEG>(v[c]);
        a[c] = c0 < M && key >= tA;
        b[c] = c0 < M && limB > 0 && key >= tB && !a[c];
        cand = cand || a[c] || b[c];
      }
      if (__builtin_amdgcn_ballot_w64(cand) != 0) {  // most loads of a wide row hold no candidate
        uint64_t m[G];
        uint32_t pos = wn;
#pragma unroll
        for (int c = 0; c < G; ++c) {
          m[c] = __builtin_amdgcn_ballot_w64(a[c] || b[c]);
          pos = lanes_below(m[c], pos);
          wnA += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(a[c]));
        }
#pragma unroll
        for (int c = 0; c < G; ++c) {
          if ((a[c] || b[c]) && pos < (uint32_t)kListPerWave)
            list[pos] = make_uint2(__float_as_uint(v[c]), (uint32_t)(c0 + c) | (a[c] ? 0u : 0x80000000u));
          pos += (a[c] || b[c]) ? 1u : 0u;
          wn += (uint32_t)__builtin_popcountll(m[c]);
        }
      }
    }
    if (lane == 0) {
      s_pre[0][wave] = (int)wn;
      s_pre[1][wave] = (int)wnA;
    }
    __syncthreads();
    uint32_t beforeA = 0, beforeB = 0;
    bool fits = true;
#pragma unroll
    for (int w = 0; w < kStreamWaves; ++w) {
      const uint32_t n = (uint32_t)s_pre[0][w], nA = (uint32_t)s_pre[1][w];
      fits = fits && n <= (uint32_t)kListPerWave;
      beforeA += w < wave ? nA : 0u;
      beforeB += w < wave ? n - nA : 0u;
    }
    if (fits) {  // uniform over the workgroup
      listed = true;
      for (uint32_t j0 = 0; j0 < wn; j0 += kWave) {
        const uint32_t j = j0 + (uint32_t)lane;
        const bool live = j < wn;
        const uint2 e = live ? list[j] : make_uint2(0u, 0u);
        const bool isA = live && !(e.y >> 31), isB = live && (e.y >> 31);
        const uint64_t mA = __builtin_amdgcn_ballot_w64(isA), mB = __builtin_amdgcn_ballot_w64(isB);
        const uint32_t posA = lanes_below(mA, beforeA), posB = lanes_below(mB, beforeB);
        if ((isA && posA < (uint32_t)limA) || (isB && posB < (uint32_t)limB)) {
          const uint32_t pos = (posA < (uint32_t)limA ? posA : (uint32_t)limA) + (posB < (uint32_t)limB ? posB : (uint32_t)limB);
          ov[pos] = __uint_as_float(e.x);
          oi[pos] = (int32_t)(e.y & 0x7fffffffu);
        }
        beforeA += (uint32_t)__builtin_popcountll(mA);
        beforeB += (uint32_t)__builtin_popcountll(mB);
      }
    }
    __syncthreads();  // s_pre is used again below
  }
  if (listed) return;

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
