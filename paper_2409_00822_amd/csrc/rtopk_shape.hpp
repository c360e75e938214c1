// Shape classification of the row-wise top-k library: which kernel family and which register layout a
// call's row width, element type and pointer alignment map to.  Host code only (no HIP headers), so that
// it can also be compiled and swept by a CPU test under the address / undefined-behaviour sanitizers.
//
// A layout is (g, ng, w): a lane owns ng groups of g consecutive columns, and a row is spread over w
// wavefronts (w = 1: one wavefront per row, rtopk_kernel.hpp; w > 1: one workgroup per row,
// rtopk_block_kernel.hpp), so a layout holds rows of up to 64 * g * ng * w columns.  Which (g, ng, w) are
// compiled is fixed by the lists below; the instantiation tables (rtopk_inst_*.hip) expand the same lists,
// so a layout this header can return always has a kernel behind it.
#pragma once

#include <stdint.h>

// Groups per lane that are instantiated, per load width.  X(n) is expanded once per entry, ascending.
#define RTOPK_NG_LIST_G4(X) X(1) X(2) X(3) X(4) X(6) X(8) X(12) X(16) X(24) X(32)   /* fp32, 128-bit loads */
#define RTOPK_NG_LIST_H8(X) X(1) X(2) X(3) X(4) X(6) X(8) X(12) X(16)               /* 16-bit rows, 128-bit loads */
#define RTOPK_NG_LIST_G1(X) X(1) X(2) X(4) X(8) X(16) X(32) X(64) X(128)            /* scalar-load fallback */
#define RTOPK_NG_LIST_BLOCK_G1(X) X(16) X(32) X(64)                                 /* scalar-load fallback, 16 wavefronts */

namespace rtopk {

// Which algorithm of the paper (Section 3.1) a kernel instance runs.
enum Mode : int {
  kEarly = 0,  // Algorithm 2: max_iter steps, one-pass selection against min
  kExact = 1,  // Algorithm 1 at epsilon = 0
  kEps = 2     // Algorithm 1 with epsilon = eps_rel * |max|, optional exit-iteration output
};

// Element type of the input matrix and of the value output.
enum DType : int {
  kF32 = 0,
  kF16 = 1,  // IEEE half
  kBF16 = 2  // bfloat16
};

constexpr int kMaxM = 1 << 24;       // widest row at all (fp32 rows, int32 columns: streamed beyond kMaxBlockM)
constexpr int kMaxBlockM = 65536;    // widest row one workgroup holds in registers; the limit of the 16-bit and dense forms
constexpr int kMaxWaveM = 8192;      // widest row one wavefront holds in registers
constexpr int kBackwardRowsM = 2048;  // backward edge: widest row assembled whole in a wavefront's LDS (8 KiB)

enum Family : int {
  kFamSmall = 0,  // launch_small: even M <= 128 (g = 2) and the scalar-load fallback (g = 1)
  kFamG4 = 1,     // launch_g4_*: fp32, 128-bit loads
  kFamH16 = 2,    // launch_h16_*: half / bfloat16 rows, one wavefront per row
  kFamBlock = 3,  // launch_block_*: one workgroup per row, the row in registers
  kFamStream = 4  // launch_stream: one workgroup per row, the row streamed several times (fp32, int32 columns)
};

struct Shape {
  int family;
  int g, ng, w;
  bool full;  // M == 64 * g * ng * w: the kernel needs no column-validity tests
  int capacity() const { return 64 * g * ng * w; }
};

inline bool is_aligned(uintptr_t p, uintptr_t a) { return p % a == 0; }

// Smallest listed ng with 64 * g * ng >= M; `fallback` (the list's largest) when none is.
inline int pick_ng_g4(int M) {
#define X(n) if (M <= 256 * n) return n;
  RTOPK_NG_LIST_G4(X)
#undef X
  return 32;
}
inline int pick_ng_h8(int M) {
#define X(n) if (M <= 512 * n) return n;
  RTOPK_NG_LIST_H8(X)
#undef X
  return 16;
}
inline int pick_ng_g1(int M) {
#define X(n) if (M <= 64 * n) return n;
  RTOPK_NG_LIST_G1(X)
#undef X
  return 128;
}

// Wavefronts per row of the workgroup-per-row kernel: a lane holds up to 64 values.
inline int block_waves(int M) { return M <= 16384 ? 4 : (M <= 32768 ? 8 : 16); }

// Layout for the pair-output entry points.  `in` is the address of the input matrix (its alignment
// decides the load width); `plain` = fp32 rows, the k largest, Algorithm 2 or exact mode (the variants
// that have the 12-groups-per-lane workgroup kernels).  Requires 1 <= M <= kMaxM (kMaxBlockM for 16-bit rows).
inline Shape classify(int M, int dtype, bool plain, uintptr_t in) {
  Shape s{};
  s.w = 1;
  if (M > kMaxBlockM) {
    // streamed: nothing is held, so the "layout" is only the load width (full is never claimed)
    s.family = kFamStream;
    s.g = (M % 4 == 0 && is_aligned(in, 16)) ? 4 : 1;
    s.ng = 0;
    s.w = 16;
    s.full = false;
    return s;
  }
  if (M > kMaxWaveM) {
    s.family = kFamBlock;
    if (dtype == kF32 && M % 4 == 0 && is_aligned(in, 16)) {
      s.g = 4;
      s.w = block_waves(M);
      s.ng = (plain && M <= 64 * s.w * 4 * 12) ? 12 : 16;
    } else if (dtype != kF32 && M % 8 == 0 && is_aligned(in, 16)) {
      s.g = 8;
      s.w = block_waves(M);
      s.ng = 8;
    } else {
      s.g = 1;
      s.w = 16;
      s.ng = 16;
      while (1024 * s.ng < M) s.ng <<= 1;
    }
  } else if (dtype != kF32) {
    // 16-bit rows: the widest load whose 64 lanes the row still fills, else the scalar-load fallback
    s.family = kFamH16;
    if (M > 256 && M % 8 == 0 && is_aligned(in, 16)) {
      s.g = 8;
      s.ng = pick_ng_h8(M);
    } else if (M > 128 && M <= 256 && M % 4 == 0 && is_aligned(in, 8)) {
      s.g = 4;
      s.ng = 1;
    } else if (M > 64 && M <= 128 && M % 2 == 0 && is_aligned(in, 4)) {
      s.g = 2;
      s.ng = 1;
    } else {
      s.g = 1;
      s.ng = pick_ng_g1(M);
    }
  } else if (M > 128 && M % 4 == 0 && is_aligned(in, 16)) {
    s.family = kFamG4;
    s.g = 4;
    s.ng = pick_ng_g4(M);
  } else if (M > 64 && M <= 128 && M % 2 == 0 && is_aligned(in, 8)) {
    s.family = kFamSmall;
    s.g = 2;
    s.ng = 1;
  } else {
    s.family = kFamSmall;
    s.g = 1;
    s.ng = pick_ng_g1(M);
  }
  s.full = (M == s.capacity());
  return s;
}

// Layout for the dense-output entry point (fp32): the row is stored with the accesses it was loaded
// with, so the output's alignment counts as well.
inline Shape classify_dense(int M, uintptr_t in, uintptr_t out) {
  Shape s{};
  s.w = 1;
  if (M > kMaxWaveM) {
    s.family = kFamBlock;
    if (M % 4 == 0 && is_aligned(in, 16) && is_aligned(out, 16)) {
      s.g = 4;
      s.w = block_waves(M);
      s.ng = 16;
    } else {
      s.g = 1;
      s.w = 16;
      s.ng = 16;
      while (1024 * s.ng < M) s.ng <<= 1;
    }
  } else if (M > 128 && M % 4 == 0 && is_aligned(in, 16) && is_aligned(out, 16)) {
    s.family = kFamG4;
    s.g = 4;
    s.ng = pick_ng_g4(M);
  } else if (M > 64 && M <= 128 && M % 2 == 0 && is_aligned(in, 8) && is_aligned(out, 8)) {
    s.family = kFamSmall;
    s.g = 2;
    s.ng = 1;
  } else {
    s.family = kFamSmall;
    s.g = 1;
    s.ng = pick_ng_g1(M);
  }
  s.full = (M == s.capacity());
  return s;
}

// True when (g, ng, w) is in the compiled set of its family (the same lists the instantiation tables
// expand).  `plain` and `dense` as above.
inline bool instantiated(const Shape& s, int dtype, bool plain, bool dense) {
  auto in_list = [](int n, int which) {
    bool hit = false;
#define X(v) hit = hit || (n == v);
    if (which == 0) { RTOPK_NG_LIST_G4(X) }
    if (which == 1) { RTOPK_NG_LIST_H8(X) }
    if (which == 2) { RTOPK_NG_LIST_G1(X) }
    if (which == 3) { RTOPK_NG_LIST_BLOCK_G1(X) }
#undef X
    return hit;
  };
  switch (s.family) {
    case kFamSmall:
      return s.w == 1 && ((s.g == 2 && s.ng == 1) || (s.g == 1 && in_list(s.ng, 2)));
    case kFamG4:
      return s.w == 1 && s.g == 4 && dtype == kF32 && in_list(s.ng, 0);
    case kFamH16:
      if (s.w != 1 || dtype == kF32) return false;
      return (s.g == 8 && in_list(s.ng, 1)) || ((s.g == 4 || s.g == 2) && s.ng == 1) || (s.g == 1 && in_list(s.ng, 2));
    case kFamStream:
      return dtype == kF32 && !dense && s.w == 16 && (s.g == 4 || s.g == 1);
    case kFamBlock:
      if (s.g == 1) return s.w == 16 && in_list(s.ng, 3);
      if (s.w != 4 && s.w != 8 && s.w != 16) return false;
      if (dtype != kF32) return !dense && s.g == 8 && s.ng == 8;
      return s.g == 4 && (s.ng == 16 || (s.ng == 12 && plain && !dense));
    default:
      return false;
  }
}

// Largest max_iter that is evaluated literally.  Each step of Algorithm 2 halves hi - lo, so on finite
// fp32 input the rounded midpoint equals lo or hi after at most ~300 steps (from a range of 2^129 down
// to the smallest subnormal, plus 24 mantissa bits); from then on a step changes neither bound, so a
// larger step count gives bit-identical output.  The clamp keeps a huge max_iter (a caller's way of
// saying "no early stop") from spinning on rows whose k-th place is tied and so never count exactly k.
constexpr int kMaxIterClamp = 512;

// True when the byte ranges [a, a + na) and [b, b + nb) share a byte.
inline bool ranges_overlap(uintptr_t a, uint64_t na, uintptr_t b, uint64_t nb) {
  if (na == 0 || nb == 0) return false;
  return a < b + nb && b < a + na;
}

}  // namespace rtopk
