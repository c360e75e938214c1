// C ABI of the row-wise top-k library: argument checks, shape classification, launch.
// Declarations and the full contract are in include/rtopk.h.
#include "rtopk.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rtopk_dispatch.hpp"

namespace {

constexpr int kMaxM = 65536;     // one workgroup per row beyond kMaxWaveM
constexpr int kMaxWaveM = 8192;  // widest row one wavefront holds in registers
constexpr int kVersion = 500;  // 0.5.0

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Shared body of the selection entry points.
//   mode: rtopk::kEarly (Algorithm 2, max_iter steps), kExact (Algorithm 1, epsilon = 0) or
//         kEps (Algorithm 1, epsilon = eps_rel * |max|, optional exit-iteration output).
//   u8:   out_idx is uint8_t[N][k] (requires M <= 256), else int32_t[N][k].
//   dtype: element type of `in` and `out_vals` (rtopk::kF32, kF16, kBF16).
int run(const void* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float eps_rel, int mode, void* out_vals,
        void* out_idx, int32_t* out_iters, bool u8, void* stream, bool smallest = false, int dtype = rtopk::kF32) {
  const uintptr_t esz = dtype == rtopk::kF32 ? 4 : 2;
  if (N < 0 || M < 1 || k < 1 || k > M) return RTOPK_ERR_BAD_SHAPE;
  if (mode == rtopk::kEarly && max_iter < 0) return RTOPK_ERR_BAD_MAX_ITER;
  if (mode == rtopk::kEps && !(eps_rel >= 0.0f)) return RTOPK_ERR_BAD_EPSILON;
  if (M > kMaxM || (u8 && M > 256)) return RTOPK_ERR_M_TOO_LARGE;
  if (N == 0) return RTOPK_OK;
  if (!in || !out_vals || !out_idx) return RTOPK_ERR_NULL_POINTER;
  if (!aligned(in, esz) || !aligned(out_vals, esz) || (!u8 && !aligned(out_idx, 4)) || !aligned(out_iters, 4))
    return RTOPK_ERR_MISALIGNED;

  // k == M: every column is selected.  Algorithm 2 with zero steps returns the first k columns,
  // which is that answer without a search that would otherwise run down to float resolution.
  if (mode == rtopk::kExact && k == M) {
    mode = rtopk::kEarly;
    max_iter = 0;
  }

  rtopk::LaunchArgs a;
  a.in = in;
  a.N = N;
  a.M = M;
  a.k = k;
  a.max_iter = max_iter;
  a.eps_rel = eps_rel;
  a.out_iters = out_iters;
  a.smallest = smallest;
  a.out_vals = out_vals;
  a.out_idx = out_idx;
  a.vec_store = (k % 4 == 0) && aligned(out_vals, 4 * esz) && aligned(out_idx, u8 ? 4 : 16);
  a.stream = static_cast<hipStream_t>(stream);

  hipError_t err;
  if (M > kMaxWaveM) {
    if (N > 0x7fffffffLL) return RTOPK_ERR_BAD_SHAPE;  // one workgroup per row: the grid holds 2^31 - 1 rows
    // a lane holds up to 64 values: 4 wavefronts up to 16384 columns, 8 up to 32768, 16 beyond
    int g = 1, ng = 16, w = 16;
    const bool plain = dtype == rtopk::kF32 && !smallest && mode != rtopk::kEps;
    if (dtype == rtopk::kF32 && M % 4 == 0 && aligned(in, 16)) {
      g = 4;
      w = M <= 16384 ? 4 : (M <= 32768 ? 8 : 16);
      ng = (plain && M <= 64 * w * 4 * 12) ? 12 : 16;
    } else if (dtype != rtopk::kF32 && M % 8 == 0 && aligned(in, 16)) {
      g = 8;
      w = M <= 16384 ? 4 : (M <= 32768 ? 8 : 16);
      ng = 8;
    } else {
      while (1024 * ng < M) ng <<= 1;
    }
    err = dtype != rtopk::kF32 ? rtopk::launch_block_h16(dtype, g, ng, w, mode, a)
          : plain              ? rtopk::launch_block_plain(g, ng, w, mode, a)
                               : rtopk::launch_block_variant(g, ng, w, mode, smallest, a);
  } else if (dtype != rtopk::kF32) {
    // 16-bit rows: the widest load whose 64 lanes the row still fills, else the scalar-load fallback
    int g = 1, ng = 1;
    bool full = false;
    if (M > 256 && M % 8 == 0 && aligned(in, 16)) {
      static const int kNg[] = {1, 2, 3, 4, 6, 8, 12, 16};
      g = 8;
      ng = 16;
      for (int cand : kNg) {
        if (M <= 512 * cand) {
          ng = cand;
          break;
        }
      }
    } else if (M > 128 && M <= 256 && M % 4 == 0 && aligned(in, 8)) {
      g = 4;
    } else if (M > 64 && M <= 128 && M % 2 == 0 && aligned(in, 4)) {
      g = 2;
    } else {
      while (64 * ng < M) ng <<= 1;
    }
    full = (M == 64 * g * ng);
    err = mode == rtopk::kExact ? rtopk::launch_h16_exact(dtype, g, ng, full, a)
                                : rtopk::launch_h16_early(dtype, g, ng, full, a);
  } else if (M > 128 && M % 4 == 0 && aligned(in, 16)) {
    // 128-bit loads; groups per lane rounded up to an instantiated count
    static const int kNg[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32};
    int ng = 32;
    for (int cand : kNg) {
      if (M <= 256 * cand) {
        ng = cand;
        break;
      }
    }
    const bool full = (M == 256 * ng);
    err = mode == rtopk::kExact   ? rtopk::launch_g4_exact(ng, full, u8, a)
          : mode == rtopk::kEarly ? rtopk::launch_g4_early(ng, full, u8, a)
                                  : rtopk::launch_g4_eps(ng, full, a);
  } else if (M > 64 && M <= 128 && M % 2 == 0 && aligned(in, 8)) {
    err = rtopk::launch_small(2, 1, M == 128, mode, u8, a);
  } else {
    int ng = 1;
    while (64 * ng < M) ng <<= 1;
    err = rtopk::launch_small(1, ng, M == 64 * ng, mode, u8, a);
  }
  return err == hipSuccess ? RTOPK_OK : RTOPK_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int rtopk_rowwise(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out_vals,
                  int32_t* out_idx, void* stream) {
  return run(in, N, M, k, max_iter, 0.0f, rtopk::kEarly, out_vals, out_idx, nullptr, false, stream);
}

int rtopk_rowwise_exact(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, int32_t* out_idx,
                        void* stream) {
  return run(in, N, M, k, 0, 0.0f, rtopk::kExact, out_vals, out_idx, nullptr, false, stream);
}

int rtopk_rowwise_u8(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out_vals,
                     uint8_t* out_idx, void* stream) {
  return run(in, N, M, k, max_iter, 0.0f, rtopk::kEarly, out_vals, out_idx, nullptr, true, stream);
}

int rtopk_rowwise_exact_u8(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, uint8_t* out_idx,
                           void* stream) {
  return run(in, N, M, k, 0, 0.0f, rtopk::kExact, out_vals, out_idx, nullptr, true, stream);
}

int rtopk_rowwise_eps(const float* in, int64_t N, int32_t M, int32_t k, float eps_rel, float* out_vals,
                      int32_t* out_idx, int32_t* out_iters, void* stream) {
  return run(in, N, M, k, 0, eps_rel, rtopk::kEps, out_vals, out_idx, out_iters, false, stream);
}

int rtopk_rowwise_smallest(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out_vals,
                           int32_t* out_idx, void* stream) {
  return run(in, N, M, k, max_iter, 0.0f, rtopk::kEarly, out_vals, out_idx, nullptr, false, stream, true);
}

int rtopk_rowwise_exact_smallest(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, int32_t* out_idx,
                                 void* stream) {
  return run(in, N, M, k, 0, 0.0f, rtopk::kExact, out_vals, out_idx, nullptr, false, stream, true);
}

int rtopk_rowwise_f16(const uint16_t* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, uint16_t* out_vals,
                      int32_t* out_idx, void* stream) {
  return run(in, N, M, k, max_iter, 0.0f, rtopk::kEarly, out_vals, out_idx, nullptr, false, stream, false, rtopk::kF16);
}

int rtopk_rowwise_exact_f16(const uint16_t* in, int64_t N, int32_t M, int32_t k, uint16_t* out_vals, int32_t* out_idx,
                            void* stream) {
  return run(in, N, M, k, 0, 0.0f, rtopk::kExact, out_vals, out_idx, nullptr, false, stream, false, rtopk::kF16);
}

int rtopk_rowwise_bf16(const uint16_t* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, uint16_t* out_vals,
                       int32_t* out_idx, void* stream) {
  return run(in, N, M, k, max_iter, 0.0f, rtopk::kEarly, out_vals, out_idx, nullptr, false, stream, false,
             rtopk::kBF16);
}

int rtopk_rowwise_exact_bf16(const uint16_t* in, int64_t N, int32_t M, int32_t k, uint16_t* out_vals,
                             int32_t* out_idx, void* stream) {
  return run(in, N, M, k, 0, 0.0f, rtopk::kExact, out_vals, out_idx, nullptr, false, stream, false, rtopk::kBF16);
}

int rtopk_maxk_dense(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out, void* stream) {
  if (N < 0 || M < 1 || k < 1 || k > M) return RTOPK_ERR_BAD_SHAPE;
  if (M > kMaxM) return RTOPK_ERR_M_TOO_LARGE;
  if (N == 0) return RTOPK_OK;
  if (!in || !out) return RTOPK_ERR_NULL_POINTER;
  if (!aligned(in, 4) || !aligned(out, 4)) return RTOPK_ERR_MISALIGNED;
  int mode = max_iter < 0 ? rtopk::kExact : rtopk::kEarly;
  if (mode == rtopk::kExact && k == M) {  // everything is kept: no search needed
    mode = rtopk::kEarly;
    max_iter = 0;
  }
  rtopk::LaunchArgs a{};
  a.in = in;
  a.N = N;
  a.M = M;
  a.k = k;
  a.max_iter = max_iter < 0 ? 0 : max_iter;
  a.out_vals = out;
  a.stream = static_cast<hipStream_t>(stream);
  int g = 1, ng = 1;
  if (M > kMaxWaveM) {
    if (N > 0x7fffffffLL) return RTOPK_ERR_BAD_SHAPE;  // one workgroup per row
    int w = 16;
    ng = 16;
    if (M % 4 == 0 && aligned(in, 16) && aligned(out, 16)) {
      g = 4;
      w = M <= 16384 ? 4 : (M <= 32768 ? 8 : 16);
    } else {
      while (1024 * ng < M) ng <<= 1;
    }
    const hipError_t e = rtopk::launch_block_dense(g, ng, w, mode, a);
    return e == hipSuccess ? RTOPK_OK : RTOPK_ERR_LAUNCH;
  }
  if (M > 128 && M % 4 == 0 && aligned(in, 16) && aligned(out, 16)) {
    static const int kNg[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32};
    g = 4;
    ng = 32;
    for (int cand : kNg) {
      if (M <= 256 * cand) {
        ng = cand;
        break;
      }
    }
  } else if (M > 64 && M <= 128 && M % 2 == 0 && aligned(in, 8) && aligned(out, 8)) {
    g = 2;
  } else {
    while (64 * ng < M) ng <<= 1;
  }
  const hipError_t err = rtopk::launch_dense_any(g, ng, M == 64 * g * ng, mode, a);
  return err == hipSuccess ? RTOPK_OK : RTOPK_ERR_LAUNCH;
}

const char* rtopk_status_string(int status) {
  switch (status) {
    case RTOPK_OK: return "ok";
    case RTOPK_ERR_NULL_POINTER: return "null data pointer with N > 0";
    case RTOPK_ERR_BAD_SHAPE: return "bad shape: need N >= 0 and 1 <= k <= M";
    case RTOPK_ERR_BAD_MAX_ITER: return "max_iter must be >= 0";
    case RTOPK_ERR_M_TOO_LARGE: return "M exceeds the supported row width (65536; 256 for uint8 columns)";
    case RTOPK_ERR_MISALIGNED: return "pointer not aligned to its element size";
    case RTOPK_ERR_LAUNCH: return "the HIP runtime refused the launch";
    case RTOPK_ERR_BAD_EPSILON: return "eps_rel must be >= 0";
    default: return "unknown status";
  }
}

int rtopk_version(void) { return kVersion; }

int rtopk_max_m(void) { return kMaxM; }

}  // extern "C"
