// C ABI of the row-wise top-k library: argument checks, shape classification, launch.
// Declarations and the full contract are in include/rtopk.h.
#include "rtopk.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rtopk_dispatch.hpp"

namespace {

constexpr int kMaxM = 4096;
constexpr int kVersion = 100;  // 0.1.0

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Shared body of the four selection entry points.
//   exact: Algorithm 1 at epsilon = 0; otherwise Algorithm 2 with max_iter steps.
//   u8:    out_idx is uint8_t[N][k] (requires M <= 256), else int32_t[N][k].
int run(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, bool exact, float* out_vals,
        void* out_idx, bool u8, void* stream) {
  if (N < 0 || M < 1 || k < 1 || k > M) return RTOPK_ERR_BAD_SHAPE;
  if (!exact && max_iter < 0) return RTOPK_ERR_BAD_MAX_ITER;
  if (M > kMaxM || (u8 && M > 256)) return RTOPK_ERR_M_TOO_LARGE;
  if (N == 0) return RTOPK_OK;
  if (!in || !out_vals || !out_idx) return RTOPK_ERR_NULL_POINTER;
  if (!aligned(in, 4) || !aligned(out_vals, 4) || (!u8 && !aligned(out_idx, 4))) return RTOPK_ERR_MISALIGNED;

  // k == M: every column is selected.  Algorithm 2 with zero steps returns the first k columns,
  // which is that answer without a search that would otherwise run down to float resolution.
  if (exact && k == M) {
    exact = false;
    max_iter = 0;
  }

  rtopk::LaunchArgs a;
  a.in = in;
  a.N = N;
  a.M = M;
  a.k = k;
  a.max_iter = max_iter;
  a.out_vals = out_vals;
  a.out_idx = out_idx;
  a.vec_store = (k % 4 == 0) && aligned(out_vals, 16) && aligned(out_idx, u8 ? 4 : 16);
  a.stream = static_cast<hipStream_t>(stream);

  hipError_t err;
  if (M > 128 && M % 4 == 0 && aligned(in, 16)) {
    // 128-bit loads; groups per lane rounded up to an instantiated count
    static const int kNg[] = {1, 2, 3, 4, 6, 8, 12, 16};
    int ng = 16;
    for (int cand : kNg) {
      if (M <= 256 * cand) {
        ng = cand;
        break;
      }
    }
    const bool full = (M == 256 * ng);
    err = exact ? rtopk::launch_g4_exact(ng, full, u8, a) : rtopk::launch_g4_early(ng, full, u8, a);
  } else if (M > 64 && M <= 128 && M % 2 == 0 && aligned(in, 8)) {
    err = rtopk::launch_small(2, 1, M == 128, exact, u8, a);
  } else {
    int ng = 1;
    while (64 * ng < M) ng <<= 1;
    err = rtopk::launch_small(1, ng, M == 64 * ng, exact, u8, a);
  }
  return err == hipSuccess ? RTOPK_OK : RTOPK_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int rtopk_rowwise(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out_vals,
                  int32_t* out_idx, void* stream) {
  return run(in, N, M, k, max_iter, false, out_vals, out_idx, false, stream);
}

int rtopk_rowwise_exact(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, int32_t* out_idx,
                        void* stream) {
  return run(in, N, M, k, 0, true, out_vals, out_idx, false, stream);
}

int rtopk_rowwise_u8(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out_vals,
                     uint8_t* out_idx, void* stream) {
  return run(in, N, M, k, max_iter, false, out_vals, out_idx, true, stream);
}

int rtopk_rowwise_exact_u8(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, uint8_t* out_idx,
                           void* stream) {
  return run(in, N, M, k, 0, true, out_vals, out_idx, true, stream);
}

const char* rtopk_status_string(int status) {
  switch (status) {
    case RTOPK_OK: return "ok";
    case RTOPK_ERR_NULL_POINTER: return "null data pointer with N > 0";
    case RTOPK_ERR_BAD_SHAPE: return "bad shape: need N >= 0 and 1 <= k <= M";
    case RTOPK_ERR_BAD_MAX_ITER: return "max_iter must be >= 0";
    case RTOPK_ERR_M_TOO_LARGE: return "M exceeds the supported row width (4096; 256 for uint8 columns)";
    case RTOPK_ERR_MISALIGNED: return "pointer not aligned to its element size";
    case RTOPK_ERR_LAUNCH: return "the HIP runtime refused the launch";
    case RTOPK_ERR_BAD_EPSILON: return "eps_rel must be >= 0";
    default: return "unknown status";
  }
}

int rtopk_version(void) { return kVersion; }

int rtopk_max_m(void) { return kMaxM; }

}  // extern "C"
