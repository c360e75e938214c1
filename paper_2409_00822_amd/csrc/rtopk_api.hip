// C ABI of the row-wise top-k library: argument checks, shape classification, launch.
// Declarations and the full contract are in include/rtopk.h.
#include "rtopk.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rtopk_dispatch.hpp"

namespace {

constexpr int kVersion = 700;  // 0.7.0

inline uintptr_t addr(const void* p) { return reinterpret_cast<uintptr_t>(p); }
inline bool aligned(const void* p, uintptr_t a) { return rtopk::is_aligned(addr(p), a); }

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
  if (M > (dtype == rtopk::kF32 ? rtopk::kMaxM : rtopk::kMaxBlockM) || (u8 && M > 256)) return RTOPK_ERR_M_TOO_LARGE;
  if (M > rtopk::kMaxWaveM && N > 0x7fffffffLL) return RTOPK_ERR_BAD_SHAPE;  // one workgroup per row: 2^31 - 1 rows
  if (N == 0) return RTOPK_OK;
  if (!in || !out_vals || !out_idx) return RTOPK_ERR_NULL_POINTER;
  if (!aligned(in, esz) || !aligned(out_vals, esz) || (!u8 && !aligned(out_idx, 4)) || !aligned(out_iters, 4))
    return RTOPK_ERR_MISALIGNED;
  {
    // the input must not share a byte with any output, nor the outputs with one another
    const uint64_t n_in = (uint64_t)N * (uint64_t)M * esz, n_v = (uint64_t)N * (uint64_t)k * esz;
    const uint64_t n_i = (uint64_t)N * (uint64_t)k * (u8 ? 1 : 4), n_t = out_iters ? (uint64_t)N * 4 : 0;
    const uintptr_t p[4] = {addr(in), addr(out_vals), addr(out_idx), addr(out_iters)};
    const uint64_t n[4] = {n_in, n_v, n_i, n_t};
    for (int i = 0; i < 4; ++i)
      for (int j = i + 1; j < 4; ++j)
        if (rtopk::ranges_overlap(p[i], n[i], p[j], n[j])) return RTOPK_ERR_OVERLAP;
  }

  // k == M: every column is selected.  Algorithm 2 with zero steps returns the first k columns,
  // which is that answer without a search that would otherwise run down to float resolution.
  if (mode == rtopk::kExact && k == M) {
    mode = rtopk::kEarly;
    max_iter = 0;
  }
  // steps beyond the clamp cannot change the result (see kMaxIterClamp)
  if (max_iter > rtopk::kMaxIterClamp) max_iter = rtopk::kMaxIterClamp;

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

  const bool plain = dtype == rtopk::kF32 && !smallest && mode != rtopk::kEps;
  const rtopk::Shape sh = rtopk::classify(M, dtype, plain, addr(in));
  hipError_t err;
  switch (sh.family) {
    case rtopk::kFamStream:
      err = rtopk::launch_stream_any(sh.g, mode, smallest, a);
      break;
    case rtopk::kFamBlock:
      err = dtype != rtopk::kF32 ? rtopk::launch_block_h16(dtype, sh.g, sh.ng, sh.w, mode, a)
            : plain              ? rtopk::launch_block_plain(sh.g, sh.ng, sh.w, mode, a)
                                 : rtopk::launch_block_variant(sh.g, sh.ng, sh.w, mode, smallest, a);
      break;
    case rtopk::kFamH16:
      err = mode == rtopk::kExact ? rtopk::launch_h16_exact(dtype, sh.g, sh.ng, sh.full, a)
                                  : rtopk::launch_h16_early(dtype, sh.g, sh.ng, sh.full, a);
      break;
    case rtopk::kFamG4:
      err = mode == rtopk::kExact   ? rtopk::launch_g4_exact(sh.ng, sh.full, u8, a)
            : mode == rtopk::kEarly ? rtopk::launch_g4_early(sh.ng, sh.full, u8, a)
                                    : rtopk::launch_g4_eps(sh.ng, sh.full, a);
      break;
    default:
      err = rtopk::launch_small(sh.g, sh.ng, sh.full, mode, u8, a);
      break;
  }
  return err == hipSuccess ? RTOPK_OK : RTOPK_ERR_LAUNCH;
}

// Shared body of the backward entry points.  dense = the [N][M] array (output of the scatter, input of
// the gather), pairs = the [N][k] gradient array (input of the scatter, output of the gather).
int run_backward(bool gather, const float* dense, const float* pairs, const void* idx, bool u8, int64_t N, int32_t M,
                 int32_t k, void* stream) {
  if (N < 0 || M < 1 || k < 1 || k > M) return RTOPK_ERR_BAD_SHAPE;
  if (M > rtopk::kMaxBlockM || (u8 && M > 256)) return RTOPK_ERR_M_TOO_LARGE;
  if (M > rtopk::kBackwardRowsM && N > 0x7fffffffLL) return RTOPK_ERR_BAD_SHAPE;  // one workgroup per row
  if (N == 0) return RTOPK_OK;
  if (!dense || !pairs || !idx) return RTOPK_ERR_NULL_POINTER;
  if (!aligned(dense, 4) || !aligned(pairs, 4) || (!u8 && !aligned(idx, 4))) return RTOPK_ERR_MISALIGNED;
  const uint64_t n_d = (uint64_t)N * (uint64_t)M * 4, n_p = (uint64_t)N * (uint64_t)k * 4;
  const uint64_t n_i = (uint64_t)N * (uint64_t)k * (u8 ? 1 : 4);
  if (rtopk::ranges_overlap(addr(dense), n_d, addr(pairs), n_p) || rtopk::ranges_overlap(addr(dense), n_d, addr(idx), n_i) ||
      (gather && rtopk::ranges_overlap(addr(pairs), n_p, addr(idx), n_i)))
    return RTOPK_ERR_OVERLAP;
  const bool vec = M % 4 == 0 && aligned(dense, 16);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const hipError_t err = gather ? rtopk::launch_maxk_backward_gather(dense, idx, u8, N, M, k, const_cast<float*>(pairs), vec, s)
                                : rtopk::launch_maxk_backward(pairs, idx, u8, N, M, k, const_cast<float*>(dense), vec, s);
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
  if (M > rtopk::kMaxBlockM) return RTOPK_ERR_M_TOO_LARGE;
  if (M > rtopk::kMaxWaveM && N > 0x7fffffffLL) return RTOPK_ERR_BAD_SHAPE;  // one workgroup per row
  if (N == 0) return RTOPK_OK;
  if (!in || !out) return RTOPK_ERR_NULL_POINTER;
  if (!aligned(in, 4) || !aligned(out, 4)) return RTOPK_ERR_MISALIGNED;
  const uint64_t bytes = (uint64_t)N * (uint64_t)M * 4;
  if (rtopk::ranges_overlap(addr(in), bytes, addr(out), bytes)) return RTOPK_ERR_OVERLAP;
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
  a.max_iter = max_iter < 0 ? 0 : (max_iter > rtopk::kMaxIterClamp ? rtopk::kMaxIterClamp : max_iter);
  a.out_vals = out;
  a.stream = static_cast<hipStream_t>(stream);
  const rtopk::Shape sh = rtopk::classify_dense(M, addr(in), addr(out));
  hipError_t err;
  if (sh.family == rtopk::kFamBlock) {
    err = rtopk::launch_block_dense(sh.g, sh.ng, sh.w, mode, a);
  } else {
    err = rtopk::launch_dense_any(sh.g, sh.ng, sh.full, mode, a);
  }
  return err == hipSuccess ? RTOPK_OK : RTOPK_ERR_LAUNCH;
}

int rtopk_maxk_backward(const float* grad_vals, const int32_t* idx, int64_t N, int32_t M, int32_t k, float* grad_in,
                        void* stream) {
  return run_backward(false, grad_in, grad_vals, idx, false, N, M, k, stream);
}

int rtopk_maxk_backward_u8(const float* grad_vals, const uint8_t* idx, int64_t N, int32_t M, int32_t k, float* grad_in,
                           void* stream) {
  return run_backward(false, grad_in, grad_vals, idx, true, N, M, k, stream);
}

int rtopk_maxk_backward_gather(const float* grad_out, const int32_t* idx, int64_t N, int32_t M, int32_t k,
                               float* grad_vals, void* stream) {
  return run_backward(true, grad_out, grad_vals, idx, false, N, M, k, stream);
}

int rtopk_maxk_backward_gather_u8(const float* grad_out, const uint8_t* idx, int64_t N, int32_t M, int32_t k,
                                  float* grad_vals, void* stream) {
  return run_backward(true, grad_out, grad_vals, idx, true, N, M, k, stream);
}

const char* rtopk_status_string(int status) {
  switch (status) {
    case RTOPK_OK: return "ok";
    case RTOPK_ERR_NULL_POINTER: return "null data pointer with N > 0";
    case RTOPK_ERR_BAD_SHAPE: return "bad shape: need N >= 0 and 1 <= k <= M";
    case RTOPK_ERR_BAD_MAX_ITER: return "max_iter must be >= 0";
    case RTOPK_ERR_M_TOO_LARGE:
      return "M exceeds the supported row width (2^24 for fp32 rows with int32 columns; 65536 for 16-bit rows, the dense "
             "form and the backward edge; 256 for uint8 columns)";
    case RTOPK_ERR_MISALIGNED: return "pointer not aligned to its element size";
    case RTOPK_ERR_LAUNCH: return "the HIP runtime refused the launch";
    case RTOPK_ERR_BAD_EPSILON: return "eps_rel must be >= 0";
    case RTOPK_ERR_OVERLAP: return "input and output buffers overlap";
    default: return "unknown status";
  }
}

int rtopk_version(void) { return kVersion; }

int rtopk_max_m(void) { return rtopk::kMaxM; }

}  // extern "C"
