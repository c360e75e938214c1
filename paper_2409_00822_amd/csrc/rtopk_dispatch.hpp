// Host-side dispatch table between the C ABI (rtopk_api.hip) and the kernel instantiations, which
// are spread over several translation units so that they compile in parallel.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rtopk_shape.hpp"

namespace rtopk {

struct LaunchArgs {
  const void* in;
  int64_t N;
  int M, k, max_iter;
  float eps_rel;       // kEps only
  int32_t* out_iters;  // kEps only, may be null
  bool smallest;       // select the k smallest instead of the k largest (kEarly / kExact, int32 columns)
  void* out_vals;
  void* out_idx;
  int vec_store;  // 1: k % 4 == 0 and both outputs aligned for 128-bit (values) / whole-word (columns) stores
  hipStream_t stream;
};

// Vector-load paths: M % G == 0 and `in` aligned to 4*G bytes.  ng = groups per lane (M <= 64*G*ng).
// full = (M == 64*G*ng): no column-validity tests in the kernel.
hipError_t launch_g4_exact(int ng, bool full, bool u8, const LaunchArgs& a);
hipError_t launch_g4_early(int ng, bool full, bool u8, const LaunchArgs& a);
hipError_t launch_g4_eps(int ng, bool full, const LaunchArgs& a);  // int32 columns only
// Rows stored in 16 bits (dtype kF16 or kBF16; kEarly / kExact, int32 columns).  g = elements per load
// (8, 4, 2 or 1: M % g == 0 and `in` aligned to 2*g bytes), ng = loads per lane (M <= 64*g*ng).
hipError_t launch_h16_exact(int dtype, int g, int ng, bool full, const LaunchArgs& a);
hipError_t launch_h16_early(int dtype, int g, int ng, bool full, const LaunchArgs& a);
// Rows wider than 8192 columns: one workgroup of w wavefronts per row (int32 columns).  g = elements per
// load (4 for fp32 / 8 for 16-bit rows: M % g == 0 and 16-byte aligned pointers; else 1), ng = loads per
// lane, M <= 64*w*g*ng.
hipError_t launch_block_plain(int g, int ng, int w, int mode, const LaunchArgs& a);                   // fp32, kEarly / kExact
hipError_t launch_block_variant(int g, int ng, int w, int mode, bool smallest, const LaunchArgs& a);  // fp32: kEps, or the k smallest
hipError_t launch_block_dense(int g, int ng, int w, int mode, const LaunchArgs& a);                   // fp32 dense output
hipError_t launch_block_h16(int dtype, int g, int ng, int w, int mode, const LaunchArgs& a);          // half / bfloat16 rows
// Rows wider than 65536 columns (fp32, int32 columns, every mode, the k largest or smallest): one
// workgroup per row, the row streamed.  g = 4 (M % 4 == 0 and 16-byte aligned input) or 1.
hipError_t launch_stream_any(int g, int mode, bool smallest, const LaunchArgs& a);
// Dense-output form (fp32; a.out_vals is the [N][M] output, a.out_idx unused).  g, ng, full as above;
// mode kEarly or kExact.
hipError_t launch_dense_any(int g, int ng, bool full, int mode, const LaunchArgs& a);
// Narrow rows and scalar-load fallback (any M, 4-byte alignment).
hipError_t launch_small(int g, int ng, bool full, int mode, bool u8, const LaunchArgs& a);


// Backward edge of the MaxK non-linearity (rtopk_backward.hpp).  idx is int32_t[N][k] or, with u8,
// uint8_t[N][k]; vec = M % 4 == 0 and the dense [N][M] array 16-byte aligned (128-bit accesses).
hipError_t launch_maxk_backward(const float* grad_vals, const void* idx, bool u8, int64_t N, int M, int k, float* grad_in,
                                bool vec, hipStream_t stream);
hipError_t launch_maxk_backward_gather(const float* grad_out, const void* idx, bool u8, int64_t N, int M, int k,
                                       float* grad_vals, bool vec, hipStream_t stream);

}  // namespace rtopk
