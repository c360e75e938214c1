// Backward edge of the MaxK non-linearity for gfx950 (MI355X).
//
// RTop-K (arXiv 2409.00822) is used as the non-linearity of a MaxK-GNN layer (Section 1 / Fig. 1;
// Section 4.3 measures it inside training): forward, a row keeps its k selected entries and every other
// entry becomes zero, so the derivative with respect to the row is that same 0/1 mask.  With the k
// columns saved by the forward pass (rtopk_rowwise*: idx[N][k]) the backward step is pure data movement:
//
//   scatter:  grad_in[r][c]  = grad_vals[r][j] if c == idx[r][j] for some j, else 0      ([N][k] -> [N][M])
//   gather:   grad_vals[r][j] = grad_out[r][idx[r][j]]                                     ([N][M] -> [N][k])
//
// Both are bound by HBM bandwidth; the kernels below exist to keep every global access coalesced.
// A column outside [0, M) is ignored by the scatter and yields 0 in the gather, so a corrupt index
// cannot make either kernel touch memory outside its buffers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rtopk_kernel.hpp"

namespace rtopk {

// How the lanes of a wavefront are laid over (row, j) pairs of an [rows][k] array: when k <= 32, 64 >> kshift
// rows share one instruction (lane = sub_row * 2^kshift + j); otherwise one row at a time, j strided by 64.
struct PairLanes {
  int kshift;  // log2 of the lanes given to one row (6 when k > 32)
};
inline PairLanes pair_lanes(int k) {
  int s = 0;
  while ((1 << s) < k && s < 6) ++s;
  return PairLanes{s};
}

// ---- scatter, narrow rows: one wavefront per R rows, rows assembled in LDS ------------------------------
//
// The wavefront's R rows are contiguous in grad_in (R * M floats).  They are built in LDS -- zero fill,
// then one 4-byte LDS write per saved column -- and leave as whole 128-bit stores (VEC) that cover the R
// rows back to back, so HBM sees each output byte written once, in order.  The LDS queue of a wavefront
// is served in order, so the three phases need no barrier.
template <typename IdxT, int R, bool VEC>
__global__ void __launch_bounds__(256)
    maxk_scatter_rows_kernel(const float* __restrict__ grad_vals, const IdxT* __restrict__ idx, int64_t N, int M, int k,
                             int kshift, float* __restrict__ grad_in) {
  extern __shared__ __attribute__((aligned(16))) float s_rows[];  // [waves per block][R * M]
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int waves_per_block = (int)(blockDim.x >> 6);
  const int64_t r0 = ((int64_t)blockIdx.x * waves_per_block + wave) * R;
  if (r0 >= N) return;
  const int nrows = (N - r0 < R) ? (int)(N - r0) : R;
  float* rows = s_rows + (size_t)wave * R * M;
  const int total = nrows * M;

  // the saved columns and their gradients: issued first, consumed after the zero fill
  const int lanes_per_row = 1 << kshift;
  const int rows_per_step = kWave >> kshift;
  const int sub = lane >> kshift, j0 = lane & (lanes_per_row - 1);
  // (row, j) pairs of step s: rows s * rows_per_step + sub; R steps cover the R rows even at one row a step
  float g[R];
  int c[R];
  const bool one_pass = k <= lanes_per_row;  // every (row, j) of a step has a lane of its own
  if (one_pass) {
#pragma unroll
    for (int s = 0; s < R; ++s) {
      c[s] = -1;
      g[s] = 0.0f;
      if (s * rows_per_step < nrows) {  // uniform over the wavefront
        const int rr = s * rows_per_step + sub;
        const bool live = rr < nrows && j0 < k;
        const int64_t e = (r0 + (live ? rr : 0)) * (int64_t)k + (live ? j0 : 0);
        g[s] = __builtin_nontemporal_load(grad_vals + e);
        c[s] = live ? (int)__builtin_nontemporal_load(idx + e) : -1;
      }
    }
  }

  if constexpr (VEC) {
    float4* rows4 = reinterpret_cast<float4*>(rows);
    for (int q = lane; q < (total >> 2); q += kWave) rows4[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  } else {
    for (int q = lane; q < total; q += kWave) rows[q] = 0.0f;
  }

  if (one_pass) {
#pragma unroll
    for (int s = 0; s < R; ++s) {
      const int rr = s * rows_per_step + sub;
      if ((unsigned)c[s] < (unsigned)M) rows[rr * M + c[s]] = g[s];
    }
  } else {
    for (int rr = 0; rr < nrows; ++rr) {
      for (int j = lane; j < k; j += kWave) {
        const int64_t e = (r0 + rr) * (int64_t)k + j;
        const int col = (int)idx[e];
        if ((unsigned)col < (unsigned)M) rows[rr * M + col] = grad_vals[e];
      }
    }
  }

  float* out = grad_in + r0 * (int64_t)M;
  if constexpr (VEC) {
    const uint4* rows4 = reinterpret_cast<const uint4*>(rows);
#pragma unroll 1
    for (int q = lane; q < (total >> 2); q += kWave) store_streaming(reinterpret_cast<uint4*>(out) + q, rows4[q]);
  } else {
#pragma unroll 1
    for (int q = lane; q < total; q += kWave) out[q] = rows[q];
  }
}

// ---- scatter, wide rows: one workgroup per row, the row assembled in LDS chunk by chunk -----------------
constexpr int kScatterChunk = 8192;  // columns per chunk (32 KiB of LDS)

template <typename IdxT, bool VEC>
__global__ void __launch_bounds__(256)
    maxk_scatter_block_kernel(const float* __restrict__ grad_vals, const IdxT* __restrict__ idx, int64_t N, int M, int k,
                              float* __restrict__ grad_in) {
  __shared__ __attribute__((aligned(16))) float s_chunk[kScatterChunk];
  const int64_t r = blockIdx.x;
  if (r >= N) return;
  const float* gv = grad_vals + r * (int64_t)k;
  const IdxT* ix = idx + r * (int64_t)k;
  float* out = grad_in + r * (int64_t)M;
  for (int c0 = 0; c0 < M; c0 += kScatterChunk) {
    const int width = M - c0 < kScatterChunk ? M - c0 : kScatterChunk;
    for (int q = threadIdx.x; q < width; q += blockDim.x) s_chunk[q] = 0.0f;
    __syncthreads();
    for (int j = threadIdx.x; j < k; j += blockDim.x) {
      const int col = (int)ix[j] - c0;
      if ((unsigned)col < (unsigned)width) s_chunk[col] = gv[j];
    }
    __syncthreads();
    if constexpr (VEC) {  // M % 4 == 0, so every chunk width is a multiple of 4
      const uint4* c4 = reinterpret_cast<const uint4*>(s_chunk);
      for (int q = threadIdx.x; q < (width >> 2); q += blockDim.x)
        store_streaming(reinterpret_cast<uint4*>(out + c0) + q, c4[q]);
    } else {
      for (int q = threadIdx.x; q < width; q += blockDim.x) out[c0 + q] = s_chunk[q];
    }
    __syncthreads();  // the chunk buffer is zeroed again by the next round
  }
}

// ---- gather: the dense gradient row is read once, through LDS, with 128-bit loads ------------------------
//
// One wavefront per R rows.  The R rows (contiguous: R * M floats) are copied to LDS with whole
// 128-bit loads, the k saved columns of each row are then read from LDS, and the R * k results -- again
// contiguous in the output -- are stored coalesced.
template <typename IdxT, int R, bool VEC>
__global__ void __launch_bounds__(256)
    maxk_gather_rows_kernel(const float* __restrict__ grad_out, const IdxT* __restrict__ idx, int64_t N, int M, int k,
                            int kshift, float* __restrict__ grad_vals) {
  extern __shared__ __attribute__((aligned(16))) float s_rows[];  // [waves per block][R * M]
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int waves_per_block = (int)(blockDim.x >> 6);
  const int64_t r0 = ((int64_t)blockIdx.x * waves_per_block + wave) * R;
  if (r0 >= N) return;
  const int nrows = (N - r0 < R) ? (int)(N - r0) : R;
  float* rows = s_rows + (size_t)wave * R * M;
  const int total = nrows * M;
  const float* src = grad_out + r0 * (int64_t)M;

  if constexpr (VEC) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4* src4 = reinterpret_cast<const f4*>(src);
    f4* rows4 = reinterpret_cast<f4*>(rows);
#pragma unroll 4
    for (int q = lane; q < (total >> 2); q += kWave) rows4[q] = __builtin_nontemporal_load(src4 + q);
  } else {
    for (int q = lane; q < total; q += kWave) rows[q] = __builtin_nontemporal_load(src + q);
  }

  const int lanes_per_row = 1 << kshift;
  const int rows_per_step = kWave >> kshift;
  const int sub = lane >> kshift, j0 = lane & (lanes_per_row - 1);
  for (int rr0 = 0; rr0 < nrows; rr0 += rows_per_step) {
    const int rr = rr0 + sub;
    if (rr < nrows) {
      for (int j = j0; j < k; j += lanes_per_row) {
        const int64_t e = (r0 + rr) * (int64_t)k + j;
        const int col = (int)__builtin_nontemporal_load(idx + e);
        grad_vals[e] = (unsigned)col < (unsigned)M ? rows[rr * M + col] : 0.0f;
      }
    }
  }
}

// ---- gather, wide rows: the saved columns are read straight from memory ---------------------------------
// (k scattered 4-byte reads per row; for k << M this touches far less than the whole row.)
template <typename IdxT>
__global__ void __launch_bounds__(256)
    maxk_gather_block_kernel(const float* __restrict__ grad_out, const IdxT* __restrict__ idx, int64_t N, int M, int k,
                             float* __restrict__ grad_vals) {
  const int64_t r = blockIdx.x;
  if (r >= N) return;
  const float* row = grad_out + r * (int64_t)M;
  for (int j = threadIdx.x; j < k; j += blockDim.x) {
    const int col = (int)idx[r * (int64_t)k + j];
    grad_vals[r * (int64_t)k + j] = (unsigned)col < (unsigned)M ? row[col] : 0.0f;
  }
}

// ---- host side --------------------------------------------------------------------------------------------


// rows per wavefront of the rows-in-LDS kernels: about 8 KiB of LDS per wavefront
inline int backward_rows_per_wave(int M) { return M <= 128 ? 16 : (M <= 256 ? 8 : (M <= 512 ? 4 : (M <= 1024 ? 2 : 1))); }

template <typename IdxT, bool VEC>
hipError_t launch_scatter(const float* gv, const IdxT* idx, int64_t N, int M, int k, float* gin, hipStream_t stream) {
  if (M > kBackwardRowsM) {
    if (N > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    return launch_kernel(maxk_scatter_block_kernel<IdxT, VEC>, dim3((unsigned)N), dim3(256), 0, stream, gv, idx, N, M, k,
                         gin);
  }
  const int R = backward_rows_per_wave(M);
  const int kshift = pair_lanes(k).kshift;
  const int64_t blocks = (N + R - 1) / R;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  const size_t lds = (size_t)R * M * sizeof(float);
  switch (R) {
    case 16: return launch_kernel(maxk_scatter_rows_kernel<IdxT, 16, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gv, idx, N, M, k, kshift, gin);
    case 8: return launch_kernel(maxk_scatter_rows_kernel<IdxT, 8, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gv, idx, N, M, k, kshift, gin);
    case 4: return launch_kernel(maxk_scatter_rows_kernel<IdxT, 4, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gv, idx, N, M, k, kshift, gin);
    case 2: return launch_kernel(maxk_scatter_rows_kernel<IdxT, 2, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gv, idx, N, M, k, kshift, gin);
    default: return launch_kernel(maxk_scatter_rows_kernel<IdxT, 1, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gv, idx, N, M, k, kshift, gin);
  }
}

template <typename IdxT, bool VEC>
hipError_t launch_gather(const float* gout, const IdxT* idx, int64_t N, int M, int k, float* gv, hipStream_t stream) {
  if (M > kBackwardRowsM) {
    if (N > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    return launch_kernel(maxk_gather_block_kernel<IdxT>, dim3((unsigned)N), dim3(256), 0, stream, gout, idx, N, M, k, gv);
  }
  const int R = backward_rows_per_wave(M);
  const int kshift = pair_lanes(k).kshift;
  const int64_t blocks = (N + R - 1) / R;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  const size_t lds = (size_t)R * M * sizeof(float);
  switch (R) {
    case 16: return launch_kernel(maxk_gather_rows_kernel<IdxT, 16, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gout, idx, N, M, k, kshift, gv);
    case 8: return launch_kernel(maxk_gather_rows_kernel<IdxT, 8, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gout, idx, N, M, k, kshift, gv);
    case 4: return launch_kernel(maxk_gather_rows_kernel<IdxT, 4, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gout, idx, N, M, k, kshift, gv);
    case 2: return launch_kernel(maxk_gather_rows_kernel<IdxT, 2, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gout, idx, N, M, k, kshift, gv);
    default: return launch_kernel(maxk_gather_rows_kernel<IdxT, 1, VEC>, dim3((unsigned)blocks), dim3(kWave), lds, stream, gout, idx, N, M, k, kshift, gv);
  }
}

}  // namespace rtopk
