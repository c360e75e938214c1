// Instantiations: backward edge of the MaxK non-linearity (scatter and gather forms, int32 and uint8 columns).
#include "rtopk_backward.hpp"

namespace rtopk {

hipError_t launch_maxk_backward(const float* grad_vals, const void* idx, bool u8, int64_t N, int M, int k, float* grad_in,
                                bool vec, hipStream_t stream) {
  if (u8) {
    const uint8_t* ix = static_cast<const uint8_t*>(idx);
    return vec ? launch_scatter<uint8_t, true>(grad_vals, ix, N, M, k, grad_in, stream)
               : launch_scatter<uint8_t, false>(grad_vals, ix, N, M, k, grad_in, stream);
  }
  const int32_t* ix = static_cast<const int32_t*>(idx);
  return vec ? launch_scatter<int32_t, true>(grad_vals, ix, N, M, k, grad_in, stream)
             : launch_scatter<int32_t, false>(grad_vals, ix, N, M, k, grad_in, stream);
}

hipError_t launch_maxk_backward_gather(const float* grad_out, const void* idx, bool u8, int64_t N, int M, int k,
                                       float* grad_vals, bool vec, hipStream_t stream) {
  if (u8) {
    const uint8_t* ix = static_cast<const uint8_t*>(idx);
    return vec ? launch_gather<uint8_t, true>(grad_out, ix, N, M, k, grad_vals, stream)
               : launch_gather<uint8_t, false>(grad_out, ix, N, M, k, grad_vals, stream);
  }
  const int32_t* ix = static_cast<const int32_t*>(idx);
  return vec ? launch_gather<int32_t, true>(grad_out, ix, N, M, k, grad_vals, stream)
             : launch_gather<int32_t, false>(grad_out, ix, N, M, k, grad_vals, stream);
}

}  // namespace rtopk
