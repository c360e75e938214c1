// Instantiations: one workgroup of W wavefronts per row, for rows wider than 8192 columns -- rows stored as half or bfloat16.
#include "rtopk_block_kernel.hpp"

namespace rtopk {

// 128-bit loads bring 8 values; 8 loads per lane (W = 4, 8 or 16), or the scalar-load fallback (W = 16).
template <int G, int NG, int W, int DT>
static hipError_t pick(int mode, const LaunchArgs& a) {
  if (mode == kExact) return launch_block<G, NG, W, kExact, false, DT>(a);
  if (mode == kEarly) return launch_block<G, NG, W, kEarly, false, DT>(a);
  return hipErrorInvalidValue;
}

template <int DT>
static hipError_t pick_shape(int g, int ng, int w, int mode, const LaunchArgs& a) {
  if (g == 8) {
    if (ng != 8) return hipErrorInvalidValue;
    if (w == 4) return pick<8, 8, 4, DT>(mode, a);
    if (w == 8) return pick<8, 8, 8, DT>(mode, a);
    if (w == 16) return pick<8, 8, 16, DT>(mode, a);
    return hipErrorInvalidValue;
  }
  if (g != 1 || w != 16) return hipErrorInvalidValue;
  switch (ng) {
#define X(n) case n: return pick<1, n, 16, DT>(mode, a);
    RTOPK_NG_LIST_BLOCK_G1(X)
#undef X
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_block_h16(int dtype, int g, int ng, int w, int mode, const LaunchArgs& a) {
  if (dtype == kF16) return pick_shape<kF16>(g, ng, w, mode, a);
  if (dtype == kBF16) return pick_shape<kBF16>(g, ng, w, mode, a);
  return hipErrorInvalidValue;
}

}  // namespace rtopk
