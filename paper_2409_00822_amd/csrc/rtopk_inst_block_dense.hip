// Instantiations: one workgroup of W wavefronts per row, for rows wider than 8192 columns -- fp32 dense output.
#include "rtopk_block_kernel.hpp"

namespace rtopk {

template <int G, int NG, int W>
static hipError_t pick(int mode, const LaunchArgs& a) {
  if (mode == kExact) return launch_block<G, NG, W, kExact, false, kF32, true>(a);
  if (mode == kEarly) return launch_block<G, NG, W, kEarly, false, kF32, true>(a);
  return hipErrorInvalidValue;
}

hipError_t launch_block_dense(int g, int ng, int w, int mode, const LaunchArgs& a) {
  if (g == 4) {
    if (ng != 16) return hipErrorInvalidValue;
    if (w == 4) return pick<4, 16, 4>(mode, a);
    if (w == 8) return pick<4, 16, 8>(mode, a);
    if (w == 16) return pick<4, 16, 16>(mode, a);
    return hipErrorInvalidValue;
  }
  if (g != 1 || w != 16) return hipErrorInvalidValue;
  switch (ng) {
#define X(n) case n: return pick<1, n, 16>(mode, a);
    RTOPK_NG_LIST_BLOCK_G1(X)
#undef X
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
