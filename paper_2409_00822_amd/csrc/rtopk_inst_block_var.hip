// Instantiations: one workgroup of W wavefronts per row, for rows wider than 8192 columns -- fp32 pairs: precision-bounded mode and the k smallest.
#include "rtopk_block_kernel.hpp"

namespace rtopk {

// 128-bit loads with 16 loads per lane (W = 4, 8 or 16), or the scalar-load fallback (W = 16).
template <int G, int NG, int W>
static hipError_t pick(int mode, bool smallest, const LaunchArgs& a) {
  if (smallest) {
    if (mode == kExact) return launch_block<G, NG, W, kExact, true>(a);
    if (mode == kEarly) return launch_block<G, NG, W, kEarly, true>(a);
    return hipErrorInvalidValue;
  }
  if (mode == kEps) return launch_block<G, NG, W, kEps>(a);
  return hipErrorInvalidValue;
}

hipError_t launch_block_variant(int g, int ng, int w, int mode, bool smallest, const LaunchArgs& a) {
  if (g == 4) {
    if (ng != 16) return hipErrorInvalidValue;
    if (w == 4) return pick<4, 16, 4>(mode, smallest, a);
    if (w == 8) return pick<4, 16, 8>(mode, smallest, a);
    if (w == 16) return pick<4, 16, 16>(mode, smallest, a);
    return hipErrorInvalidValue;
  }
  if (g != 1 || w != 16) return hipErrorInvalidValue;
  switch (ng) {
#define X(n) case n: return pick<1, n, 16>(mode, smallest, a);
    RTOPK_NG_LIST_BLOCK_G1(X)
#undef X
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
