// Instantiations: one workgroup of W wavefronts per row, for rows wider than 8192 columns -- fp32 pairs, Algorithm 2 and exact mode.
#include "rtopk_block_kernel.hpp"

namespace rtopk {

// 128-bit loads: W = 4 up to 16384 columns, 8 up to 32768, 16 up to 65536, with 12 or 16 loads per lane.
// Scalar-load fallback (M % 4 != 0 or unaligned input): W = 16 with 16, 32 or 64 loads per lane.
template <int G, int NG, int W>
static hipError_t pick(int mode, const LaunchArgs& a) {
  if (mode == kExact) return launch_block<G, NG, W, kExact>(a);
  if (mode == kEarly) return launch_block<G, NG, W, kEarly>(a);
  return hipErrorInvalidValue;
}

hipError_t launch_block_plain(int g, int ng, int w, int mode, const LaunchArgs& a) {
  if (g == 4) {
    if (w == 4 && ng == 12) return pick<4, 12, 4>(mode, a);
    if (w == 4 && ng == 16) return pick<4, 16, 4>(mode, a);
    if (w == 8 && ng == 12) return pick<4, 12, 8>(mode, a);
    if (w == 8 && ng == 16) return pick<4, 16, 8>(mode, a);
    if (w == 16 && ng == 12) return pick<4, 12, 16>(mode, a);
    if (w == 16 && ng == 16) return pick<4, 16, 16>(mode, a);
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
