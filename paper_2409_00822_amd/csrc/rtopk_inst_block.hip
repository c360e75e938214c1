// Instantiations: one workgroup of 16 wavefronts per row, for rows wider than 8192 columns.
#include "rtopk_block_kernel.hpp"

namespace rtopk {

template <int G, int NG>
static hipError_t pick(int mode, const LaunchArgs& a) {
  if (mode == kExact) return launch_block<G, NG, 16, kExact>(a);
  if (mode == kEarly) return launch_block<G, NG, 16, kEarly>(a);
  return hipErrorInvalidValue;
}

hipError_t launch_block_any(int g, int ng, int mode, const LaunchArgs& a) {
  if (g == 4) {
    switch (ng) {
      case 3: return pick<4, 3>(mode, a);
      case 4: return pick<4, 4>(mode, a);
      case 6: return pick<4, 6>(mode, a);
      case 8: return pick<4, 8>(mode, a);
      case 12: return pick<4, 12>(mode, a);
      case 16: return pick<4, 16>(mode, a);
      default: return hipErrorInvalidValue;
    }
  }
  if (g != 1) return hipErrorInvalidValue;
  switch (ng) {
    case 16: return pick<1, 16>(mode, a);
    case 32: return pick<1, 32>(mode, a);
    case 64: return pick<1, 64>(mode, a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
