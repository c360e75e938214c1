// Instantiations: dense-output form of the selection (chosen values in place, zero elsewhere), fp32.
#include "rtopk_kernel.hpp"

namespace rtopk {

template <int G, int NG>
static hipError_t pick(bool full, int mode, const LaunchArgs& a) {
  constexpr int R = rows_per_wave(G * NG);
  if (mode == kExact) return full ? launch_dense<G, NG, R, true, kExact>(a) : launch_dense<G, NG, R, false, kExact>(a);
  if (mode == kEarly) return full ? launch_dense<G, NG, R, true, kEarly>(a) : launch_dense<G, NG, R, false, kEarly>(a);
  return hipErrorInvalidValue;
}

hipError_t launch_dense_any(int g, int ng, bool full, int mode, const LaunchArgs& a) {
  if (g == 4) {
    switch (ng) {
      case 1: return pick<4, 1>(full, mode, a);
      case 2: return pick<4, 2>(full, mode, a);
      case 3: return pick<4, 3>(full, mode, a);
      case 4: return pick<4, 4>(full, mode, a);
      case 6: return pick<4, 6>(full, mode, a);
      case 8: return pick<4, 8>(full, mode, a);
      case 12: return pick<4, 12>(full, mode, a);
      case 16: return pick<4, 16>(full, mode, a);
      case 24: return pick<4, 24>(full, mode, a);
      case 32: return pick<4, 32>(full, mode, a);
      default: return hipErrorInvalidValue;
    }
  }
  if (g == 2 && ng == 1) return pick<2, 1>(full, mode, a);
  if (g != 1) return hipErrorInvalidValue;
  switch (ng) {
    case 1: return pick<1, 1>(full, mode, a);
    case 2: return pick<1, 2>(full, mode, a);
    case 4: return pick<1, 4>(full, mode, a);
    case 8: return pick<1, 8>(full, mode, a);
    case 16: return pick<1, 16>(full, mode, a);
    case 32: return pick<1, 32>(full, mode, a);
    case 64: return pick<1, 64>(full, mode, a);
    case 128: return pick<1, 128>(full, mode, a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
