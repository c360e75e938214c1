// Instantiations: 128-bit-load path (G = 4), Algorithm 1 with a relative precision epsilon'.
#include "rtopk_kernel.hpp"

namespace rtopk {

template <int NG>
static hipError_t pick(bool full, const LaunchArgs& a) {
  constexpr int R = rows_per_wave(4 * NG);
  return full ? launch<4, NG, R, true, kEps, int32_t>(a) : launch<4, NG, R, false, kEps, int32_t>(a);
}

hipError_t launch_g4_eps(int ng, bool full, const LaunchArgs& a) {
  switch (ng) {
    case 1: return pick<1>(full, a);
    case 2: return pick<2>(full, a);
    case 3: return pick<3>(full, a);
    case 4: return pick<4>(full, a);
    case 6: return pick<6>(full, a);
    case 8: return pick<8>(full, a);
    case 12: return pick<12>(full, a);
    case 16: return pick<16>(full, a);
    case 24: return pick<24>(full, a);
    case 32: return pick<32>(full, a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
