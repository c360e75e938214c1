// Instantiations: 128-bit-load path (G = 4), exact mode.
#include "rtopk_kernel.hpp"

namespace rtopk {

template <int NG>
static hipError_t pick(bool full, bool u8, const LaunchArgs& a) {
  constexpr int R = rows_per_wave(4 * NG);
  if constexpr (NG == 1) {
    if (u8 && !a.smallest) return full ? launch<4, NG, R, true, kExact, uint8_t>(a) : launch<4, NG, R, false, kExact, uint8_t>(a);
  }
  if (a.smallest) {
    if (u8) return hipErrorInvalidValue;
    return full ? launch<4, NG, R, true, kExact, int32_t, true>(a) : launch<4, NG, R, false, kExact, int32_t, true>(a);
  }
  if constexpr (R > kRowsPerWaveFew) {
    if (a.N < kFewRows) {
      return full ? launch<4, NG, kRowsPerWaveFew, true, kExact, int32_t>(a)
                  : launch<4, NG, kRowsPerWaveFew, false, kExact, int32_t>(a);
    }
  }
  return full ? launch<4, NG, R, true, kExact, int32_t>(a) : launch<4, NG, R, false, kExact, int32_t>(a);
}

hipError_t launch_g4_exact(int ng, bool full, bool u8, const LaunchArgs& a) {
  switch (ng) {
    case 1: return pick<1>(full, u8, a);
    case 2: return pick<2>(full, u8, a);
    case 3: return pick<3>(full, u8, a);
    case 4: return pick<4>(full, u8, a);
    case 6: return pick<6>(full, u8, a);
    case 8: return pick<8>(full, u8, a);
    case 12: return pick<12>(full, u8, a);
    case 16: return pick<16>(full, u8, a);
    case 24: return pick<24>(full, u8, a);
    case 32: return pick<32>(full, u8, a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
