// Instantiations: 64-bit-load path for even M <= 128 (G = 2) and the scalar-load fallback (G = 1)
// that serves every other shape (odd M, or `in` not 16-byte aligned).
#include "rtopk_kernel.hpp"

namespace rtopk {

template <int G, int NG, int MODE>
static hipError_t pick(bool full, bool u8, const LaunchArgs& a) {
  constexpr int R = rows_per_wave(G * NG);
  if constexpr (64 * G * NG <= 256 && MODE != kEps) {
    if (u8 && !a.smallest) return full ? launch<G, NG, R, true, MODE, uint8_t>(a) : launch<G, NG, R, false, MODE, uint8_t>(a);
  }
  if constexpr (MODE != kEps) {
    if (a.smallest) {
      if (u8) return hipErrorInvalidValue;
      return full ? launch<G, NG, R, true, MODE, int32_t, true>(a) : launch<G, NG, R, false, MODE, int32_t, true>(a);
    }
  }
  if constexpr (R > kRowsPerWaveFew && G == 2) {
    if (a.N < kFewRows) {
      return full ? launch<G, NG, kRowsPerWaveFew, true, MODE, int32_t>(a)
                  : launch<G, NG, kRowsPerWaveFew, false, MODE, int32_t>(a);
    }
  }
  return full ? launch<G, NG, R, true, MODE, int32_t>(a) : launch<G, NG, R, false, MODE, int32_t>(a);
}

template <int MODE>
static hipError_t pick_mode(int g, int ng, bool full, bool u8, const LaunchArgs& a) {
  if (g == 2 && ng == 1) return pick<2, 1, MODE>(full, u8, a);
  if (g != 1) return hipErrorInvalidValue;
  switch (ng) {
    case 1: return pick<1, 1, MODE>(full, u8, a);
    case 2: return pick<1, 2, MODE>(full, u8, a);
    case 4: return pick<1, 4, MODE>(full, u8, a);
    case 8: return pick<1, 8, MODE>(full, u8, a);
    case 16: return pick<1, 16, MODE>(full, u8, a);
    case 32: return pick<1, 32, MODE>(full, u8, a);
    case 64: return pick<1, 64, MODE>(full, u8, a);
    case 128: return pick<1, 128, MODE>(full, u8, a);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_small(int g, int ng, bool full, int mode, bool u8, const LaunchArgs& a) {
  switch (mode) {
    case kEarly: return pick_mode<kEarly>(g, ng, full, u8, a);
    case kExact: return pick_mode<kExact>(g, ng, full, u8, a);
    case kEps: return u8 ? hipErrorInvalidValue : pick_mode<kEps>(g, ng, full, false, a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
