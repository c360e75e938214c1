// Instantiations: 64-bit-load path for even M <= 128 (G = 2) and the scalar-load fallback (G = 1)
// that serves every other shape (odd M, or `in` not 16-byte aligned).
#include "rtopk_kernel.hpp"

namespace rtopk {

template <int G, int NG, bool EXACT>
static hipError_t pick(bool full, bool u8, const LaunchArgs& a) {
  constexpr int R = rows_per_wave(G * NG);
  if constexpr (64 * G * NG <= 256) {
    if (u8) return full ? launch<G, NG, R, true, EXACT, uint8_t>(a) : launch<G, NG, R, false, EXACT, uint8_t>(a);
  }
  return full ? launch<G, NG, R, true, EXACT, int32_t>(a) : launch<G, NG, R, false, EXACT, int32_t>(a);
}

template <bool EXACT>
static hipError_t pick_mode(int g, int ng, bool full, bool u8, const LaunchArgs& a) {
  if (g == 2 && ng == 1) return pick<2, 1, EXACT>(full, u8, a);
  if (g != 1) return hipErrorInvalidValue;
  switch (ng) {
    case 1: return pick<1, 1, EXACT>(full, u8, a);
    case 2: return pick<1, 2, EXACT>(full, u8, a);
    case 4: return pick<1, 4, EXACT>(full, u8, a);
    case 8: return pick<1, 8, EXACT>(full, u8, a);
    case 16: return pick<1, 16, EXACT>(full, u8, a);
    case 32: return pick<1, 32, EXACT>(full, u8, a);
    case 64: return pick<1, 64, EXACT>(full, u8, a);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_small(int g, int ng, bool full, bool exact, bool u8, const LaunchArgs& a) {
  return exact ? pick_mode<true>(g, ng, full, u8, a) : pick_mode<false>(g, ng, full, u8, a);
}

}  // namespace rtopk
