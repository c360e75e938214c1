// Instantiations: 64-bit-load path for even M <= 128 (G = 2) and the scalar-load fallback (G = 1)
// that serves every other shape (odd M, or `in` not 16-byte aligned).
#include "rtopk_kernel.hpp"

namespace rtopk {

// R rows per wavefront; the column type and the k-smallest variant are picked here.
template <int G, int NG, int R, int MODE>
static hipError_t pick_rows(bool full, bool u8, const LaunchArgs& a) {
  if constexpr (64 * G * NG <= 256 && MODE != kEps) {
    if (u8 && !a.smallest) return full ? launch<G, NG, R, true, MODE, uint8_t>(a) : launch<G, NG, R, false, MODE, uint8_t>(a);
  }
  if constexpr (MODE != kEps) {
    if (a.smallest) {
      if (u8) return hipErrorInvalidValue;
      return full ? launch<G, NG, R, true, MODE, int32_t, true>(a) : launch<G, NG, R, false, MODE, int32_t, true>(a);
    }
  }
  return full ? launch<G, NG, R, true, MODE, int32_t>(a) : launch<G, NG, R, false, MODE, int32_t>(a);
}

template <int G, int NG, int MODE>
static hipError_t pick(bool full, bool u8, const LaunchArgs& a) {
  constexpr int R = rows_per_wave(G * NG);
  if constexpr (R > kRowsPerWaveFew && G == 2) {
    if (a.N < kFewRows) return pick_rows<G, NG, kRowsPerWaveFew, MODE>(full, u8, a);
  }
  return pick_rows<G, NG, R, MODE>(full, u8, a);
}

template <int MODE>
static hipError_t pick_mode(int g, int ng, bool full, bool u8, const LaunchArgs& a) {
  if (g == 2 && ng == 1) return pick<2, 1, MODE>(full, u8, a);
  if (g != 1) return hipErrorInvalidValue;
  switch (ng) {
#define X(n) case n: return pick<1, n, MODE>(full, u8, a);
    RTOPK_NG_LIST_G1(X)
#undef X
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
