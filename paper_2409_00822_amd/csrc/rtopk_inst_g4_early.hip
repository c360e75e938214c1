// Instantiations: 128-bit-load path (G = 4), early mode.
#include "rtopk_kernel.hpp"

namespace rtopk {

// R rows per wavefront; the column type and the k-smallest variant are picked here.
template <int NG, int R>
static hipError_t pick_rows(bool full, bool u8, const LaunchArgs& a) {
  if constexpr (NG == 1) {
    if (u8 && !a.smallest) return full ? launch<4, NG, R, true, kEarly, uint8_t>(a) : launch<4, NG, R, false, kEarly, uint8_t>(a);
  }
  if (a.smallest) {
    if (u8) return hipErrorInvalidValue;
    return full ? launch<4, NG, R, true, kEarly, int32_t, true>(a) : launch<4, NG, R, false, kEarly, int32_t, true>(a);
  }
  return full ? launch<4, NG, R, true, kEarly, int32_t>(a) : launch<4, NG, R, false, kEarly, int32_t>(a);
}

template <int NG>
static hipError_t pick(bool full, bool u8, const LaunchArgs& a) {
  constexpr int R = rows_per_wave(4 * NG);
  if constexpr (R > kRowsPerWaveFew) {
    if (a.N < kFewRows) return pick_rows<NG, kRowsPerWaveFew>(full, u8, a);  // every variant, not only int32 columns
  }
  if constexpr (NG == 1) {
    if (!u8) return pick_rows<NG, kRowsPerWaveFp32M256>(full, u8, a);
  }
  return pick_rows<NG, R>(full, u8, a);
}

hipError_t launch_g4_early(int ng, bool full, bool u8, const LaunchArgs& a) {
  switch (ng) {
#define X(n) case n: return pick<n>(full, u8, a);
    RTOPK_NG_LIST_G4(X)
#undef X
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
