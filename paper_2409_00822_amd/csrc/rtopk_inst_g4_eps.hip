// Instantiations: 128-bit-load path (G = 4), Algorithm 1 with a relative precision epsilon'.
#include "rtopk_kernel.hpp"

namespace rtopk {

template <int NG>
static hipError_t pick(bool full, const LaunchArgs& a) {
  constexpr int R = NG == 1 ? kRowsPerWaveFp32M256 : rows_per_wave(4 * NG);
  if constexpr (R > kRowsPerWaveFew) {
    if (a.N < kFewRows) {
      return full ? launch<4, NG, kRowsPerWaveFew, true, kEps, int32_t>(a)
                  : launch<4, NG, kRowsPerWaveFew, false, kEps, int32_t>(a);
    }
  }
  return full ? launch<4, NG, R, true, kEps, int32_t>(a) : launch<4, NG, R, false, kEps, int32_t>(a);
}

hipError_t launch_g4_eps(int ng, bool full, const LaunchArgs& a) {
  switch (ng) {
#define X(n) case n: return pick<n>(full, a);
    RTOPK_NG_LIST_G4(X)
#undef X
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
