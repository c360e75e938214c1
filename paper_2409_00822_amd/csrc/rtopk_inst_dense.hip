// Instantiations: dense-output form of the selection (chosen values in place, zero elsewhere), fp32.
#include "rtopk_kernel.hpp"

namespace rtopk {

template <int G, int NG, int R>
static hipError_t pick_rows(bool full, int mode, const LaunchArgs& a) {
  if (mode == kExact) return full ? launch_dense<G, NG, R, true, kExact>(a) : launch_dense<G, NG, R, false, kExact>(a);
  if (mode == kEarly) return full ? launch_dense<G, NG, R, true, kEarly>(a) : launch_dense<G, NG, R, false, kEarly>(a);
  return hipErrorInvalidValue;
}

template <int G, int NG>
static hipError_t pick(bool full, int mode, const LaunchArgs& a) {
  constexpr int R = (G == 4 && NG == 1) ? kRowsPerWaveFp32M256 : rows_per_wave(G * NG);
  if constexpr (R > kRowsPerWaveFew && G > 1) {
    if (a.N < kFewRows) return pick_rows<G, NG, kRowsPerWaveFew>(full, mode, a);
  }
  return pick_rows<G, NG, R>(full, mode, a);
}

hipError_t launch_dense_any(int g, int ng, bool full, int mode, const LaunchArgs& a) {
  if (g == 4) {
    switch (ng) {
#define X(n) case n: return pick<4, n>(full, mode, a);
      RTOPK_NG_LIST_G4(X)
#undef X
      default: return hipErrorInvalidValue;
    }
  }
  if (g == 2 && ng == 1) return pick<2, 1>(full, mode, a);
  if (g != 1) return hipErrorInvalidValue;
  switch (ng) {
#define X(n) case n: return pick<1, n>(full, mode, a);
    RTOPK_NG_LIST_G1(X)
#undef X
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rtopk
