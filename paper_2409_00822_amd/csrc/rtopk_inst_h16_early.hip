// Instantiations: rows stored as IEEE half or bfloat16, early mode, int32 columns.
#include "rtopk_kernel.hpp"

namespace rtopk {

template <int DT, int G, int NG>
static hipError_t pick(bool full, const LaunchArgs& a) {
  constexpr int R = rows_per_wave(G * NG);
  if constexpr (R > kRowsPerWaveFew && G > 1) {
    if (a.N < kFewRows) {
      return full ? launch<G, NG, kRowsPerWaveFew, true, kEarly, int32_t, false, DT>(a)
                  : launch<G, NG, kRowsPerWaveFew, false, kEarly, int32_t, false, DT>(a);
    }
  }
  return full ? launch<G, NG, R, true, kEarly, int32_t, false, DT>(a) : launch<G, NG, R, false, kEarly, int32_t, false, DT>(a);
}

template <int DT>
static hipError_t pick_shape(int g, int ng, bool full, const LaunchArgs& a) {
  if (g == 8) {
    switch (ng) {
#define X(n) case n: return pick<DT, 8, n>(full, a);
      RTOPK_NG_LIST_H8(X)
#undef X
      default: return hipErrorInvalidValue;
    }
  }
  if (g == 4 && ng == 1) return pick<DT, 4, 1>(full, a);
  if (g == 2 && ng == 1) return pick<DT, 2, 1>(full, a);
  if (g != 1) return hipErrorInvalidValue;
  switch (ng) {
#define X(n) case n: return pick<DT, 1, n>(full, a);
    RTOPK_NG_LIST_G1(X)
#undef X
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_h16_early(int dtype, int g, int ng, bool full, const LaunchArgs& a) {
  if (dtype == kF16) return pick_shape<kF16>(g, ng, full, a);
  if (dtype == kBF16) return pick_shape<kBF16>(g, ng, full, a);
  return hipErrorInvalidValue;
}

}  // namespace rtopk
