// Instantiations: rows stored as IEEE half or bfloat16, exact mode, int32 columns.
#include "rtopk_kernel.hpp"

namespace rtopk {

template <int DT, int G, int NG>
static hipError_t pick(bool full, const LaunchArgs& a) {
  constexpr int R = rows_per_wave(G * NG);
  return full ? launch<G, NG, R, true, kExact, int32_t, false, DT>(a) : launch<G, NG, R, false, kExact, int32_t, false, DT>(a);
}

template <int DT>
static hipError_t pick_shape(int g, int ng, bool full, const LaunchArgs& a) {
  if (g == 8) {
    switch (ng) {
      case 1: return pick<DT, 8, 1>(full, a);
      case 2: return pick<DT, 8, 2>(full, a);
      case 3: return pick<DT, 8, 3>(full, a);
      case 4: return pick<DT, 8, 4>(full, a);
      case 6: return pick<DT, 8, 6>(full, a);
      case 8: return pick<DT, 8, 8>(full, a);
      case 12: return pick<DT, 8, 12>(full, a);
      case 16: return pick<DT, 8, 16>(full, a);
      default: return hipErrorInvalidValue;
    }
  }
  if (g == 4 && ng == 1) return pick<DT, 4, 1>(full, a);
  if (g == 2 && ng == 1) return pick<DT, 2, 1>(full, a);
  if (g != 1) return hipErrorInvalidValue;
  switch (ng) {
    case 1: return pick<DT, 1, 1>(full, a);
    case 2: return pick<DT, 1, 2>(full, a);
    case 4: return pick<DT, 1, 4>(full, a);
    case 8: return pick<DT, 1, 8>(full, a);
    case 16: return pick<DT, 1, 16>(full, a);
    case 32: return pick<DT, 1, 32>(full, a);
    case 64: return pick<DT, 1, 64>(full, a);
    case 128: return pick<DT, 1, 128>(full, a);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_h16_exact(int dtype, int g, int ng, bool full, const LaunchArgs& a) {
  if (dtype == kF16) return pick_shape<kF16>(g, ng, full, a);
  if (dtype == kBF16) return pick_shape<kBF16>(g, ng, full, a);
  return hipErrorInvalidValue;
}

}  // namespace rtopk
