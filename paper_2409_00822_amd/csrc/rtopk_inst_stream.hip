// Instantiations: rows wider than 65536 columns, streamed (fp32 rows, int32 columns).
#include "rtopk_stream_kernel.hpp"

namespace rtopk {

template <int G>
static hipError_t pick(int mode, bool smallest, const LaunchArgs& a) {
  if (smallest) {
    if (mode == kExact) return launch_stream<G, kExact, true>(a);
    if (mode == kEarly) return launch_stream<G, kEarly, true>(a);
    return hipErrorInvalidValue;
  }
  if (mode == kExact) return launch_stream<G, kExact, false>(a);
  if (mode == kEarly) return launch_stream<G, kEarly, false>(a);
  if (mode == kEps) return launch_stream<G, kEps, false>(a);
  return hipErrorInvalidValue;
}

hipError_t launch_stream_any(int g, int mode, bool smallest, const LaunchArgs& a) {
  if (g == 4) return pick<4>(mode, smallest, a);
  if (g == 1) return pick<1>(mode, smallest, a);
  return hipErrorInvalidValue;
}

}  // namespace rtopk
