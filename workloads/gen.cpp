// Seeded synthetic input generator for the row-wise top-k workloads.
//
// This file is test/benchmark infrastructure shared by the CPU oracle's tests
// and the GPU path's tests.  It holds no selection arithmetic: it only fills
// N x M fp32 matrices.  Every value is a pure function of (seed, flat index),
// so any sub-block of a matrix can be regenerated without the rest.
//
// Distributions mirror the paper's workloads: i.i.d. normal rows (Section 3.1,
// Tables 1, 2 and 5 use normally distributed vectors), MaxK-GNN hidden-feature
// shaped matrices (Section 4.3: N = #nodes, M = 256), and the wide-row sweep of
// Appendix B.
//
// Build: g++ -O2 -fopenmp -shared -fPIC gen.cpp -o libworkloads.so

#include <cmath>
#include <cstdint>

namespace {

// splitmix64 finaliser: a bijective 64-bit mixer used as a counter-based RNG.
inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Independent 64-bit word for (seed, stream, counter).
inline uint64_t word(uint64_t seed, uint64_t stream, uint64_t ctr) {
  return mix64(mix64(seed * 0xD1342543DE82EF95ull + stream) ^ (ctr * 0x2545F4914F6CDD1Dull + stream));
}

// Uniform double in the open interval (0, 1), 53 random bits.
inline double u01(uint64_t w) { return ((double)(w >> 11) + 0.5) * (1.0 / 9007199254740992.0); }

inline double std_normal(uint64_t seed, uint64_t idx) {
  const double u1 = u01(word(seed, 1, idx));
  const double u2 = u01(word(seed, 2, idx));
  return std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586476925 * u2);
}

}  // namespace

extern "C" {

// out[r*M + c] = s_r * z, z ~ N(0,1); s_r = 1 when row_scale == 0, else
// s_r ~ U(scale_lo, scale_hi) drawn once per row.
int wl_fill_normal(float* out, int64_t N, int32_t M, uint64_t seed, int32_t row_scale, double scale_lo,
                   double scale_hi) {
  if (!out || N < 0 || M < 1) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < N; ++r) {
    double s = 1.0;
    if (row_scale) s = scale_lo + (scale_hi - scale_lo) * u01(word(seed, 3, (uint64_t)r));
    for (int32_t c = 0; c < M; ++c) {
      const uint64_t idx = (uint64_t)r * (uint64_t)M + (uint64_t)c;
      out[idx] = (float)(s * std_normal(seed, idx));
    }
  }
  return 0;
}

// out ~ U(lo, hi)
int wl_fill_uniform(float* out, int64_t N, int32_t M, uint64_t seed, double lo, double hi) {
  if (!out || N < 0 || M < 1) return -1;
  const int64_t total = N * (int64_t)M;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < total; ++i) out[i] = (float)(lo + (hi - lo) * u01(word(seed, 1, (uint64_t)i)));
  return 0;
}

// out ~ Laplace(0, 1) by inverse CDF.
int wl_fill_laplace(float* out, int64_t N, int32_t M, uint64_t seed) {
  if (!out || N < 0 || M < 1) return -1;
  const int64_t total = N * (int64_t)M;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < total; ++i) {
    const double u = u01(word(seed, 1, (uint64_t)i)) - 0.5;
    const double a = std::fabs(u);
    const double x = -std::log(1.0 - 2.0 * a);
    out[i] = (float)(u < 0 ? -x : x);
  }
  return 0;
}

// N(0,1) entries; each entry independently, with probability p, is replaced by
// the nearest of `levels` shared values level0 + step*j.  Forces exact ties
// within and across rows.
int wl_fill_normal_ties(float* out, int64_t N, int32_t M, uint64_t seed, double p, int32_t levels, double level0,
                        double step) {
  if (!out || N < 0 || M < 1 || levels < 1) return -1;
  const int64_t total = N * (int64_t)M;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < total; ++i) {
    double z = std_normal(seed, (uint64_t)i);
    if (u01(word(seed, 4, (uint64_t)i)) < p) {
      double j = std::nearbyint((z - level0) / step);
      if (j < 0) j = 0;
      if (j > levels - 1) j = levels - 1;
      z = level0 + step * j;
    }
    out[i] = (float)z;
  }
  return 0;
}

}  // extern "C"
