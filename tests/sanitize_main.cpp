// CPU-only sanitizer target (built and run by tests/test_sanitize_cpu.py with
// -fsanitize=address,undefined): the oracle, the input generator and the library's host-side shape
// classification, exercised in one process so that any out-of-bounds access, use of an uninitialised
// index, signed overflow or misaligned access in them aborts the test.
//
//   1. the Algorithm 2 hand traces of tests/golden/alg2_handtrace.txt against the sanitized oracle;
//   2. brute force (a stable sort written out here) against the oracle's exact mode, Algorithm 1 at
//      epsilon = 0 and the k-smallest variant on tiny tie-heavy rows from the sanitized generator;
//   3. the shape classification for every row width 1..65536 (and a sample of the streamed widths up to
//      2^24), every element type, both kernel variants and a set of pointer alignments: the layout
//      returned must be compiled and must hold the row.
//
// Usage: sanitize_main <path to alg2_handtrace.txt>.  Exit code 0 = all checks passed.
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <fstream>
#include <sstream>
#include <string>
#include <vector>

#include "rtopk_shape.hpp"

extern "C" {
int oracle_topk_exact(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, int32_t* out_idx);
int oracle_topk_earlystop(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out_vals,
                          int32_t* out_idx);
int oracle_alg1(const float* in, int64_t N, int32_t M, int32_t k, float eps_rel, int32_t collect, float* out_vals,
                int32_t* out_idx, int32_t* out_iters);
int oracle_topk_exact_smallest(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, int32_t* out_idx);
int oracle_maxk_backward(const float* grad_vals, const int32_t* idx, int64_t N, int32_t M, int32_t k, float* grad_in);
int wl_fill_normal_ties(float* out, int64_t N, int32_t M, uint64_t seed, double p, int32_t levels, double level0,
                        double step);
int wl_fill_normal(float* out, int64_t N, int32_t M, uint64_t seed, int32_t row_scale, double scale_lo,
                   double scale_hi);
}

static int g_failures = 0;
#define CHECK(cond, ...)                          \
  do {                                            \
    if (!(cond)) {                                \
      std::fprintf(stderr, "FAIL %s:%d: ", __FILE__, __LINE__); \
      std::fprintf(stderr, __VA_ARGS__);          \
      std::fprintf(stderr, "\n");                 \
      if (++g_failures > 20) std::exit(1);        \
    }                                             \
  } while (0)

// ---- 1. hand traces -------------------------------------------------------------------------------
static int run_hand_traces(const char* path) {
  std::ifstream f(path);
  if (!f) {
    std::fprintf(stderr, "cannot open %s\n", path);
    return -1;
  }
  std::string line;
  int cases = 0;
  while (std::getline(f, line)) {
    if (line.empty() || line[0] == '#') continue;
    std::vector<std::string> part;
    std::stringstream ss(line);
    std::string item;
    while (std::getline(ss, item, '|')) part.push_back(item);
    CHECK(part.size() == 4, "malformed line: %s", line.c_str());
    if (part.size() != 4) continue;
    std::vector<float> v;
    {
      std::stringstream s0(part[0]);
      float x;
      while (s0 >> x) v.push_back(x);
    }
    const int k = std::atoi(part[1].c_str()), mi = std::atoi(part[2].c_str());
    std::vector<int32_t> want;
    {
      std::stringstream s3(part[3]);
      int x;
      while (s3 >> x) want.push_back(x);
    }
    CHECK((int)want.size() == k, "k does not match the expected columns: %s", line.c_str());
    std::vector<float> ov((size_t)k);
    std::vector<int32_t> oi((size_t)k);
    const int rc = oracle_topk_earlystop(v.data(), 1, (int32_t)v.size(), k, mi, ov.data(), oi.data());
    CHECK(rc == 0, "oracle_topk_earlystop rc %d", rc);
    CHECK(oi == want, "hand trace differs: %s", line.c_str());
    for (int j = 0; j < k; ++j) CHECK(ov[(size_t)j] == v[(size_t)oi[(size_t)j]], "value is not a copy of the input");
    ++cases;
  }
  return cases;
}

// ---- 2. brute force ---------------------------------------------------------------------------------
// The plain definition: order columns by value descending (ascending for the k smallest), ties by column
// ascending; take the first k; report them in ascending column order.
static std::vector<int32_t> brute(const float* v, int M, int k, bool smallest) {
  std::vector<int32_t> order((size_t)M);
  for (int i = 0; i < M; ++i) order[(size_t)i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
    return smallest ? v[a] < v[b] : v[a] > v[b];
  });
  order.resize((size_t)k);
  std::sort(order.begin(), order.end());
  return order;
}

static int run_brute_force() {
  int rows_checked = 0;
  for (int M : {1, 2, 3, 5, 8, 12, 17, 33}) {
    const int N = 200;
    std::vector<float> x((size_t)N * M);
    // half of the entries snapped to three shared levels: ties within every row
    CHECK(wl_fill_normal_ties(x.data(), N, M, 900 + (uint64_t)M, 0.5, 3, -0.5, 0.5) == 0, "generator failed");
    for (int i = 0; i < N * M; i += 7) x[(size_t)i] = (i % 14 == 0) ? -0.0f : 0.0f;  // signed zeros
    for (int k = 1; k <= M; ++k) {
      std::vector<float> ov((size_t)N * k), av((size_t)N * k), sv((size_t)N * k);
      std::vector<int32_t> oi((size_t)N * k), ai((size_t)N * k), si((size_t)N * k), it((size_t)N);
      CHECK(oracle_topk_exact(x.data(), N, M, k, ov.data(), oi.data()) == 0, "exact rc");
      CHECK(oracle_alg1(x.data(), N, M, k, 0.0f, 1, av.data(), ai.data(), it.data()) == 0, "alg1 rc");
      CHECK(oracle_topk_exact_smallest(x.data(), N, M, k, sv.data(), si.data()) == 0, "smallest rc");
      for (int r = 0; r < N; ++r) {
        const float* row = x.data() + (size_t)r * M;
        const std::vector<int32_t> want = brute(row, M, k, false), want_s = brute(row, M, k, true);
        for (int j = 0; j < k; ++j) {
          const size_t o = (size_t)r * k + j;
          CHECK(oi[o] == want[(size_t)j], "exact: M=%d k=%d row %d", M, k, r);
          CHECK(ai[o] == want[(size_t)j], "alg1 eps=0: M=%d k=%d row %d", M, k, r);
          CHECK(si[o] == want_s[(size_t)j], "smallest: M=%d k=%d row %d", M, k, r);
          CHECK(ov[o] == row[oi[o]] && av[o] == row[ai[o]] && sv[o] == row[si[o]], "values are not copies");
        }
        ++rows_checked;
      }
    }
  }
  // the backward edge: gradients scattered to the saved columns, zero elsewhere
  {
    const int N = 50, M = 37, k = 9;
    std::vector<float> x((size_t)N * M), g((size_t)N * k), v((size_t)N * k), gin((size_t)N * M);
    std::vector<int32_t> idx((size_t)N * k);
    CHECK(wl_fill_normal(x.data(), N, M, 77, 0, 0, 0) == 0 && wl_fill_normal(g.data(), N, k, 78, 0, 0, 0) == 0, "generator");
    CHECK(oracle_topk_exact(x.data(), N, M, k, v.data(), idx.data()) == 0, "exact rc");
    CHECK(oracle_maxk_backward(g.data(), idx.data(), N, M, k, gin.data()) == 0, "backward rc");
    for (int r = 0; r < N; ++r) {
      std::vector<float> want((size_t)M, 0.0f);
      for (int j = 0; j < k; ++j) want[(size_t)idx[(size_t)r * k + j]] = g[(size_t)r * k + j];
      for (int c = 0; c < M; ++c) CHECK(gin[(size_t)r * M + c] == want[(size_t)c], "backward scatter row %d col %d", r, c);
    }
  }
  return rows_checked;
}

// ---- 3. shape classification ---------------------------------------------------------------------
static long run_shape_sweep() {
  long n = 0;
  const uintptr_t base = 0x7f0000000000ull;  // never dereferenced: only its alignment is looked at
  const uintptr_t offs[] = {0, 2, 4, 6, 8, 12, 16, 20, 24, 32};
  for (int M = 1; M <= rtopk::kMaxBlockM; ++M) {
    for (int dtype : {rtopk::kF32, rtopk::kF16, rtopk::kBF16}) {
      const uintptr_t esz = dtype == rtopk::kF32 ? 4 : 2;
      for (uintptr_t off : offs) {
        if (off % esz) continue;  // the entry points reject pointers not aligned to the element size
        for (int plain = 0; plain <= (dtype == rtopk::kF32 ? 1 : 0); ++plain) {
          const rtopk::Shape s = rtopk::classify(M, dtype, plain != 0, base + off);
          CHECK(rtopk::instantiated(s, dtype, plain != 0, false), "M=%d dtype=%d off=%d plain=%d: (%d,%d,%d) family %d not compiled",
                M, dtype, (int)off, plain, s.g, s.ng, s.w, s.family);
          CHECK(s.capacity() >= M, "M=%d: layout (%d,%d,%d) holds only %d", M, s.g, s.ng, s.w, s.capacity());
          CHECK(s.full == (s.capacity() == M), "M=%d: full flag", M);
          CHECK(M % s.g == 0 && (base + off) % (esz * (uintptr_t)s.g) == 0, "M=%d off=%d: load width %d not usable", M,
                (int)off, s.g);
          CHECK((s.w == 1) == (M <= rtopk::kMaxWaveM), "M=%d: wavefronts per row %d", M, s.w);
          CHECK(s.w == 1 ? s.g * s.ng <= 128 : s.g * s.ng <= 64, "M=%d: %d values per lane", M, s.g * s.ng);
          ++n;
        }
      }
    }
    for (uintptr_t oi : {0, 4, 8, 16})
      for (uintptr_t oo : {0, 4, 8, 16}) {
        const rtopk::Shape s = rtopk::classify_dense(M, base + oi, base + 0x100000 + oo);
        CHECK(rtopk::instantiated(s, rtopk::kF32, false, true), "dense M=%d: (%d,%d,%d) not compiled", M, s.g, s.ng, s.w);
        CHECK(s.capacity() >= M && s.full == (s.capacity() == M), "dense M=%d capacity", M);
        CHECK(M % s.g == 0 && (base + oi) % (4u * (uintptr_t)s.g) == 0 && (base + oo) % (4u * (uintptr_t)s.g) == 0,
              "dense M=%d: load width %d not usable", M, s.g);
        ++n;
      }
  }
  // beyond the widest row a workgroup holds: fp32 rows are streamed, with 128-bit loads where they can be
  for (int64_t M = rtopk::kMaxBlockM + 1; M <= rtopk::kMaxM; M += (M < 70000 ? 1 : 9973)) {
    for (uintptr_t off : offs) {
      if (off % 4) continue;
      for (int plain = 0; plain <= 1; ++plain) {
        const rtopk::Shape s = rtopk::classify((int)M, rtopk::kF32, plain != 0, base + off);
        CHECK(s.family == rtopk::kFamStream && rtopk::instantiated(s, rtopk::kF32, plain != 0, false), "M=%ld: not streamed", (long)M);
        CHECK((s.g == 4) == (M % 4 == 0 && (base + off) % 16 == 0) && (s.g == 4 || s.g == 1), "M=%ld off=%d: load width %d", (long)M,
              (int)off, s.g);
        ++n;
      }
    }
  }
  // range overlap helper
  CHECK(!rtopk::ranges_overlap(100, 10, 110, 10), "adjacent ranges do not overlap");
  CHECK(rtopk::ranges_overlap(100, 11, 110, 10), "one shared byte");
  CHECK(rtopk::ranges_overlap(100, 50, 120, 5), "containment");
  CHECK(!rtopk::ranges_overlap(100, 0, 100, 10), "empty range");
  CHECK(!rtopk::ranges_overlap(~(uintptr_t)0 - 7, 8, 0, 8), "top of the address space");
  return n;
}

int main(int argc, char** argv) {
  if (argc < 2) {
    std::fprintf(stderr, "usage: %s <alg2_handtrace.txt>\n", argv[0]);
    return 2;
  }
  const int traces = run_hand_traces(argv[1]);
  if (traces < 0) return 2;
  const int rows = run_brute_force();
  const long shapes = run_shape_sweep();
  std::printf("hand traces %d, brute-force rows %d, shapes %ld, failures %d\n", traces, rows, shapes, g_failures);
  return g_failures == 0 ? 0 : 1;
}
