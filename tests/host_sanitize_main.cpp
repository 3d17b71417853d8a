// Driver for the sanitizer builds of the host translation unit (csrc/lorc_host.cpp): exercises the threaded SVD
// (thread team, barriers, spin-waits), the rank schedule, the error bound and the index helpers, and checks the
// results against properties that need no reference implementation.  Exit status 0 = every check passed; the
// sanitizer runtimes turn a detected error into a non-zero status on their own.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "lorc.h"

static int fails = 0;
#define CHECK(c)                                          \
  do {                                                    \
    if (!(c)) {                                           \
      std::fprintf(stderr, "check failed: %s\n", #c);     \
      ++fails;                                            \
    }                                                     \
  } while (0)

static double lcg(unsigned long long& s) {  // uniform in (-1, 1)
  s = s * 6364136223846793005ull + 1442695040888963407ull;
  return ((double)(s >> 11) / 9007199254740992.0) * 2.0 - 1.0;
}

static void factorize_case(int rows, int cols, int rank) {
  unsigned long long seed = 12345u + rows * 131u + cols;
  std::vector<double> W((size_t)rows * cols);
  for (auto& v : W) v = lcg(seed);
  for (int i = 0; i < rows; ++i)
    for (int j = 0; j < cols; ++j) W[(size_t)i * cols + j] /= (1.0 + j);  // decaying column scales
  std::vector<double> A((size_t)rows * rank), B((size_t)rank * cols), sigma(cols);
  double eps = -1;
  CHECK(lorc_factorize(W.data(), rows, cols, rank, A.data(), B.data(), sigma.data(), &eps) == LORC_OK);
  for (int j = 1; j < cols; ++j) CHECK(sigma[j - 1] >= sigma[j] && sigma[j] >= 0);
  // rows of B orthonormal
  for (int a = 0; a < rank; ++a)
    for (int b = a; b < rank; ++b) {
      double d = 0;
      for (int j = 0; j < cols; ++j) d += B[(size_t)a * cols + j] * B[(size_t)b * cols + j];
      CHECK(std::fabs(d - (a == b ? 1.0 : 0.0)) < 1e-10);
    }
  // ||W - A B||_F^2 = sum of the discarded sigma^2 (Eckart-Young), and eps is its relative form
  double res2 = 0, w2 = 0, tail2 = 0;
  for (int i = 0; i < rows; ++i)
    for (int j = 0; j < cols; ++j) {
      double v = 0;
      for (int c = 0; c < rank; ++c) v += A[(size_t)i * rank + c] * B[(size_t)c * cols + j];
      const double d = W[(size_t)i * cols + j] - v;
      res2 += d * d;
      w2 += W[(size_t)i * cols + j] * W[(size_t)i * cols + j];
    }
  for (int j = rank; j < cols; ++j) tail2 += sigma[j] * sigma[j];
  CHECK(std::fabs(res2 - tail2) <= 1e-9 * w2);
  CHECK(std::fabs(eps - std::sqrt(tail2 / w2)) < 1e-10);
}

int main() {
  factorize_case(96, 48, 16);
  factorize_case(130, 64, 64);
  factorize_case(75, 33, 7);  // odd column count: the Jacobi ring is padded with a phantom column
  CHECK(lorc_factorize(nullptr, 4, 4, 2, nullptr, nullptr, nullptr, nullptr) == LORC_EINVAL);

  // rank schedule: first layer d_max, last layer d_min, non-increasing
  const int L = 6, n = 16;
  std::vector<double> sk((size_t)L * n), sv((size_t)L * n);
  for (int l = 0; l < L; ++l)
    for (int i = 0; i < n; ++i) sk[(size_t)l * n + i] = sv[(size_t)l * n + i] = std::pow(i + 1.0, -0.5 - 0.1 * l);
  std::vector<int32_t> ranks(L);
  CHECK(lorc_rank_schedule(sk.data(), sv.data(), L, n, 16, 4, 2, 0.0, ranks.data()) == LORC_OK);
  CHECK(ranks[0] == 16 && ranks[L - 1] == 4);
  for (int l = 1; l < L; ++l) CHECK(ranks[l] <= ranks[l - 1]);

  std::vector<double> terms(L);
  double bound = -1;
  std::vector<int32_t> rk(L, 8);
  CHECK(lorc_error_bound(sk.data(), rk.data(), L, n, 1.0, terms.data(), &bound) == LORC_OK);
  double sum = 0;
  for (double t : terms) sum += t;
  CHECK(std::fabs(sum - bound) < 1e-12 && bound > 0);

  lorc_layer_desc d = {256, 4, 2, 64, 32, 64, 10000.0f, 0.0f, LORC_PAGE_TOKENS};
  CHECK(lorc_page_bytes(&d) == (size_t)64 * (32 + 64) * 2);
  std::vector<char> seen(64 * (32 + 64), 0);
  for (int t = 0; t < 64; ++t) {
    for (int j = 0; j < 32; ++j) seen[lorc_cache_index_k(&d, t, j)]++;
    for (int j = 0; j < 64; ++j) seen[lorc_cache_index_v(&d, t, j)]++;
  }
  for (char c : seen) CHECK(c == 1);  // the two tilings together are a bijection onto the page
  CHECK(lorc_cache_index_k(&d, 64, 0) == -1 && lorc_cache_index_v(&d, 0, 64) == -1);
  std::printf("host sanitizer driver: %d failed checks\n", fails);
  return fails ? 1 : 0;
}
