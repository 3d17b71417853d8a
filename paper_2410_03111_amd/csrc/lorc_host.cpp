// Host side of the LoRC library: truncated SVD of the K/V projection weights (Section 4.1, Algorithm 1),
// the progressive rank schedule (Section 4.2), error strings and the cache index helpers.
// Plain C++ threads, fp64 throughout; nothing here touches the GPU.
#include <sched.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <limits>
#include <numeric>
#include <thread>
#include <vector>

#include "lorc.h"
#include "lorc_layout.h"

namespace {

// ------------------------------------------------------------------------------------------ thread team
int host_threads() {
  int n = 0;
  cpu_set_t set;
  if (sched_getaffinity(0, sizeof(set), &set) == 0) n = CPU_COUNT(&set);
  if (n <= 0) n = (int)std::thread::hardware_concurrency();
  if (const char* e = std::getenv("LORC_NUM_THREADS")) {
    int v = std::atoi(e);
    if (v > 0) n = v;
  }
  return std::max(1, std::min(n, 16));
}

// A team of workers that repeatedly runs body(tid) phases separated by barriers.
class Barrier {
 public:
  explicit Barrier(int n) : n_(n), count_(0), phase_(0) {}
  void wait() {
    int ph = phase_.load(std::memory_order_acquire);
    if (count_.fetch_add(1, std::memory_order_acq_rel) == n_ - 1) {
      count_.store(0, std::memory_order_relaxed);
      phase_.store(ph + 1, std::memory_order_release);
    } else {
      int spins = 0;
      while (phase_.load(std::memory_order_acquire) == ph) {
        if (++spins > 2000) std::this_thread::yield();
      }
    }
  }

 private:
  const int n_;
  std::atomic<int> count_;
  std::atomic<int> phase_;
};

void run_team(int nthreads, const std::function<void(int)>& body) {
  std::vector<std::thread> th;
  for (int t = 1; t < nthreads; ++t) th.emplace_back(body, t);
  body(0);
  for (auto& t : th) t.join();
}

// ------------------------------------------------------------------------------------------ vector kernels
// The inner loops of the factorisation, each built twice: for the baseline x86-64 ISA and for AVX2 + FMA, picked
// once at run time.  Fixed summation order (eight partial sums), so results do not depend on the thread count.
#define LORC_VECTOR_KERNELS(SUFFIX, ATTR)                                                                   \
  ATTR double dot_##SUFFIX(const double* a, const double* b, int n) {                                       \
    double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};                                                                 \
    int i = 0;                                                                                              \
    for (; i + 8 <= n; i += 8)                                                                              \
      for (int u = 0; u < 8; ++u) s[u] += a[i + u] * b[i + u];                                              \
    for (; i < n; ++i) s[i & 7] += a[i] * b[i];                                                             \
    return ((s[0] + s[4]) + (s[2] + s[6])) + ((s[1] + s[5]) + (s[3] + s[7]));                               \
  }                                                                                                         \
  ATTR void rot_##SUFFIX(double* a, double* b, int n, double cs, double sn) {                               \
    for (int i = 0; i < n; ++i) {                                                                           \
      const double x = a[i], y = b[i];                                                                      \
      a[i] = cs * x - sn * y;                                                                               \
      b[i] = sn * x + cs * y;                                                                               \
    }                                                                                                       \
  }                                                                                                         \
  ATTR void axpy_##SUFFIX(double* y, const double* x, int n, double alpha) {                                \
    for (int i = 0; i < n; ++i) y[i] -= alpha * x[i];                                                       \
  }
LORC_VECTOR_KERNELS(base, )
LORC_VECTOR_KERNELS(avx2, __attribute__((target("avx2,fma"))))
#undef LORC_VECTOR_KERNELS

struct VectorKernels {
  double (*dot)(const double*, const double*, int);
  void (*rot)(double*, double*, int, double, double);
  void (*axpy)(double*, const double*, int, double);
};
const VectorKernels& vk() {
  static const VectorKernels k = (__builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma"))
                                     ? VectorKernels{dot_avx2, rot_avx2, axpy_avx2}
                                     : VectorKernels{dot_base, rot_base, axpy_base};
  return k;
}

// ------------------------------------------------------------------------------------------ Householder QR
// M is column-major [m x n] (column j at M + j*m).  On return the upper triangle holds R and the
// reflector of step k is stored below the diagonal of column k with an implicit leading 1; beta[k] is
// its scale (H_k = I - beta v v^T).  With perm != nullptr columns are pivoted (largest remaining norm first)
// and perm[k] is the original index of the column that ended up at k.
//
// Without pivoting the columns are walked in panels of 32: a panel's reflectors are formed one after the other
// (each applied to the rest of the panel at once), then every later column takes the 32 reflectors in one visit,
// so the trailing matrix is streamed from memory once per panel instead of once per column.  The arithmetic per
// column is that of the unblocked algorithm.
void make_reflector(double* ck, int k, int m, double& beta_k) {
  const double norm2 = vk().dot(ck + k + 1, ck + k + 1, m - k - 1);
  const double alpha = ck[k];
  if (norm2 == 0.0) {
    beta_k = 0.0;
    return;
  }
  const double nrm = std::sqrt(alpha * alpha + norm2);
  const double v0 = alpha <= 0 ? alpha - nrm : -norm2 / (alpha + nrm);
  beta_k = 2.0 * v0 * v0 / (norm2 + v0 * v0);
  const double inv = 1.0 / v0;
  for (int i = k + 1; i < m; ++i) ck[i] *= inv;
  ck[k] = nrm;  // R_kk (sign folded: H x = +nrm e_k)
}

inline void apply_reflector(const double* ck, double b, double* cj, int k, int m) {
  if (b == 0.0) return;
  const double dot = b * (cj[k] + vk().dot(ck + k + 1, cj + k + 1, m - k - 1));
  cj[k] -= dot;
  vk().axpy(cj + k + 1, ck + k + 1, m - k - 1, dot);
}

void householder_qr(double* M, int m, int n, std::vector<double>& beta, int nthreads, std::vector<int>* perm = nullptr) {
  beta.assign(n, 0.0);
  const int steps = std::min(m, n);
  std::vector<double> cnorm;
  if (perm) {
    perm->resize(n);
    std::iota(perm->begin(), perm->end(), 0);
    cnorm.assign(n, 0.0);
  }
  Barrier bar(nthreads);
  const int nb = perm ? 1 : 32;
  run_team(nthreads, [&](int tid) {
    if (perm) {
      for (int j = tid; j < n; j += nthreads) cnorm[j] = vk().dot(M + (size_t)j * m, M + (size_t)j * m, m);
      bar.wait();
    }
    for (int k0 = 0; k0 < steps; k0 += nb) {
      const int k1 = std::min(k0 + nb, steps);
      for (int k = k0; k < k1; ++k) {
        double* ck = M + (size_t)k * m;
        if (tid == 0) {
          if (perm) {
            int best = k;
            for (int j = k + 1; j < n; ++j)
              if (cnorm[j] > cnorm[best]) best = j;
            if (best != k) {
              std::swap_ranges(ck, ck + m, M + (size_t)best * m);
              std::swap(cnorm[k], cnorm[best]);
              std::swap((*perm)[k], (*perm)[best]);
            }
          }
          make_reflector(ck, k, m, beta[k]);
        }
        bar.wait();
        const double b = beta[k];
        const int jend = perm ? n : k1;  // pivoting: the whole trailing matrix now; panels: the panel only
        for (int j = k + 1 + tid; j < jend; j += nthreads) {
          double* cj = M + (size_t)j * m;
          apply_reflector(ck, b, cj, k, m);
          if (perm) cnorm[j] = vk().dot(cj + k + 1, cj + k + 1, m - k - 1);  // exact norm of what is left of column j
        }
        bar.wait();
      }
      if (!perm) {
        for (int j = k1 + tid; j < n; j += nthreads) {
          double* cj = M + (size_t)j * m;
          for (int k = k0; k < k1; ++k) apply_reflector(M + (size_t)k * m, beta[k], cj, k, m);
        }
        bar.wait();
      }
    }
  });
}

// X (column-major [m x c]) <- Q X with Q = H_0 H_1 ... H_{n-1} from householder_qr.  A thread takes eight columns
// at a time, so that a reflector fetched from memory serves all eight.
void apply_q(const double* M, const std::vector<double>& beta, int m, int n, double* X, int c, int nthreads) {
  constexpr int kCols = 8;
  const int groups = (c + kCols - 1) / kCols;
  run_team(nthreads, [&](int tid) {
    for (int g = tid; g < groups; g += nthreads) {
      const int j0 = g * kCols, j1 = std::min(c, j0 + kCols);
      for (int k = std::min(m, n) - 1; k >= 0; --k)
        for (int j = j0; j < j1; ++j) apply_reflector(M + (size_t)k * m, beta[k], X + (size_t)j * m, k, m);
    }
  });
}

// ------------------------------------------------------------------------------------------ one-sided Jacobi
// X column-major [m x n].  Rotates column pairs until all columns are mutually orthogonal; afterwards
// X = X_0 J with J orthogonal, i.e. the columns are the left singular vectors of X_0 scaled by the singular values.
// J is not accumulated: the caller recovers what it needs from X_0 and the final X.
// Ordering: the columns are cut into blocks of 16; a sweep first rotates the pairs inside every block, then walks
// the round-robin schedule over BLOCKS, a thread rotating all 16 x 16 column pairs of its block pair while the 32
// columns sit in its cache (the plain round-robin over columns streams the whole matrix once per round, n - 1
// times per sweep).  Squared column norms are carried along and updated by the rotation formulas, and refreshed
// from the columns at the start of every sweep.  Returns the number of sweeps, or -1.
int jacobi_orthogonalise(double* X, int m, int n, int nthreads) {
  constexpr int kBlock = 16;
  const int nblk = (n + kBlock - 1) / kBlock;
  const int np = nblk + (nblk & 1);  // pad to even with a phantom block
  const double tol = 4.0 * std::numeric_limits<double>::epsilon();
  const int max_sweeps = 60;
  std::vector<double> nrm2(n);
  std::atomic<long> rotations(0);
  std::atomic<int> result(-1);
  Barrier bar(nthreads);
  auto rotate_pair = [&](int p, int q) -> bool {
    double* xp = X + (size_t)p * m;
    double* xq = X + (size_t)q * m;
    const double a = nrm2[p], b = nrm2[q];
    const double c = vk().dot(xp, xq, m);
    if (c == 0.0 || std::fabs(c) <= tol * std::sqrt(a * b)) return false;
    const double zeta = (b - a) / (2.0 * c);
    const double t = (zeta >= 0 ? 1.0 : -1.0) / (std::fabs(zeta) + std::sqrt(1.0 + zeta * zeta));
    const double cs = 1.0 / std::sqrt(1.0 + t * t), sn = cs * t;
    vk().rot(xp, xq, m, cs, sn);
    nrm2[p] = a - t * c;
    nrm2[q] = b + t * c;
    return true;
  };
  run_team(nthreads, [&](int tid) {
    for (int sweep = 0; sweep < max_sweeps; ++sweep) {
      long mine = 0;
      for (int j = tid; j < n; j += nthreads) nrm2[j] = vk().dot(X + (size_t)j * m, X + (size_t)j * m, m);
      bar.wait();
      for (int blk = tid; blk < nblk; blk += nthreads) {  // pairs inside a block
        const int c0 = blk * kBlock, c1 = std::min(n, c0 + kBlock);
        for (int p = c0; p < c1; ++p)
          for (int q = p + 1; q < c1; ++q) mine += rotate_pair(p, q);
      }
      bar.wait();
      for (int round = 0; round < np - 1; ++round) {
        // round-robin over blocks, block 0 fixed: position k holds block 0 (k = 0) or 1 + (k - 1 - round) mod (np - 1)
        auto at = [&](int k) { return k == 0 ? 0 : 1 + ((k - 1 - round) % (np - 1) + (np - 1)) % (np - 1); };
        for (int k = tid; k < np / 2; k += nthreads) {
          int bi = at(k), bj = at(np - 1 - k);
          if (bi >= nblk || bj >= nblk) continue;
          if (bi > bj) std::swap(bi, bj);
          const int p0 = bi * kBlock, p1 = std::min(n, p0 + kBlock), q0 = bj * kBlock, q1 = std::min(n, q0 + kBlock);
          for (int p = p0; p < p1; ++p)
            for (int q = q0; q < q1; ++q) mine += rotate_pair(p, q);
        }
        bar.wait();
      }
      rotations.fetch_add(mine, std::memory_order_relaxed);
      bar.wait();
      const bool done = rotations.load() == 0;
      bar.wait();
      if (tid == 0) rotations.store(0);
      bar.wait();
      if (done) {
        if (tid == 0) result.store(sweep + 1);
        return;
      }
    }
  });
  return result.load();
}

bool desc_ok(const lorc_layer_desc* d) { return d && lorc::check_desc(*d) == LORC_OK; }

}  // namespace

extern "C" {

const char* lorc_strerror(int code) {
  switch (code) {
    case LORC_OK: return "ok";
    case LORC_EINVAL: return "invalid argument (NULL pointer, bad size or inconsistent shape)";
    case LORC_EUNSUPPORTED: return "unsupported geometry (head_dim, rank or page size has no kernel)";
    case LORC_ENOCONV: return "SVD iteration did not converge";
    case LORC_EWORKSPACE: return "workspace too small";
    case LORC_EHIP: return "HIP runtime error at launch";
    default: return "unknown lorc status";
  }
}

int lorc_factorize(const double* W, int32_t rows, int32_t cols, int32_t rank, double* A, double* B,
                   double* sigma, double* rel_frob_err) {
  if (!W || !A || !B || rows <= 0 || cols <= 0 || rows < cols || rank < 1 || rank > cols) return LORC_EINVAL;
  const int m = rows, n = cols;
  const int nt = host_threads();
  // Step 1: W = Q_1 R_1 (Householder, panels), so that everything after runs on an n x n matrix.
  std::vector<double> M((size_t)m * n);
  double frob2 = 0;
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) {
      double v = W[(size_t)i * n + j];
      if (!std::isfinite(v)) return LORC_EINVAL;
      M[(size_t)j * m + i] = v;
      frob2 += v * v;
    }
  std::vector<double> beta1;
  householder_qr(M.data(), m, n, beta1, nt);
  // Step 2: R_1 P = Q_2 R_2 with column pivoting.  The Jacobi iteration then runs on X = R_2^T, whose columns are
  // far closer to orthogonal than those of R_1 (the preconditioning of Drmac and Veselic): a few sweeps instead of ten.
  std::vector<double> R1((size_t)n * n, 0.0);
  for (int j = 0; j < n; ++j)
    for (int i = 0; i <= j; ++i) R1[(size_t)j * n + i] = M[(size_t)j * m + i];
  std::vector<double> beta2;
  std::vector<int> perm;
  householder_qr(R1.data(), n, n, beta2, nt, &perm);
  std::vector<double> X((size_t)n * n, 0.0);  // X = R_2^T, column-major: X[j*n + i] = R_2[j][i] for i >= j
  for (int j = 0; j < n; ++j)
    for (int i = 0; i <= j; ++i) X[(size_t)i * n + j] = R1[(size_t)j * n + i];
  // Step 3: X J = U_X diag(sigma) (one-sided Jacobi), hence R_2 = J diag(sigma) U_X^T and
  //   W = (Q_1 Q_2 J) diag(sigma) (P U_X)^T,   with   J diag(sigma) = R_2 U_X.
  if (jacobi_orthogonalise(X.data(), n, n, nt) < 0) return LORC_ENOCONV;
  std::vector<double> s(n);
  for (int j = 0; j < n; ++j) s[j] = std::sqrt(vk().dot(&X[(size_t)j * n], &X[(size_t)j * n], n));
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return s[a] > s[b]; });
  if (sigma)
    for (int j = 0; j < n; ++j) sigma[j] = s[order[j]];
  if (rel_frob_err) {
    double tail = 0;
    for (int j = rank; j < n; ++j) tail += s[order[j]] * s[order[j]];
    *rel_frob_err = frob2 > 0 ? std::sqrt(tail / frob2) : 0.0;
  }
  // B = rows (P u_c)^T of the leading `rank` right singular vectors, u_c = X_c / sigma_c, with the sign convention;
  // A = Q_1 Q_2 (R_2 u_c) (the columns carry sigma).  A direction whose singular value vanished is completed to an
  // orthonormal row from the coordinate vectors (its column of A is zero either way).
  std::vector<double> Uc((size_t)n * rank), Y((size_t)n * rank, 0.0);
  const double tiny = s[order[0]] * std::numeric_limits<double>::min() * 4.0;
  for (int c = 0; c < rank; ++c) {
    const int src = order[c];
    double* u = &Uc[(size_t)c * n];
    if (s[src] > tiny) {
      const double inv = 1.0 / s[src];
      for (int i = 0; i < n; ++i) u[i] = X[(size_t)src * n + i] * inv;
    } else {
      bool found = false;
      for (int e = 0; e < n && !found; ++e) {
        for (int i = 0; i < n; ++i) u[i] = i == e ? 1.0 : 0.0;
        for (int pass = 0; pass < 2; ++pass)
          for (int d = 0; d < c; ++d) {
            const double* ud = &Uc[(size_t)d * n];
            vk().axpy(u, ud, n, vk().dot(u, ud, n));
          }
        const double nr = std::sqrt(vk().dot(u, u, n));
        if (nr > 0.5) {
          for (int i = 0; i < n; ++i) u[i] /= nr;
          found = true;
        }
      }
      if (!found) return LORC_ENOCONV;
    }
  }
  // y = R_2 u: after the pivoted factorisation R1's upper triangle holds R_2 (column j: rows 0 .. j)
  run_team(nt, [&](int tid) {
    for (int c = tid; c < rank; c += nt) {
      if (!(s[order[c]] > tiny)) continue;
      const double* u = &Uc[(size_t)c * n];
      double* y = &Y[(size_t)c * n];
      for (int j = 0; j < n; ++j) {
        const double uj = u[j];
        const double* col = &R1[(size_t)j * n];
        for (int i = 0; i <= j; ++i) y[i] += col[i] * uj;
      }
    }
  });
  apply_q(R1.data(), beta2, n, n, Y.data(), rank, nt);  // Q_2 y
  std::vector<double> Z((size_t)m * rank, 0.0);
  for (int c = 0; c < rank; ++c) {
    const double* u = &Uc[(size_t)c * n];
    int arg = 0;
    for (int i = 1; i < n; ++i)
      if (std::fabs(u[i]) > std::fabs(u[arg])) arg = i;
    const double sign = u[arg] < 0 ? -1.0 : 1.0;
    for (int i = 0; i < n; ++i) {
      Z[(size_t)c * m + i] = sign * Y[(size_t)c * n + i];
      B[(size_t)c * n + perm[i]] = sign * u[i];
    }
  }
  apply_q(M.data(), beta1, m, n, Z.data(), rank, nt);  // Q_1 [y; 0]
  for (int i = 0; i < m; ++i)
    for (int c = 0; c < rank; ++c) A[(size_t)i * rank + c] = Z[(size_t)c * m + i];
  return LORC_OK;
}

int lorc_rank_schedule(const double* sigma_k, const double* sigma_v, int32_t n_layers, int32_t n_sigma,
                       int32_t d_max, int32_t d_min, int32_t align, double log_threshold, int32_t* ranks) {
  if (!sigma_k || !sigma_v || !ranks || n_layers < 1 || n_sigma < 1 || align < 1 || d_min < 1 || d_max < d_min)
    return LORC_EINVAL;
  // log kappa of one matrix = log(sigma_max) - log(sigma_min); the cumulative value of layer l sums the
  // K and V terms of layers l..L-1 (the product of Eq. 12 taken in log space).
  std::vector<double> cum(n_layers);
  double run = 0;
  for (int l = n_layers - 1; l >= 0; --l) {
    for (const double* s : {sigma_k + (size_t)l * n_sigma, sigma_v + (size_t)l * n_sigma}) {
      double hi = 0, lo = std::numeric_limits<double>::infinity();
      for (int i = 0; i < n_sigma; ++i) {
        if (!(s[i] >= 0)) return LORC_EINVAL;
        hi = std::max(hi, s[i]);
        lo = std::min(lo, s[i]);
      }
      run += (lo == 0.0) ? std::numeric_limits<double>::infinity() : std::log(hi / lo);
    }
    cum[l] = run;
  }
  double hi = *std::max_element(cum.begin(), cum.end());
  double lo = *std::min_element(cum.begin(), cum.end());
  const bool use_thr = std::isfinite(log_threshold) && log_threshold > 0;
  for (int l = 0; l < n_layers; ++l) {
    double dc = d_max;
    if (std::isfinite(hi) && hi > lo) dc = d_max * (1.0 - (hi - cum[l]) / (hi - lo) * (1.0 - (double)d_min / d_max));
    long q = (long)std::floor(dc / align + 0.5) * align;
    q = std::max<long>(d_min, std::min<long>(d_max, q));
    ranks[l] = (use_thr && cum[l] > log_threshold) ? n_sigma : (int32_t)q;
  }
  return LORC_OK;
}

int lorc_error_bound(const double* sigma, const int32_t* ranks, int32_t n_layers, int32_t n_sigma, double lipschitz,
                     double* terms, double* bound) {
  if (!sigma || !ranks || !bound || n_layers < 1 || n_sigma < 1 || !(lipschitz >= 0)) return LORC_EINVAL;
  for (int l = 0; l < n_layers; ++l)
    if (ranks[l] < 0 || ranks[l] > n_sigma) return LORC_EINVAL;
  // term_i = (first singular value dropped by layer i) * L_phi^(L-1-i) * product of the spectral norms (largest
  // singular values) of the layers after i; walking from the last layer keeps that trailing factor as a running product
  double tail = 1.0, total = 0.0;
  for (int l = n_layers - 1; l >= 0; --l) {
    const double* s = sigma + (size_t)l * n_sigma;
    const double dropped = ranks[l] < n_sigma ? s[ranks[l]] : 0.0;
    if (!(dropped >= 0) || !(s[0] >= 0)) return LORC_EINVAL;
    const double t = dropped * tail;
    if (terms) terms[l] = t;
    total += t;
    tail *= lipschitz * s[0];
  }
  *bound = total;
  return LORC_OK;
}

size_t lorc_page_bytes(const lorc_layer_desc* desc) {
  if (!desc_ok(desc)) return 0;
  return lorc::page_elems(desc->rank_k, desc->rank_v) * sizeof(uint16_t);
}

int64_t lorc_cache_index_k(const lorc_layer_desc* desc, int32_t slot, int32_t j) {
  if (!desc_ok(desc) || slot < 0 || slot >= LORC_PAGE_TOKENS || j < 0 || j >= desc->rank_k) return -1;
  return lorc::k_index(desc->rank_k, slot, j);
}

int64_t lorc_cache_index_v(const lorc_layer_desc* desc, int32_t slot, int32_t j) {
  if (!desc_ok(desc) || slot < 0 || slot >= LORC_PAGE_TOKENS || j < 0 || j >= desc->rank_v) return -1;
  return lorc::v_index(desc->rank_k, slot, j);
}

}  // extern "C"
