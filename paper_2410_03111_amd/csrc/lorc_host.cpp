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

// ------------------------------------------------------------------------------------------ Householder QR
// M is column-major [m x n] (column j at M + j*m).  On return the upper triangle holds R and the
// reflector of step k is stored below the diagonal of column k with an implicit leading 1; beta[k] is
// its scale (H_k = I - beta v v^T).
void householder_qr(double* M, int m, int n, std::vector<double>& beta, int nthreads) {
  beta.assign(n, 0.0);
  Barrier bar(nthreads);
  run_team(nthreads, [&](int tid) {
    for (int k = 0; k < n; ++k) {
      double* ck = M + (size_t)k * m;
      if (tid == 0) {
        double norm2 = 0;
        for (int i = k + 1; i < m; ++i) norm2 += ck[i] * ck[i];
        double alpha = ck[k];
        if (norm2 == 0.0) {
          beta[k] = 0.0;
        } else {
          double nrm = std::sqrt(alpha * alpha + norm2);
          double v0 = alpha <= 0 ? alpha - nrm : -norm2 / (alpha + nrm);
          beta[k] = 2.0 * v0 * v0 / (norm2 + v0 * v0);
          for (int i = k + 1; i < m; ++i) ck[i] /= v0;
          ck[k] = nrm;  // R_kk (sign folded: H x = +nrm e_k)
        }
      }
      bar.wait();
      const double b = beta[k];
      if (b != 0.0) {
        for (int j = k + 1 + tid; j < n; j += nthreads) {
          double* cj = M + (size_t)j * m;
          double dot = cj[k];
          for (int i = k + 1; i < m; ++i) dot += ck[i] * cj[i];
          dot *= b;
          cj[k] -= dot;
          for (int i = k + 1; i < m; ++i) cj[i] -= dot * ck[i];
        }
      }
      bar.wait();
    }
  });
}

// X (column-major [m x c]) <- Q X with Q = H_0 H_1 ... H_{n-1} from householder_qr.
void apply_q(const double* M, const std::vector<double>& beta, int m, int n, double* X, int c, int nthreads) {
  run_team(nthreads, [&](int tid) {
    for (int j = tid; j < c; j += nthreads) {
      double* xj = X + (size_t)j * m;
      for (int k = n - 1; k >= 0; --k) {
        const double b = beta[k];
        if (b == 0.0) continue;
        const double* ck = M + (size_t)k * m;
        double dot = xj[k];
        for (int i = k + 1; i < m; ++i) dot += ck[i] * xj[i];
        dot *= b;
        xj[k] -= dot;
        for (int i = k + 1; i < m; ++i) xj[i] -= dot * ck[i];
      }
    }
  });
}

// ------------------------------------------------------------------------------------------ one-sided Jacobi
// G column-major [m x n], V column-major [n x n] (starts as identity).  Rotates column pairs until all are
// mutually orthogonal: afterwards G = U diag(sigma) and the input equals G V^T.  Round-robin ordering gives
// n/2 disjoint pairs per round, shared among the threads.  Returns the number of sweeps, or -1.
int jacobi_orthogonalise(double* G, double* V, int m, int n, int nthreads) {
  const int np = n + (n & 1);  // pad to even with a phantom column
  std::vector<int> ring(np);
  std::iota(ring.begin(), ring.end(), 0);
  const double tol = 4.0 * std::numeric_limits<double>::epsilon();
  const int max_sweeps = 60;
  std::atomic<long> rotations(0);
  std::atomic<int> result(-1);
  Barrier bar(nthreads);
  run_team(nthreads, [&](int tid) {
    for (int sweep = 0; sweep < max_sweeps; ++sweep) {
      for (int round = 0; round < np - 1; ++round) {
        for (int k = tid; k < np / 2; k += nthreads) {
          int p = ring[k], q = ring[np - 1 - k];
          if (p >= n || q >= n) continue;
          if (p > q) std::swap(p, q);
          double* gp = G + (size_t)p * m;
          double* gq = G + (size_t)q * m;
          double a = 0, b = 0, c = 0;
          for (int i = 0; i < m; ++i) {
            a += gp[i] * gp[i];
            b += gq[i] * gq[i];
            c += gp[i] * gq[i];
          }
          if (c == 0.0 || std::fabs(c) <= tol * std::sqrt(a * b)) continue;
          rotations.fetch_add(1, std::memory_order_relaxed);
          double zeta = (b - a) / (2.0 * c);
          double t = (zeta >= 0 ? 1.0 : -1.0) / (std::fabs(zeta) + std::sqrt(1.0 + zeta * zeta));
          double cs = 1.0 / std::sqrt(1.0 + t * t), sn = cs * t;
          for (int i = 0; i < m; ++i) {
            double x = gp[i], y = gq[i];
            gp[i] = cs * x - sn * y;
            gq[i] = sn * x + cs * y;
          }
          double* vp = V + (size_t)p * n;
          double* vq = V + (size_t)q * n;
          for (int i = 0; i < n; ++i) {
            double x = vp[i], y = vq[i];
            vp[i] = cs * x - sn * y;
            vq[i] = sn * x + cs * y;
          }
        }
        bar.wait();
        if (tid == 0) std::rotate(ring.begin() + 1, ring.end() - 1, ring.end());  // keep ring[0] fixed
        bar.wait();
      }
      bool done = rotations.load() == 0;
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
  // Step 1: W = Q R (Householder), so that the Jacobi iteration runs on an n x n matrix.
  std::vector<double> M((size_t)m * n);
  double frob2 = 0;
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) {
      double v = W[(size_t)i * n + j];
      if (!std::isfinite(v)) return LORC_EINVAL;
      M[(size_t)j * m + i] = v;
      frob2 += v * v;
    }
  std::vector<double> beta;
  householder_qr(M.data(), m, n, beta, nt);
  // Step 2: R = G V^T with orthogonal columns in G (one-sided Jacobi): G = U_R diag(sigma).
  std::vector<double> G((size_t)n * n, 0.0), V((size_t)n * n, 0.0);
  for (int j = 0; j < n; ++j) {
    for (int i = 0; i <= j; ++i) G[(size_t)j * n + i] = M[(size_t)j * m + i];
    V[(size_t)j * n + j] = 1.0;
  }
  if (jacobi_orthogonalise(G.data(), V.data(), n, n, nt) < 0) return LORC_ENOCONV;
  // Step 3: order by singular value, keep the leading `rank` triplets.
  std::vector<double> s(n);
  for (int j = 0; j < n; ++j) {
    double a = 0;
    for (int i = 0; i < n; ++i) a += G[(size_t)j * n + i] * G[(size_t)j * n + i];
    s[j] = std::sqrt(a);
  }
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
  // A = Q [G_r; 0]  (columns of G already carry sigma), B = V_r^T, with the sign convention on B's rows.
  std::vector<double> X((size_t)m * rank, 0.0);
  for (int c = 0; c < rank; ++c) {
    const int src = order[c];
    const double* v = &V[(size_t)src * n];
    int arg = 0;
    for (int i = 1; i < n; ++i)
      if (std::fabs(v[i]) > std::fabs(v[arg])) arg = i;
    const double sign = v[arg] < 0 ? -1.0 : 1.0;
    for (int i = 0; i < n; ++i) {
      X[(size_t)c * m + i] = sign * G[(size_t)src * n + i];
      B[(size_t)c * n + i] = sign * v[i];
    }
  }
  apply_q(M.data(), beta, m, n, X.data(), rank, nt);
  for (int i = 0; i < m; ++i)
    for (int c = 0; c < rank; ++c) A[(size_t)i * rank + c] = X[(size_t)c * m + i];
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
