// Autotuner of the trigger thresholds (R1, R2): host code only (no kernel, no HIP call).
//
// Sec. 3.3 and the appendix on the BO autotuner: the thresholds are tuned by Bayesian optimisation
// of the measured time per accepted token: Gaussian-process regression with a Matern kernel as the
// surrogate, Expected Improvement (exploration parameter 0.1 in the paper) as the acquisition
// function, search space (0,1)^2, one random initial sample, 16 samples in all.  The paper names
// these ingredients and nothing else; what is fixed here beyond them: smoothness 5/2, observations
// standardised before regression, hyper-parameters given by the caller (no likelihood fit), EI on
// the standardised scale, and the maximiser of EI taken over the midpoints of a uniform grid.
//
// The regression is done with a Cholesky factor of the kernel matrix (n <= 4096 observations),
// fp64 throughout.
#include <math.h>

#include <new>
#include <vector>

#include "../../include/pipesd.h"

namespace {

constexpr int32_t kMaxObservations = 4096;
constexpr int32_t kMaxGrid = 1024;

bool finite_pos(double v) { return v > 0.0 && isfinite(v); }

double matern52(double dx, double dy, double inv_len) {
  const double r = sqrt(dx * dx + dy * dy) * inv_len, s5 = sqrt(5.0);
  return (1.0 + s5 * r + (5.0 / 3.0) * r * r) * exp(-s5 * r);
}

// The surrogate after n observations: lower Cholesky factor L of K + noise I (row-major, n x n),
// the weights w = (K + noise I)^-1 y_s, and how the observations were standardised.
struct Surrogate {
  int32_t n = 0;
  double inv_len = 0.0, mean = 0.0, scale = 1.0, best_s = 0.0;
  std::vector<double> L, w;
  const double* x = nullptr;

  // returns false if the matrix is not positive definite (duplicate points without noise)
  bool fit(const double* xs, const double* ys, int32_t count, double length_scale, double noise) {
    n = count;
    x = xs;
    inv_len = 1.0 / length_scale;
    double sum = 0.0;
    for (int32_t i = 0; i < n; ++i) sum += ys[i];
    mean = sum / n;
    double ss = 0.0;
    for (int32_t i = 0; i < n; ++i) ss += (ys[i] - mean) * (ys[i] - mean);
    scale = sqrt(ss / n);
    if (!(scale > 0.0)) scale = 1.0;
    L.assign((size_t)n * n, 0.0);
    w.assign((size_t)n, 0.0);
    best_s = INFINITY;
    for (int32_t i = 0; i < n; ++i) {
      w[i] = (ys[i] - mean) / scale;
      if (w[i] < best_s) best_s = w[i];
    }
    // column-by-column Cholesky of the kernel matrix, built on the fly
    for (int32_t j = 0; j < n; ++j) {
      double d = 1.0 + noise;
      for (int32_t k = 0; k < j; ++k) d -= L[(size_t)j * n + k] * L[(size_t)j * n + k];
      if (!(d > 0.0)) return false;
      const double ljj = sqrt(d);
      L[(size_t)j * n + j] = ljj;
      for (int32_t i = j + 1; i < n; ++i) {
        double v = matern52(xs[2 * i] - xs[2 * j], xs[2 * i + 1] - xs[2 * j + 1], inv_len);
        for (int32_t k = 0; k < j; ++k) v -= L[(size_t)i * n + k] * L[(size_t)j * n + k];
        L[(size_t)i * n + j] = v / ljj;
      }
    }
    // w <- L^-T L^-1 y_s
    for (int32_t i = 0; i < n; ++i) {
      double v = w[i];
      for (int32_t k = 0; k < i; ++k) v -= L[(size_t)i * n + k] * w[k];
      w[i] = v / L[(size_t)i * n + i];
    }
    for (int32_t i = n - 1; i >= 0; --i) {
      double v = w[i];
      for (int32_t k = i + 1; k < n; ++k) v -= L[(size_t)k * n + i] * w[k];
      w[i] = v / L[(size_t)i * n + i];
    }
    return true;
  }

  // posterior mean and standard deviation at (q1, q2) on the standardised scale; `tmp` has n entries
  void predict(double q1, double q2, std::vector<double>& tmp, double* mu_s, double* sd_s) const {
    double mu = 0.0;
    for (int32_t i = 0; i < n; ++i) {
      tmp[i] = matern52(x[2 * i] - q1, x[2 * i + 1] - q2, inv_len);
      mu += tmp[i] * w[i];
    }
    // var = 1 - |L^-1 k|^2
    double red = 0.0;
    for (int32_t i = 0; i < n; ++i) {
      double v = tmp[i];
      for (int32_t k = 0; k < i; ++k) v -= L[(size_t)i * n + k] * tmp[k];
      tmp[i] = v / L[(size_t)i * n + i];
      red += tmp[i] * tmp[i];
    }
    const double var = 1.0 - red;
    *mu_s = mu;
    *sd_s = var > 0.0 ? sqrt(var) : 0.0;
  }
};

// E[max(best - xi - Y, 0)] for Y ~ N(mu, sd^2)
double expected_improvement(double mu, double sd, double best, double xi) {
  const double imp = best - mu - xi;
  if (!(sd > 0.0)) return imp > 0.0 ? imp : 0.0;
  const double z = imp / sd;
  const double cdf = 0.5 * (1.0 + erf(z / sqrt(2.0)));
  const double pdf = exp(-0.5 * z * z) / sqrt(2.0 * M_PI);
  return imp * cdf + sd * pdf;
}

int check_observations(const double* x, const double* y, int32_t n, double length_scale, double noise) {
  if (!x || !y || n < 1 || n > kMaxObservations) return PIPESD_EINVAL;
  if (!finite_pos(length_scale) || !(noise >= 0.0) || !isfinite(noise)) return PIPESD_EINVAL;
  for (int32_t i = 0; i < n; ++i) {
    if (!isfinite(y[i]) || !isfinite(x[2 * i]) || !isfinite(x[2 * i + 1])) return PIPESD_EINVAL;
  }
  return PIPESD_OK;
}

}  // namespace

extern "C" int pipesd_bo_posterior(const double* x, const double* y, int32_t n, double length_scale, double noise,
                                   const double* q, int32_t m, double* mean_out, double* std_out) {
  int rc = check_observations(x, y, n, length_scale, noise);
  if (rc) return rc;
  if (m < 0 || (m > 0 && (!q || !mean_out || !std_out))) return PIPESD_EINVAL;
  try {
    Surrogate s;
    if (!s.fit(x, y, n, length_scale, noise)) return PIPESD_EINVAL;
    std::vector<double> tmp((size_t)n);
    for (int32_t j = 0; j < m; ++j) {
      double mu, sd;
      s.predict(q[2 * j], q[2 * j + 1], tmp, &mu, &sd);
      mean_out[j] = s.mean + s.scale * mu;
      std_out[j] = s.scale * sd;
    }
  } catch (const std::bad_alloc&) {
    return PIPESD_ENOMEM;
  }
  return PIPESD_OK;
}

extern "C" int pipesd_bo_suggest(const double* x, const double* y, int32_t n, double length_scale, double noise, double xi,
                                 int32_t grid, double* next_out, double* ei_out) {
  int rc = check_observations(x, y, n, length_scale, noise);
  if (rc) return rc;
  if (!next_out || grid < 1 || grid > kMaxGrid || !(xi >= 0.0) || !isfinite(xi)) return PIPESD_EINVAL;
  try {
    Surrogate s;
    if (!s.fit(x, y, n, length_scale, noise)) return PIPESD_EINVAL;
    std::vector<double> tmp((size_t)n);
    double best_ei = -1.0, b1 = 0.0, b2 = 0.0;
    for (int32_t i = 0; i < grid; ++i) {
      const double r1 = ((double)i + 0.5) / (double)grid;
      for (int32_t j = 0; j < grid; ++j) {
        const double r2 = ((double)j + 0.5) / (double)grid;
        double mu, sd;
        s.predict(r1, r2, tmp, &mu, &sd);
        const double ei = expected_improvement(mu, sd, s.best_s, xi);
        if (ei > best_ei) {  // strict: the first of equal values stays
          best_ei = ei;
          b1 = r1;
          b2 = r2;
        }
      }
    }
    next_out[0] = b1;
    next_out[1] = b2;
    if (ei_out) *ei_out = best_ei;
  } catch (const std::bad_alloc&) {
    return PIPESD_ENOMEM;
  }
  return PIPESD_OK;
}
