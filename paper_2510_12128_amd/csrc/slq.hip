// Host side of the stochastic Lanczos quadrature: the Lanczos tridiagonal of the
// preconditioned operator is rebuilt from one column's CG coefficients (the classical
// CG <-> Lanczos relation, Saad, Iterative Methods for Sparse Linear Systems, Sec. 6.7)
// and e_1^T log(T) e_1 is evaluated from its eigen-decomposition; this is the Gauss
// quadrature for z^T log(A) z / |z|^2 that eq. (trace estimation) / eq. (logdet) need.
#include <cmath>
#include <vector>

#include "nugpr_internal.h"

namespace nugpr {

// Symmetric tridiagonal eigenproblem by the implicit-shift QL iteration, carrying only
// the first row of the eigenvector matrix (all the quadrature needs).
// d: diagonal (k), e: sub-diagonal (k-1, padded to k), z: out first components.
int tridiag_eigen_first_row(std::vector<double>& d, std::vector<double>& e, std::vector<double>& z) {
  const int k = (int)d.size();
  z.assign(k, 0.0);
  z[0] = 1.0;
  e.resize(k, 0.0);
  for (int l = 0; l < k; ++l) {
    int sweeps = 0;
    while (true) {
      int m = l;
      for (; m < k - 1; ++m) {
        const double scale = std::fabs(d[m]) + std::fabs(d[m + 1]);
        if (std::fabs(e[m]) <= 2.3e-16 * scale) break;
      }
      if (m == l) break;
      if (++sweeps > 80) return 1;
      double g = (d[l + 1] - d[l]) / (2.0 * e[l]);
      double r = std::hypot(g, 1.0);
      g = d[m] - d[l] + e[l] / (g + (g >= 0.0 ? r : -r));
      double s = 1.0, c = 1.0, p = 0.0;
      int i = m - 1;
      bool deflated = false;
      for (; i >= l; --i) {
        double f = s * e[i];
        const double b = c * e[i];
        r = std::hypot(f, g);
        e[i + 1] = r;
        if (r == 0.0) {
          d[i + 1] -= p;
          e[m] = 0.0;
          deflated = true;
          break;
        }
        s = f / r;
        c = g / r;
        g = d[i + 1] - p;
        r = (d[i] - g) * s + 2.0 * c * b;
        p = s * r;
        d[i + 1] = g + p;
        g = c * r - b;
        f = z[i + 1];                 // rotate the first-row entries of columns i, i+1
        z[i + 1] = s * z[i] + c * f;
        z[i] = c * z[i] - s * f;
      }
      if (deflated) continue;
      d[l] -= p;
      e[l] = g;
      e[m] = 0.0;
    }
  }
  return 0;
}

int slq_e1_log_e1(const double* alpha, const double* beta, int stride, int k, double* out) {
  if (k < 1) { *out = 0.0; return 0; }
  std::vector<double> d(k), e(k > 1 ? k - 1 : 0), z;
  d[0] = 1.0 / alpha[0];
  for (int j = 1; j < k; ++j) {
    const double a_prev = alpha[(size_t)(j - 1) * stride], b_prev = beta[(size_t)(j - 1) * stride];
    d[j] = 1.0 / alpha[(size_t)j * stride] + b_prev / a_prev;
    e[j - 1] = std::sqrt(b_prev) / a_prev;
  }
  for (int j = 0; j < k; ++j)
    if (!std::isfinite(d[j])) return 1;
  if (tridiag_eigen_first_row(d, e, z)) return 1;
  double acc = 0.0;
  for (int j = 0; j < k; ++j) {
    if (!(d[j] > 0.0)) return 1;
    acc += z[j] * z[j] * std::log(d[j]);
  }
  *out = acc;
  return 0;
}

// Smallest eigenvalue of a dense symmetric matrix (row-major n x n, overwritten): Householder reduction
// to tridiagonal form, A <- H A H with H = I - 2 v v^T / v^T v column by column, then the QL iteration
// above.  Used for lambda_0 of eq. (krep), on the host, in fp64.
int sym_smallest_eigenvalue(std::vector<double>& A, int n, double* out) {
  if (n < 1 || (size_t)n * n > A.size()) return 1;
  auto a = [&](int i, int j) -> double& { return A[(size_t)i * n + j]; };
  std::vector<double> d(n), e(n > 1 ? n - 1 : 0), v(n), q(n), z;
  for (int k = 0; k + 2 < n; ++k) {
    double nrm2 = 0.0;
    for (int i = k + 1; i < n; ++i) nrm2 += a(i, k) * a(i, k);
    const double x0 = a(k + 1, k), sigma = std::sqrt(nrm2);
    if (sigma == 0.0) { e[k] = 0.0; continue; }
    const double alpha = x0 >= 0.0 ? -sigma : sigma;          // no cancellation in v_0 = x_0 - alpha
    for (int i = k + 1; i < n; ++i) v[i] = a(i, k);
    v[k + 1] -= alpha;
    const double vtv = 2.0 * (nrm2 - alpha * x0);
    const double beta = 2.0 / vtv;
    double vtp = 0.0;
    for (int i = k + 1; i < n; ++i) {                         // p = beta A_sub v
      double acc = 0.0;
      for (int j = k + 1; j < n; ++j) acc += a(i, j) * v[j];
      q[i] = beta * acc;
      vtp += v[i] * q[i];
    }
    const double kk = vtp / vtv;
    for (int i = k + 1; i < n; ++i) q[i] -= kk * v[i];        // q = p - (v^T p / v^T v) v
    for (int i = k + 1; i < n; ++i)                           // A_sub -= v q^T + q v^T
      for (int j = k + 1; j < n; ++j) a(i, j) -= v[i] * q[j] + q[i] * v[j];
    e[k] = alpha;
  }
  for (int i = 0; i < n; ++i) d[i] = a(i, i);
  if (n >= 2) e[n - 2] = a(n - 1, n - 2);
  for (int i = 0; i < n; ++i)
    if (!std::isfinite(d[i])) return 1;
  if (tridiag_eigen_first_row(d, e, z)) return 1;
  double mn = d[0];
  for (int i = 1; i < n; ++i) mn = d[i] < mn ? d[i] : mn;
  *out = mn;
  return 0;
}

}  // namespace nugpr
