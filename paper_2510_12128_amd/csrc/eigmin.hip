// lambda_0 of eq. (krep), the smallest eigenvalue of the kernel matrix C of all representatives (Section 3.3),
// for couplings too large for a dense host eigen-solve: a matrix-free, block-preconditioned Davidson
// iteration in fp64 on the device.
//
// Why not a plain Krylov (Lanczos) process: representatives of one cluster lie close together, so the low end of
// C's spectrum is a dense cluster of small eigenvalues (often down to rounding level) under a largest eigenvalue of
// order n_c r; a polynomial in C then needs thousands of steps to resolve lambda_min to 1e-10.  The same
// structure makes the remedy cheap: the small eigenvalues come from WITHIN the diagonal blocks of C, so the
// inverse of a block-diagonal part of C, in fp64, is a preconditioner that takes the cluster apart.
//
// The matrix is applied through the strip kernels that the product K' D uses for C S, on its two-term
// representation: off the diagonal C = Chi + Clo (Chi the stored fp32 entries, Clo what fp32 dropped, itself in
// fp32: together ~2^-48 relative), on the diagonal the exact scalar alpha.
// Iteration (generalised Davidson, Rayleigh-Ritz on an orthonormal basis V with thick restart):
//   (theta, y) = smallest eigenpair of H = V^T C V;  x = V y;  res = C x - theta x;
//   t = T res with T = blockdiag(B_k + mu I)^-1, B_k the 128 x 128 diagonal blocks of C recomputed in fp64
//       from the representatives and Cholesky-factored once per assembly (mu = 1e-10 alpha);
//   t is orthogonalised against V (modified Gram-Schmidt, twice), normalised and appended; C t is computed.
// All vector work of a step runs in single workgroups with fixed-order reductions, so lambda_0 is reproducible
// to the bit.  Stop: the Ritz value theta is safe when min(|res|, 4 |res|^2 / gap) <= tol (gap: distance to the
// second Ritz value, used when it is clearly separate), or when |theta| <= tol: a kernel matrix is positive
// semi-definite, so lambda_min lies in [0, theta].  Ritz values approach lambda_min from above, so
// C - theta I misses being positive semi-definite by at most the tolerance, far below the noise variance.
// One regime converges slowly: strongly overlapping clusters with a wide lengthscale, where the small eigenvalues
// belong to modes that span many blocks.  There lambda_min is itself tiny; if the step cap is reached with
// theta <= 1e-5 alpha, theta is returned as it stands (lambda_min lies in [0, theta]; the cap makes the step
// count, and with it theta, the same smooth function of the hyperparameters on both sides of a difference
// quotient).  A run that reaches the cap with a larger theta is an error.
#include <algorithm>
#include <cmath>
#include <vector>

#include "nugpr_internal.h"

namespace nugpr {

constexpr int EB = 128;               // order of the preconditioner's diagonal blocks
constexpr int EBP = EB + 1;           // row stride of a block in LDS (odd: column accesses spread over the banks)
constexpr int DAV_MAX_BASIS = 24;     // basis vectors kept before a restart
constexpr int DAV_KEEP = 3;           // Ritz vectors a restart keeps
constexpr int DAV_MAX_STEPS = 150;

struct BlockKernelArgs {
  double inv_ell[MAX_D];
  double alpha, mu;
  int n, d;
};

// Cholesky factor (lower, row-major EB x EB doubles per block, unit rows past the end) of B_k + mu I, where
// B_k = k(R_k, R_k) for the representatives 128 k .. 128 k + 127, evaluated in fp64 with direct differences.
__global__ __launch_bounds__(256) void k_block_factor(BlockKernelArgs a, const float* __restrict__ reps,
                                                      double* __restrict__ Lout) {
  extern __shared__ __attribute__((aligned(16))) double M[];      // EB rows of EBP
  const int blk = blockIdx.x, tid = threadIdx.x;
  const int i0 = blk * EB;
  const int nb = min(EB, a.n - i0);
  for (int idx = tid; idx < EB * EB; idx += 256) {
    const int i = idx / EB, j = idx % EB;
    double v = (i == j) ? 1.0 : 0.0;
    if (i < nb && j < nb && j <= i) {
      double q = 0.0;
      const float* ri = reps + (uint64_t)(i0 + i) * a.d;
      const float* rj = reps + (uint64_t)(i0 + j) * a.d;
      for (int k = 0; k < a.d; ++k) {
        const double t = ((double)ri[k] - (double)rj[k]) * a.inv_ell[k];
        q = fma(t, t, q);
      }
      v = a.alpha * exp(-0.5 * q) + (i == j ? a.mu : 0.0);
    }
    M[i * EBP + j] = v;
  }
  __syncthreads();
  // right-looking elimination on the lower triangle; a pivot that rounding pushed below the shift is replaced by it
  for (int j = 0; j < nb; ++j) {
    if (tid == 0) {
      double p = M[j * EBP + j];
      if (!(p > 1e-3 * a.mu)) p = 1e-3 * a.mu;
      M[j * EBP + j] = sqrt(p);
    }
    __syncthreads();
    const double ljj = M[j * EBP + j];
    for (int i = j + 1 + tid; i < nb; i += 256) M[i * EBP + j] /= ljj;
    __syncthreads();
    const int m = nb - j - 1;                       // trailing rows / columns
    for (int idx = tid; idx < m * m; idx += 256) {
      const int i = j + 1 + idx / m, k = j + 1 + idx % m;
      if (k <= i) M[i * EBP + k] = fma(-M[i * EBP + j], M[k * EBP + j], M[i * EBP + k]);
    }
    __syncthreads();
  }
  double* out = Lout + (uint64_t)blk * EB * EB;
  for (int idx = tid; idx < EB * EB; idx += 256) {
    const int i = idx / EB, j = idx % EB;
    out[idx] = j <= i ? M[i * EBP + j] : 0.0;
  }
}

// t = blockdiag(L_k L_k^T)^-1 res: forward and back substitution inside each block, one workgroup per block
__global__ __launch_bounds__(128) void k_block_solve(const double* __restrict__ Lall, const double* __restrict__ res,
                                                     double* __restrict__ t, int n) {
  extern __shared__ __attribute__((aligned(16))) double Ls[];     // EB x EB factor, then EB values
  double* x = Ls + EB * EBP;
  const int blk = blockIdx.x, tid = threadIdx.x;
  const int i0 = blk * EB;
  const int nb = min(EB, n - i0);
  const double* L = Lall + (uint64_t)blk * EB * EB;
  for (int idx = tid; idx < EB * EB; idx += 128) Ls[(idx / EB) * EBP + idx % EB] = L[idx];
  double b = tid < nb ? res[i0 + tid] : 0.0;
  __syncthreads();
  for (int j = 0; j < nb; ++j) {                    // L z = res
    if (tid == j) x[j] = b / Ls[j * EBP + j];
    __syncthreads();
    if (tid > j && tid < nb) b = fma(-Ls[tid * EBP + j], x[j], b);
  }
  __syncthreads();
  b = tid < nb ? x[tid] : 0.0;
  __syncthreads();
  for (int j = nb - 1; j >= 0; --j) {               // L^T t = z
    if (tid == j) x[j] = b / Ls[j * EBP + j];
    __syncthreads();
    if (tid < j) b = fma(-Ls[j * EBP + tid], x[j], b);
  }
  __syncthreads();
  if (tid < nb) t[i0 + tid] = x[tid];
}

// v_0: a fixed +-1 pattern (integer hash of the index), normalised
__global__ void k_eig_start(double* __restrict__ v, int n) {
  const double s = 1.0 / sqrt((double)n);
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    uint32_t h = (uint32_t)i * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    v[i] = (h & 1u) ? s : -s;
  }
}

__device__ __forceinline__ double block_sum_1024(double x, double* red) {
  const int tid = threadIdx.x;
  red[tid] = x;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if (tid < w) red[tid] += red[tid + w];
    __syncthreads();
  }
  const double r = red[0];
  __syncthreads();
  return r;
}

struct Coef { double y[DAV_MAX_BASIS]; };

// AV[m] = sum of the column-slab partial sums of C V[m]; h[i] = <V[i], AV[m]>, i = 0 .. m
__global__ __launch_bounds__(1024) void k_eig_newrow(const double* __restrict__ parts, int nparts, uint64_t stride,
                                                     const double* __restrict__ V, double* __restrict__ AV, int m,
                                                     int n, int ld, double* __restrict__ out) {
  __shared__ double red[1024];
  const int tid = threadIdx.x;
  double* av = AV + (uint64_t)m * ld;
  for (int i = tid; i < n; i += 1024) {
    double w = parts[i];
    for (int p = 1; p < nparts; ++p) w += parts[(uint64_t)p * stride + i];
    av[i] = w;
  }
  __syncthreads();
  for (int k = 0; k <= m; ++k) {
    const double* v = V + (uint64_t)k * ld;
    double acc = 0.0;
    for (int i = tid; i < n; i += 1024) acc = fma(v[i], av[i], acc);
    const double s = block_sum_1024(acc, red);
    if (tid == 0) out[k] = s;
  }
}

// x = V y, res = AV y - theta x (m vectors); out[0] = |res|^2.  x is not kept: only the residual is needed.
__global__ __launch_bounds__(1024) void k_eig_residual(const double* __restrict__ V, const double* __restrict__ AV,
                                                       Coef c, double theta, int m, int n, int ld,
                                                       double* __restrict__ res, double* __restrict__ out) {
  __shared__ double red[1024];
  const int tid = threadIdx.x;
  double acc = 0.0;
  for (int i = tid; i < n; i += 1024) {
    double x = 0.0, ax = 0.0;
    for (int k = 0; k < m; ++k) {
      x = fma(c.y[k], V[(uint64_t)k * ld + i], x);
      ax = fma(c.y[k], AV[(uint64_t)k * ld + i], ax);
    }
    const double r = fma(-theta, x, ax);
    res[i] = r;
    acc = fma(r, r, acc);
  }
  const double s = block_sum_1024(acc, red);
  if (tid == 0) out[0] = s;
}

// V[m] = t orthogonalised against V[0 .. m-1] (modified Gram-Schmidt, two passes) and normalised;
// out[0] = its norm before the normalisation
__global__ __launch_bounds__(1024) void k_eig_orth(double* __restrict__ V, const double* __restrict__ t, int m, int n,
                                                   int ld, double* __restrict__ out) {
  __shared__ double red[1024];
  const int tid = threadIdx.x;
  double* vn = V + (uint64_t)m * ld;
  for (int i = tid; i < n; i += 1024) vn[i] = t[i];
  __syncthreads();
  for (int pass = 0; pass < 2; ++pass)
    for (int k = 0; k < m; ++k) {
      const double* v = V + (uint64_t)k * ld;
      double acc = 0.0;
      for (int i = tid; i < n; i += 1024) acc = fma(v[i], vn[i], acc);
      const double s = block_sum_1024(acc, red);
      for (int i = tid; i < n; i += 1024) vn[i] = fma(-s, v[i], vn[i]);
      __syncthreads();
    }
  double acc = 0.0;
  for (int i = tid; i < n; i += 1024) acc = fma(vn[i], vn[i], acc);
  const double nrm = sqrt(block_sum_1024(acc, red));
  const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
  for (int i = tid; i < n; i += 1024) vn[i] *= inv;
  if (tid == 0) out[0] = nrm;
}

// restart: V <- V Y, AV <- AV Y for the `keep` coefficient columns in c (column q at y[q * m ..]); element-wise, in place
struct RestartCoef { double y[DAV_KEEP * DAV_MAX_BASIS]; };
__global__ void k_eig_restart(double* __restrict__ V, double* __restrict__ AV, RestartCoef c, int m, int keep, int n,
                              int ld) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    double v[DAV_MAX_BASIS], av[DAV_MAX_BASIS];
    for (int k = 0; k < m; ++k) { v[k] = V[(uint64_t)k * ld + i]; av[k] = AV[(uint64_t)k * ld + i]; }
    for (int q = 0; q < keep; ++q) {
      double a = 0.0, b = 0.0;
      for (int k = 0; k < m; ++k) { a = fma(c.y[q * m + k], v[k], a); b = fma(c.y[q * m + k], av[k], b); }
      V[(uint64_t)q * ld + i] = a;
      AV[(uint64_t)q * ld + i] = b;
    }
  }
}

// what fp32 storage drops of the diagonal entries alpha - lambda_0: Chi_ii = float(alpha - lambda_0),
// Clo_ii = float((alpha - lambda_0) - Chi_ii)
__global__ void k_coupling_set_diag(float* __restrict__ Chi, float* __restrict__ Clo, uint32_t ld, int n, double value) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float hi = (float)value;
  const uint64_t at = blocked_index(ld, (uint32_t)i, (uint32_t)i);
  Chi[at] = hi;
  Clo[at] = (float)(value - (double)hi);
}

int coupling_set_diag(nugpr_ctx* c, double value, hipStream_t s) {
  const Layout& L = c->L;
  hipLaunchKernelGGL(k_coupling_set_diag, dim3((L.ncr + 255) / 256), dim3(256), 0, s, c->C, c->Clo, (uint32_t)L.ldc, L.ncr,
                     value);
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

// eigen-decomposition of a small symmetric matrix (row-major m x m, overwritten) by cyclic Jacobi rotations:
// eigenvalues ascending in ev, eigenvectors in the columns of Y (row-major m x m)
static void small_sym_eigen(std::vector<double>& A, int m, std::vector<double>& ev, std::vector<double>& Y) {
  Y.assign((size_t)m * m, 0.0);
  for (int i = 0; i < m; ++i) Y[(size_t)i * m + i] = 1.0;
  for (int sweep = 0; sweep < 60; ++sweep) {
    double off = 0.0, diag = 0.0;
    for (int i = 0; i < m; ++i)
      for (int j = 0; j < m; ++j) (i == j ? diag : off) += A[(size_t)i * m + j] * A[(size_t)i * m + j];
    if (off <= 1e-32 * diag) break;
    for (int p = 0; p < m; ++p)
      for (int q = p + 1; q < m; ++q) {
        const double apq = A[(size_t)p * m + q];
        if (apq == 0.0) continue;
        const double tau = (A[(size_t)q * m + q] - A[(size_t)p * m + p]) / (2.0 * apq);
        const double t = (tau >= 0.0 ? 1.0 : -1.0) / (std::fabs(tau) + std::sqrt(1.0 + tau * tau));
        const double cs = 1.0 / std::sqrt(1.0 + t * t), sn = t * cs;
        for (int k = 0; k < m; ++k) {             // columns p, q
          const double akp = A[(size_t)k * m + p], akq = A[(size_t)k * m + q];
          A[(size_t)k * m + p] = cs * akp - sn * akq;
          A[(size_t)k * m + q] = sn * akp + cs * akq;
        }
        for (int k = 0; k < m; ++k) {             // rows p, q
          const double apk = A[(size_t)p * m + k], aqk = A[(size_t)q * m + k];
          A[(size_t)p * m + k] = cs * apk - sn * aqk;
          A[(size_t)q * m + k] = sn * apk + cs * aqk;
        }
        for (int k = 0; k < m; ++k) {
          const double ykp = Y[(size_t)k * m + p], ykq = Y[(size_t)k * m + q];
          Y[(size_t)k * m + p] = cs * ykp - sn * ykq;
          Y[(size_t)k * m + q] = sn * ykp + cs * ykq;
        }
      }
  }
  std::vector<int> order(m);
  for (int i = 0; i < m; ++i) order[i] = i;
  std::sort(order.begin(), order.end(), [&](int a, int b) { return A[(size_t)a * m + a] < A[(size_t)b * m + b]; });
  ev.resize(m);
  std::vector<double> Ys((size_t)m * m);
  for (int q = 0; q < m; ++q) {
    ev[q] = A[(size_t)order[q] * m + order[q]];
    for (int k = 0; k < m; ++k) Ys[(size_t)k * m + q] = Y[(size_t)k * m + order[q]];
  }
  Y.swap(Ys);
}

// lambda_min of the matrix whose off-diagonal part is stored in (c->C, c->Clo) (diagonal entries of both zero)
// and whose diagonal is the scalar alpha = theta[p - 2].  Scratch: the partial-sum slabs of the coupling product
// and the Davidson area of the workspace.  Synchronises the stream once per step.
int coupling_lambda_min(nugpr_ctx* c, const double* theta, hipStream_t s, double* lambda_out, int* steps_out) {
  const Layout& L = c->L;
  const int n = L.ncr, ld = L.ldc;
  if (!c->acc64) { set_error("the matrix-free lambda_0 needs the fp64 arithmetic mode"); return NUGPR_ERR_INVALID; }
  const bool iso = (c->params.flags & NUGPR_ISOTROPIC) != 0;
  const double alpha = theta[L.p - 2];
  const int nblk = (n + EB - 1) / EB;
  double *V = c->dav, *AV = V + (size_t)DAV_MAX_BASIS * ld, *res = AV + (size_t)DAV_MAX_BASIS * ld, *tvec = res + ld,
         *small = tvec + ld, *Lblk = small + 64;
  static const hipError_t lds_attr = []() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_block_factor), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       EB * EBP * (int)sizeof(double));
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_block_solve), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (EB * EBP + EB) * (int)sizeof(double));
  }();
  NUGPR_HIP(lds_attr);
  BlockKernelArgs ba;
  for (int k = 0; k < MAX_D; ++k) ba.inv_ell[k] = k < L.d ? 1.0 / (iso ? theta[0] : theta[k]) : 0.0;
  ba.alpha = alpha; ba.mu = 1e-10 * alpha; ba.n = n; ba.d = L.d;
  hipLaunchKernelGGL(k_block_factor, dim3(nblk), dim3(256), EB * EBP * sizeof(double), s, ba, c->reps, Lblk);
  hipLaunchKernelGGL(k_eig_start, dim3(64), dim3(256), 0, s, V, n);
  NUGPR_HIP(hipGetLastError());
  const uint64_t stride = (uint64_t)n;            // one column: a slab of the partial sums is n doubles
  double* parts = static_cast<double*>(c->Ppart);
  const double tol = EIGMIN_REL_TOL * std::fabs(alpha);
  int rc;
  // C V[m] into AV[m] and the new row of H; returns after the host has the row
  std::vector<double> H((size_t)DAV_MAX_BASIS * DAV_MAX_BASIS, 0.0);
  auto extend = [&](int m) -> int {             // V[m] exists: AV[m] = C V[m], H[m][0..m]
    StripPort p{};
    p.A = c->C; p.in = V + (size_t)m * ld; p.nin = 1; p.out = parts; p.out_part_stride = stride; p.diag_add = alpha;
    if ((rc = launch_strip(c->tab_C, p, p, 1, true, s))) return rc;
    StripPort q = p;
    q.A = c->Clo; q.accumulate = 1; q.diag_add = 0.0;
    if ((rc = launch_strip(c->tab_C, q, q, 1, true, s))) return rc;
    hipLaunchKernelGGL(k_eig_newrow, dim3(1), dim3(1024), 0, s, (const double*)parts, L.nsP, stride, (const double*)V, AV, m, n,
                       ld, small + 8);
    NUGPR_HIP(hipGetLastError());
    NUGPR_HIP(hipMemcpyAsync(c->h_buf, small, (size_t)(8 + DAV_MAX_BASIS) * sizeof(double), hipMemcpyDeviceToHost, s));
    NUGPR_HIP(hipStreamSynchronize(s));
    for (int k = 0; k <= m; ++k) {
      const double h = c->h_buf[8 + k];
      if (!std::isfinite(h)) { set_error("lambda_0: the projected matrix is not finite"); return NUGPR_ERR_INVALID; }
      H[(size_t)m * DAV_MAX_BASIS + k] = H[(size_t)k * DAV_MAX_BASIS + m] = h;
    }
    return NUGPR_OK;
  };
  if ((rc = extend(0))) return rc;
  int m = 1, step = 0;
  double thetaR = H[0], est = INFINITY;
  bool done = false;
  std::vector<double> A, ev, Y;
  for (; step < DAV_MAX_STEPS; ++step) {
    A.assign((size_t)m * m, 0.0);
    for (int i = 0; i < m; ++i)
      for (int j = 0; j < m; ++j) A[(size_t)i * m + j] = H[(size_t)i * DAV_MAX_BASIS + j];
    small_sym_eigen(A, m, ev, Y);
    thetaR = ev[0];
    if (m == DAV_MAX_BASIS) {
      // thick restart: the lowest Ritz vectors become the basis, H their (diagonal) Rayleigh quotients
      RestartCoef rcf;
      for (int q = 0; q < DAV_KEEP; ++q)
        for (int k = 0; k < m; ++k) rcf.y[q * m + k] = Y[(size_t)k * m + q];
      hipLaunchKernelGGL(k_eig_restart, dim3(64), dim3(256), 0, s, V, AV, rcf, m, DAV_KEEP, n, ld);
      NUGPR_HIP(hipGetLastError());
      std::fill(H.begin(), H.end(), 0.0);
      for (int q = 0; q < DAV_KEEP; ++q) H[(size_t)q * DAV_MAX_BASIS + q] = ev[q];
      std::vector<double> ev2(ev.begin(), ev.begin() + DAV_KEEP);
      m = DAV_KEEP;
      Y.assign((size_t)m * m, 0.0);
      for (int q = 0; q < m; ++q) Y[(size_t)q * m + q] = 1.0;
      ev = ev2;
    }
    Coef cf;
    for (int k = 0; k < DAV_MAX_BASIS; ++k) cf.y[k] = k < m ? Y[(size_t)k * m + 0] : 0.0;
    hipLaunchKernelGGL(k_eig_residual, dim3(1), dim3(1024), 0, s, (const double*)V, (const double*)AV, cf, thetaR, m, n, ld,
                       res, small);
    hipLaunchKernelGGL(k_block_solve, dim3(nblk), dim3(128), (EB * EBP + EB) * sizeof(double), s, (const double*)Lblk,
                       (const double*)res, tvec, n);
    hipLaunchKernelGGL(k_eig_orth, dim3(1), dim3(1024), 0, s, V, (const double*)tvec, m, n, ld, small + 1);
    NUGPR_HIP(hipGetLastError());
    if ((rc = extend(m))) return rc;              // (also brings |res|^2 and the norm of the new direction)
    const double rn = std::sqrt(std::max(c->h_buf[0], 0.0)), tn = c->h_buf[1];
    if (!std::isfinite(rn)) { set_error("lambda_0: residual not finite"); return NUGPR_ERR_INVALID; }
    est = rn;
    if (m > 1) {
      const double gap = ev[1] - ev[0];
      if (gap > 10.0 * rn) est = std::min(est, 4.0 * rn * rn / gap);
    }
    if (est <= tol || std::fabs(thetaR) <= tol) { done = true; break; }
    if (!(tn > 1e-300)) { done = est <= 1e3 * tol; break; }       // no new direction: the basis holds an invariant subspace
    m += 1;
  }
  if (steps_out) *steps_out = std::min(step + 1, DAV_MAX_STEPS);
  if (!done && std::fabs(thetaR) <= EIGMIN_PSD_TOL * std::fabs(alpha)) done = true;   // lambda_min in [0, theta], see above
  if (!done) {
    set_error("lambda_0: the eigenvalue iteration did not reach the tolerance in " + std::to_string(DAV_MAX_STEPS) + " steps");
    return NUGPR_ERR_INVALID;
  }
  *lambda_out = thetaR;
  return NUGPR_OK;
}

}  // namespace nugpr
