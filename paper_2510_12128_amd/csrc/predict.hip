// Posterior prediction (Section 2.1, posterior forward formulae), with the approximated
// covariance K' of Section 3.3 in the place of the exact one:
//   mu_j  = <k_j, K'^-1 y>,      v_j = alpha - <k_j, K'^-1 k_j>,
// where k_j = k(X_train, x*_j) is the exact kernel between the training points and test point j
// and K_** has alpha on its diagonal.  The solves go through the same batched preconditioned CG
// as the loss: one single-column solve for y, then (for the variances) the cross-covariance
// columns in batches as wide as the context's vector blocks.  K_* is never stored: each batch of
// its columns is generated in fp64 straight into the right-hand-side block.
#include <algorithm>
#include <cmath>

#include "nugpr_internal.h"

namespace nugpr {

struct CrossArgs {
  double inv_ell[MAX_D];     // 1 / lengthscale per dimension
  double alpha;
  int d;
};

// U[i, col] = alpha exp(-0.5 sum_k ((x_ik - x*_jk) / ell_k)^2) for j = j0 + col, col < cnt;
// columns cnt..T-1 of the block are cleared (a zero right-hand side is skipped by the solver).
template <typename VT>
__global__ __launch_bounds__(256) void k_cross_block(CrossArgs a, const float* __restrict__ X,
                                                     const float* __restrict__ Xt, int64_t j0, int cnt,
                                                     int64_t n, int T, VT* __restrict__ U) {
  const int rpp = 256 / T;
  const int tid = threadIdx.x;
  const int myrow = tid / T, col = tid - myrow * T;
  if (myrow >= rpp) return;
  const bool live = col < cnt;
  const float* xt = Xt + (live ? (j0 + col) * (int64_t)a.d : 0);
  for (int64_t r = (int64_t)blockIdx.x * rpp + myrow; r < n; r += (int64_t)gridDim.x * rpp) {
    double v = 0.0;
    if (live) {
      const float* x = X + r * a.d;
      double q = 0.0;
      for (int k = 0; k < a.d; ++k) {
        const double t = ((double)x[k] - (double)xt[k]) * a.inv_ell[k];
        q = fma(t, t, q);
      }
      v = a.alpha * exp(-0.5 * q);
    }
    U[r * T + col] = (VT)v;
  }
}

// partial[0][block][col] = sum_i U[i,col] u[i],  partial[1][block][col] = sum_i U[i,col] S[i,col]
// (S may be null: then only the first set is written).  Same fixed summation order as the CG dots.
template <typename VT>
__global__ __launch_bounds__(256) void k_predict_dots(const VT* __restrict__ U, const VT* __restrict__ u,
                                                      const VT* __restrict__ S, int64_t n, int T,
                                                      double* __restrict__ partial) {
  __shared__ double red[2][256];
  const int rpp = 256 / T;
  const int tid = threadIdx.x;
  const int myrow = tid / T, col = tid - myrow * T;
  const bool live = myrow < rpp;
  const int64_t rows_per_block = (n + gridDim.x - 1) / gridDim.x;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
  double s0 = 0.0, s1 = 0.0;
  if (live) {
    for (int64_t r = r0 + myrow; r < r1; r += rpp) {
      const int64_t idx = r * T + col;
      const double k = (double)U[idx];
      s0 = fma(k, (double)u[r], s0);
      if (S) s1 = fma(k, (double)S[idx], s1);
    }
  }
  red[0][tid] = s0;
  red[1][tid] = s1;
  __syncthreads();
  if (tid < T) {
    for (int w = 0; w < 2; ++w) {
      double s = 0.0;
      for (int k = 0; k < rpp; ++k) s += red[w][k * T + tid];
      partial[((int64_t)w * gridDim.x + blockIdx.x) * MAX_COLS + tid] = s;
    }
  }
}

template <typename VT>
static int predict_t(nugpr_ctx* c, const double* theta, const float* Xt, int64_t m, double* mean, double* var,
                     int32_t* max_iters_used, hipStream_t s) {
  const Layout& L = c->L;
  const int64_t n = L.n;
  const int T = L.T;
  int worst = NUGPR_OK, mx_all = 0;
  VT *U = (VT*)c->Uv, *S = (VT*)c->Xv, *u = (VT*)c->x0;
  // u = K'^-1 y: a one-column block is just the vector
  int rc = to_internal(c, c->y, U, n, s);
  if (rc) return rc;
  int mx = 0;
  rc = run_pcg(c, U, S, 1, nullptr, nullptr, nullptr, &mx, s);
  if (rc < 0 || rc == NUGPR_INDEFINITE || rc == NUGPR_NOT_FINITE) return rc;
  worst = std::max(worst, rc);
  mx_all = std::max(mx_all, mx);
  NUGPR_HIP(hipMemcpyAsync(u, S, (size_t)n * sizeof(VT), hipMemcpyDeviceToDevice, s));

  CrossArgs a;
  const bool iso = (c->params.flags & NUGPR_ISOTROPIC) != 0;
  for (int k = 0; k < L.d; ++k) a.inv_ell[k] = 1.0 / theta[iso ? 0 : k];
  for (int k = L.d; k < MAX_D; ++k) a.inv_ell[k] = 0.0;
  a.alpha = theta[L.p - 2];
  a.d = L.d;
  const int nb = L.n_dot_blocks;
  const int rpp = 256 / T;
  const int grid = (int)std::min<int64_t>((n + rpp - 1) / rpp, 8192);
  for (int64_t j0 = 0; j0 < m; j0 += T) {
    const int cnt = (int)std::min<int64_t>(T, m - j0);
    hipLaunchKernelGGL((k_cross_block<VT>), dim3(grid), dim3(256), 0, s, a, c->X, Xt, j0, cnt, n, T, U);
    NUGPR_HIP(hipGetLastError());
    if (var) {
      rc = run_pcg(c, U, S, T, nullptr, nullptr, nullptr, &mx, s);
      if (rc < 0 || rc == NUGPR_INDEFINITE || rc == NUGPR_NOT_FINITE) return rc;
      worst = std::max(worst, rc);
      mx_all = std::max(mx_all, mx);
    }
    hipLaunchKernelGGL((k_predict_dots<VT>), dim3(nb), dim3(256), 0, s, U, u, var ? S : (const VT*)nullptr, n, T,
                       c->dotpart);
    NUGPR_HIP(hipGetLastError());
    NUGPR_HIP(hipMemcpyAsync(c->h_buf, c->dotpart, (size_t)2 * nb * MAX_COLS * sizeof(double),
                             hipMemcpyDeviceToHost, s));
    NUGPR_HIP(hipStreamSynchronize(s));
    for (int col = 0; col < cnt; ++col) {
      double d0 = 0.0, d1 = 0.0;
      for (int b = 0; b < nb; ++b) {
        d0 += c->h_buf[(size_t)b * MAX_COLS + col];
        d1 += c->h_buf[((size_t)nb + b) * MAX_COLS + col];
      }
      mean[j0 + col] = d0;
      if (var) var[j0 + col] = a.alpha - d1;
    }
  }
  if (max_iters_used) *max_iters_used = mx_all;
  return worst;
}

int run_predict(nugpr_ctx* c, const double* theta, const float* Xt, int64_t m, double* mean, double* var,
                int32_t* max_iters_used, hipStream_t s) {
  if (c->acc64) return predict_t<double>(c, theta, Xt, m, mean, var, max_iters_used, s);
  return predict_t<float>(c, theta, Xt, m, mean, var, max_iters_used, s);
}

}  // namespace nugpr
