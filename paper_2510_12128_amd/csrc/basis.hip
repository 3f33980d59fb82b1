// Nystrom basis for the rank-r off-diagonal blocks K'_ij = W_i C_ij W_j^T (Section 3.3 leaves the basis of a
// rank above one open; the default is the one-hot "nearest representative" basis, which for r = 1 is the
// paper's 1 1^T).  Here W_i = k(X_i, R_i) (k(R_i, R_i) + jitter I)^-1 at a given theta: every point is
// expressed through ALL representatives of its cluster by kernel interpolation instead of being identified
// with one of them.  The basis is computed once and then held fixed like any caller-supplied dense W (the loss
// stays a smooth function of the hyperparameters); the products go through the dense-W strips.
//
// One workgroup = one cluster and 256 of its points: the r x r kernel matrix of the cluster's
// representatives is Cholesky-factored in LDS in fp64, then the points are taken 16 at a time, 16 threads a
// point: k(x_p, R_i) into LDS, forward and back substitution with the 16 threads sharing each row's sum.
#include <cmath>

#include "nugpr_internal.h"

namespace nugpr {

constexpr int NB = 128;               // largest rank the factor fits into LDS for
constexpr int NBP = NB + 1;
constexpr int PTS = 256;              // points per workgroup

struct NystromArgs {
  double inv_ell[MAX_D];
  double alpha, jitter;
  int r, d;
  uint32_t ldw;
};

__global__ __launch_bounds__(256) void k_nystrom_W(NystromArgs a, const ClusterInfo* __restrict__ cl,
                                                   const float* __restrict__ X, const float* __restrict__ reps,
                                                   float* __restrict__ Wd, float* __restrict__ Wt) {
  extern __shared__ __attribute__((aligned(16))) double sm[];
  double* M = sm;                       // NB rows of NBP: kernel matrix of the representatives, then its factor
  double* vec = sm + NB * NBP;          // 16 right-hand sides of NB
  const ClusterInfo c = cl[blockIdx.y];
  const int tid = threadIdx.x, r = a.r, d = a.d;
  const int p_first = blockIdx.x * PTS;
  if (p_first >= (int)c.b) return;
  const float* Ri = reps + (uint64_t)blockIdx.y * r * d;
  for (int idx = tid; idx < r * r; idx += 256) {
    const int i = idx / r, j = idx % r;
    if (j > i) continue;
    double q = 0.0;
    for (int k = 0; k < d; ++k) {
      const double t = ((double)Ri[(uint64_t)i * d + k] - (double)Ri[(uint64_t)j * d + k]) * a.inv_ell[k];
      q = fma(t, t, q);
    }
    M[i * NBP + j] = a.alpha * exp(-0.5 * q) + (i == j ? a.jitter : 0.0);
  }
  __syncthreads();
  for (int j = 0; j < r; ++j) {         // right-looking Cholesky on the lower triangle
    if (tid == 0) {
      double p = M[j * NBP + j];
      if (!(p > 1e-3 * a.jitter)) p = 1e-3 * a.jitter;
      M[j * NBP + j] = sqrt(p);
    }
    __syncthreads();
    const double ljj = M[j * NBP + j];
    for (int i = j + 1 + tid; i < r; i += 256) M[i * NBP + j] /= ljj;
    __syncthreads();
    const int m = r - j - 1;
    for (int idx = tid; idx < m * m; idx += 256) {
      const int i = j + 1 + idx / m, k = j + 1 + idx % m;
      if (k <= i) M[i * NBP + k] = fma(-M[i * NBP + j], M[k * NBP + j], M[i * NBP + k]);
    }
    __syncthreads();
  }
  // 16 points at a time; the 16 threads (t = tid % 16) of a point sit in one wave
  const int g = tid >> 4, t = tid & 15;
  double* v = vec + g * NB;
  const int p_last = min((int)c.b, p_first + PTS);
  for (int base = p_first; base < p_last; base += 16) {
    const int pl = base + g;
    const bool live = pl < p_last;
    const uint64_t p = (uint64_t)c.row0 + (live ? pl : p_first);
    for (int k = t; k < r; k += 16) {
      double q = 0.0;
      for (int e = 0; e < d; ++e) {
        const double df = ((double)X[p * d + e] - (double)Ri[(uint64_t)k * d + e]) * a.inv_ell[e];
        q = fma(df, df, q);
      }
      v[k] = a.alpha * exp(-0.5 * q);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int j = 0; j < r; ++j) {       // L z = k
      double s = 0.0;
      for (int k = t; k < j; k += 16) s = fma(M[j * NBP + k], v[k], s);
      s += __shfl_xor(s, 1); s += __shfl_xor(s, 2); s += __shfl_xor(s, 4); s += __shfl_xor(s, 8);
      if (t == 0) v[j] = (v[j] - s) / M[j * NBP + j];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    for (int j = r - 1; j >= 0; --j) {  // L^T w = z
      double s = 0.0;
      for (int k = j + 1 + t; k < r; k += 16) s = fma(M[k * NBP + j], v[k], s);
      s += __shfl_xor(s, 1); s += __shfl_xor(s, 2); s += __shfl_xor(s, 4); s += __shfl_xor(s, 8);
      if (t == 0) v[j] = (v[j] - s) / M[j * NBP + j];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if (live) {
      const uint64_t row = (uint64_t)c.row0 + pl;
      for (uint32_t k = t; k < a.ldw; k += 16) Wd[row * a.ldw + k] = (int)k < r ? (float)v[k] : 0.f;
      for (int k = t; k < r; k += 16) Wt[c.wtoff + (uint64_t)k * c.ld + pl] = (float)v[k];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

int launch_nystrom_basis(nugpr_ctx* c, const double* theta, double jitter_rel, hipStream_t s) {
  const Layout& L = c->L;
  if (!theta) { set_error("theta is null"); return NUGPR_ERR_INVALID; }
  for (int i = 0; i < L.p; ++i)
    if (!(theta[i] > 0.0) || !std::isfinite(theta[i])) { set_error("theta entries must be finite and > 0"); return NUGPR_ERR_INVALID; }
  if (L.r > NB) { set_error("the Nystrom basis is built for rank <= 128"); return NUGPR_ERR_INVALID; }
  if (!(jitter_rel >= 0.0) || !(jitter_rel < 1.0)) { set_error("jitter must be in [0, 1)"); return NUGPR_ERR_INVALID; }
  const bool iso = (c->params.flags & NUGPR_ISOTROPIC) != 0;
  NystromArgs a;
  for (int k = 0; k < MAX_D; ++k) a.inv_ell[k] = k < L.d ? 1.0 / (iso ? theta[0] : theta[k]) : 0.0;
  a.alpha = theta[L.p - 2];
  a.jitter = (jitter_rel > 0.0 ? jitter_rel : 1e-4) * a.alpha;
  a.r = L.r; a.d = L.d; a.ldw = (uint32_t)L.ldw;
  const size_t lds = (size_t)(NB * NBP + 16 * NB) * sizeof(double);
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_nystrom_W),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)((NB * NBP + 16 * NB) * sizeof(double)));
  NUGPR_HIP(attr);
  uint32_t bmax = 0;
  for (const ClusterInfo& ci : L.cl) bmax = ci.b > bmax ? ci.b : bmax;
  hipLaunchKernelGGL(k_nystrom_W, dim3((bmax + PTS - 1) / PTS, (unsigned)L.nc), dim3(256), lds, s, a, c->d_cl, c->X, c->reps, c->Wd,
                     c->Wt);
  NUGPR_HIP(hipGetLastError());
  // the basis has changed: the stored operator, the factor's projections and anything solved before are stale
  c->onehot = false;
  c->z0_ready = false;
  c->factored = false;
  c->q0_gen = ~0ull;
  return NUGPR_OK;
}

}  // namespace nugpr
