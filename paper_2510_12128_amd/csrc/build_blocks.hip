// Block assembly (Section 2.1 kernel, K_diag of Section 3.2, representative-point
// coupling of Section 3.3) and the theta-independent setup (representatives, basis W).
//
// The covariance entries are written in fp32, but every scalar that multiplies ALL
// entries alike -- the per-dimension weights 1/(2 ell_k^2), the output scale alpha and
// the diagonal alpha + sigma^2 -- is carried as an fp32 (hi, lo) pair so that its
// rounding does not move between the two evaluations of a central difference (a
// rounding of 6e-8 in a scalar is amplified by 1/h = 1000 in the gradient).  The part of
// alpha + sigma^2 that fp32 cannot hold is kept as a scalar and added by the matrix-
// vector product (StripPort::diag_add).
//
// Squared distances use the direct difference form sum_k w_k (x_pk - x_qk)^2 on the
// vector ALUs; the |x|^2 + |x'|^2 - 2 x.x' contraction would put this on the matrix
// cores but cancels catastrophically in fp32.
#include <cmath>
#include <vector>

#include "nugpr_internal.h"

namespace nugpr {

struct PairArgs {
  float w_hi[MAX_D];
  float w_lo[MAX_D];
  float a_hi, a_lo;
  float diag_val;
  int32_t d;
};

// 64x64 tile of alpha * exp2(-sum_k w_k (xr_k - xc_k)^2); thread (ty, tx) holds a 4x4 patch.
// sXr / sXc: coordinates of the 64 row / column points, layout [k][64].
__device__ __forceinline__ void pair_tile(const PairArgs& a, const float (*sXr)[TILE], const float (*sXc)[TILE],
                                          int ty, int tx, float (&val)[4][4]) {
  float hi[4][4], lo[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) { hi[i][j] = 0.f; lo[i][j] = 0.f; }
  for (int k = 0; k < a.d; ++k) {
    const float4 xr = *reinterpret_cast<const float4*>(&sXr[k][4 * ty]);
    const float4 xc = *reinterpret_cast<const float4*>(&sXc[k][4 * tx]);
    const float wh = a.w_hi[k], wl = a.w_lo[k];
    const float r_[4] = {xr.x, xr.y, xr.z, xr.w};
    const float c_[4] = {xc.x, xc.y, xc.z, xc.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float df = r_[i] - c_[j];
        const float t = df * df;
        hi[i][j] = fmaf(wh, t, hi[i][j]);
        lo[i][j] = fmaf(wl, t, lo[i][j]);
      }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float e = __builtin_amdgcn_exp2f(-(hi[i][j] + lo[i][j]));
      val[i][j] = fmaf(a.a_lo, e, a.a_hi * e);
    }
}

__device__ __forceinline__ void load_points(const float* __restrict__ P, int d, int first, int valid,
                                            float (*sX)[TILE], int tid) {
  // sX[k][p] = P[(first + p) * d + k] for p < valid, else 0
  const int total = TILE * d;
  for (int idx = tid; idx < total; idx += 256) {
    const int p = idx / d, k = idx - p * d;
    sX[k][p] = p < valid ? P[(uint64_t)(first + p) * d + k] : 0.f;
  }
}

// Writes a computed tile (and its mirror image when off the diagonal of the tile grid).
// keep(p, q) decides which entries are stored as computed; the others become 0.
template <class Keep, class DiagVal>
__device__ __forceinline__ void store_tile(float* __restrict__ out, uint32_t ld, int p0, int q0, bool mirror,
                                           float (&val)[4][4], float (*sT)[TILE + 1], int ty, int tx, int tid,
                                           Keep keep, DiagVal diag) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int p = p0 + 4 * ty + i;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int q = q0 + 4 * tx + j;
      float v = keep(p, q) ? val[i][j] : 0.f;
      if (p == q) v = diag(p, v);
      val[i][j] = v;
    }
    *reinterpret_cast<float4*>(out + (uint64_t)p * ld + q0 + 4 * tx) =
        make_float4(val[i][0], val[i][1], val[i][2], val[i][3]);
  }
  if (mirror) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) sT[4 * ty + i][4 * tx + j] = val[i][j];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int q = 4 * ty + i;      // row of the mirrored tile
      *reinterpret_cast<float4*>(out + (uint64_t)(q0 + q) * ld + p0 + 4 * tx) =
          make_float4(sT[4 * tx + 0][q], sT[4 * tx + 1][q], sT[4 * tx + 2][q], sT[4 * tx + 3][q]);
    }
  }
}

__global__ __launch_bounds__(256) void k_build_diag(const PairArgs a, const ClusterInfo* __restrict__ cl,
                                                    const uint64_t* __restrict__ tiles,
                                                    const float* __restrict__ X, float* __restrict__ Kd) {
  __shared__ __attribute__((aligned(16))) float sX[2][MAX_D][TILE];
  float(*sXr)[TILE] = sX[0];
  float(*sXc)[TILE] = sX[1];
  const uint64_t t = tiles[blockIdx.x];
  const int ci = (int)(t >> 32), tr = (int)((t >> 16) & 0xffff), tc = (int)(t & 0xffff);
  const ClusterInfo c = cl[ci];
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int p0 = tr * TILE, q0 = tc * TILE;
  const int b = (int)c.b;
  load_points(X, a.d, (int)c.row0 + p0, min(TILE, b - p0), sXr, tid);
  load_points(X, a.d, (int)c.row0 + q0, min(TILE, b - q0), sXc, tid);
  __syncthreads();
  float val[4][4];
  pair_tile(a, sXr, sXc, ty, tx, val);
  float(*sT)[TILE + 1] = reinterpret_cast<float(*)[TILE + 1]>(&sX[0][0][0]);   // 64*65 floats, reused after the tile is in registers
  const float dv = a.diag_val;
  store_tile(Kd + c.koff, c.ld, p0, q0, tr != tc, val, sT, ty, tx, tid,
             [b](int p, int q) { return p < b && q < b; },
             [b, dv](int p, float v) { return p < b ? dv : v; });
}

__global__ __launch_bounds__(256) void k_build_coupling(const PairArgs a, const uint64_t* __restrict__ tiles,
                                                        const float* __restrict__ reps, float* __restrict__ C,
                                                        int ncr, int r, uint32_t ldc) {
  __shared__ __attribute__((aligned(16))) float sX[2][MAX_D][TILE];
  float(*sXr)[TILE] = sX[0];
  float(*sXc)[TILE] = sX[1];
  const uint64_t t = tiles[blockIdx.x];
  const int tr = (int)((t >> 16) & 0xffff), tc = (int)(t & 0xffff);
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int p0 = tr * TILE, q0 = tc * TILE;
  load_points(reps, a.d, p0, min(TILE, ncr - p0), sXr, tid);
  load_points(reps, a.d, q0, min(TILE, ncr - q0), sXc, tid);
  __syncthreads();
  float val[4][4];
  pair_tile(a, sXr, sXc, ty, tx, val);
  float(*sT)[TILE + 1] = reinterpret_cast<float(*)[TILE + 1]>(&sX[0][0][0]);
  // only blocks between DIFFERENT clusters enter K' (eq. (odsplit)): same-cluster entries are 0
  store_tile(C, ldc, p0, q0, tr != tc, val, sT, ty, tx, tid,
             [ncr, r](int p, int q) { return p < ncr && q < ncr && (p / r) != (q / r); },
             [](int, float v) { return v; });
}

// ---------------------------------------------------------------------------
// setup kernels (theta independent)
// ---------------------------------------------------------------------------
__global__ void k_gather_reps(const ClusterInfo* __restrict__ cl, const float* __restrict__ X,
                              float* __restrict__ reps, int r, int d, int nc) {
  const int64_t total = (int64_t)nc * r * d;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int k = (int)(idx % d);
    const int64_t pa = idx / d;
    const int a = (int)(pa % r), i = (int)(pa / r);
    reps[idx] = X[(uint64_t)(cl[i].row0 + a) * d + k];
  }
}

// One-hot nearest-representative basis.  The argmin is an integer decision, so the
// distances are accumulated in fp64 without contraction, in dimension order, exactly as a
// plain double-precision loop would: ties and near-ties resolve identically everywhere.
__global__ __launch_bounds__(256) void k_build_W(const ClusterInfo* __restrict__ cl, const float* __restrict__ X,
                                                 const float* __restrict__ reps, float* __restrict__ Wd,
                                                 float* __restrict__ Wt, int r, int d, uint32_t ldw) {
#pragma clang fp contract(off)
  const ClusterInfo c = cl[blockIdx.y];
  const int pl = blockIdx.x * blockDim.x + threadIdx.x;
  if (pl >= (int)c.b) return;
  const uint64_t p = (uint64_t)c.row0 + pl;
  const float* Ri = reps + (uint64_t)blockIdx.y * r * d;
  int best = 0;
  double bestd = 0.0;
  for (int a = 0; a < r; ++a) {
    double s = 0.0;
    for (int k = 0; k < d; ++k) {
      const double df = (double)X[p * d + k] - (double)Ri[(uint64_t)a * d + k];
      const double sq = df * df;
      s = s + sq;
    }
    if (a == 0 || s < bestd) { bestd = s; best = a; }
  }
  for (uint32_t a = 0; a < ldw; ++a) Wd[p * ldw + a] = ((int)a == best) ? 1.f : 0.f;
  for (int a = 0; a < r; ++a) Wt[c.wtoff + (uint64_t)a * c.ld + pl] = (a == best) ? 1.f : 0.f;
}

__global__ __launch_bounds__(256) void k_copy_W(const ClusterInfo* __restrict__ cl, const float* __restrict__ W,
                                                float* __restrict__ Wd, float* __restrict__ Wt, int r,
                                                uint32_t ldw) {
  const ClusterInfo c = cl[blockIdx.y];
  const int pl = blockIdx.x * blockDim.x + threadIdx.x;
  if (pl >= (int)c.b) return;
  const uint64_t p = (uint64_t)c.row0 + pl;
  for (uint32_t a = 0; a < ldw; ++a) Wd[p * ldw + a] = (int)a < r ? W[p * r + a] : 0.f;
  for (int a = 0; a < r; ++a) Wt[c.wtoff + (uint64_t)a * c.ld + pl] = W[p * r + a];
}

__global__ void k_fill(float* __restrict__ p, uint64_t n, float v) {
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
    p[i] = v;
}

// dense export with optional lower-triangle mask
__global__ void k_export(const float* __restrict__ src, uint64_t lds, float* __restrict__ dst, int64_t ldd,
                         int rows, int cols, int lower_only) {
  const int64_t total = (int64_t)rows * cols;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int p = (int)(idx / cols), q = (int)(idx - (int64_t)p * cols);
    float v = src[(uint64_t)p * lds + q];
    if (lower_only && q > p) v = 0.f;
    dst[(int64_t)p * ldd + q] = v;
  }
}

int launch_setup(nugpr_ctx* c, const float* user_reps, const float* user_W, hipStream_t s) {
  const Layout& L = c->L;
  // tile lists for the assembly kernels
  std::vector<uint64_t> tiles;
  tiles.reserve(L.n_diag_tiles + L.n_c_tiles);
  for (int i = 0; i < L.nc; ++i)
    for (uint32_t tr = 0; tr < L.cl[i].nt; ++tr)
      for (uint32_t tc = 0; tc <= tr; ++tc) tiles.push_back(((uint64_t)i << 32) | ((uint64_t)tr << 16) | tc);
  for (uint32_t tr = 0; tr < (uint32_t)(L.ldc / TILE); ++tr)
    for (uint32_t tc = 0; tc <= tr; ++tc) tiles.push_back(((uint64_t)tr << 16) | tc);
  NUGPR_HIP(hipMemcpyAsync(c->d_tiles, tiles.data(), tiles.size() * sizeof(uint64_t), hipMemcpyHostToDevice, s));
  NUGPR_HIP(hipStreamSynchronize(s));   // `tiles` is about to go out of scope
  // padding of Wt (columns b..ld of every row) must read as zero
  hipLaunchKernelGGL(k_fill, dim3(1024), dim3(256), 0, s, c->Wt, L.wt_elems, 0.f);
  if (user_reps) {
    NUGPR_HIP(hipMemcpyAsync(c->reps, user_reps, (size_t)L.ncr * L.d * sizeof(float), hipMemcpyDeviceToDevice, s));
  } else {
    hipLaunchKernelGGL(k_gather_reps, dim3(256), dim3(256), 0, s, c->d_cl, c->X, c->reps, L.r, L.d, L.nc);
  }
  uint32_t bmax = 0;
  for (auto& ci : L.cl) bmax = std::max(bmax, ci.b);
  dim3 grid((bmax + 255) / 256, L.nc);
  if (user_W)
    hipLaunchKernelGGL(k_copy_W, grid, dim3(256), 0, s, c->d_cl, user_W, c->Wd, c->Wt, L.r, (uint32_t)L.ldw);
  else
    hipLaunchKernelGGL(k_build_W, grid, dim3(256), 0, s, c->d_cl, c->X, c->reps, c->Wd, c->Wt, L.r, L.d,
                       (uint32_t)L.ldw);
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

int launch_build(nugpr_ctx* c, const double* theta, hipStream_t s) {
  const Layout& L = c->L;
  if (!theta) { set_error("theta is null"); return NUGPR_ERR_INVALID; }
  for (int i = 0; i < L.p; ++i)
    if (!(theta[i] > 0.0) || !std::isfinite(theta[i])) { set_error("theta entries must be finite and > 0"); return NUGPR_ERR_INVALID; }
  const bool iso = (c->params.flags & NUGPR_ISOTROPIC) != 0;
  const double alpha = theta[L.p - 2], sigma2 = theta[L.p - 1];
  PairArgs a;
  const double half_log2e = 0.5 * 1.4426950408889634074;
  for (int k = 0; k < MAX_D; ++k) { a.w_hi[k] = 0.f; a.w_lo[k] = 0.f; }
  for (int k = 0; k < L.d; ++k) {
    const double ell = iso ? theta[0] : theta[k];
    const double w = half_log2e / (ell * ell);
    a.w_hi[k] = (float)w;
    a.w_lo[k] = (float)(w - (double)a.w_hi[k]);
  }
  a.a_hi = (float)alpha;
  a.a_lo = (float)(alpha - (double)a.a_hi);
  a.diag_val = (float)(alpha + sigma2);
  a.d = L.d;
  c->diag_residual = (float)((alpha + sigma2) - (double)a.diag_val);
  hipLaunchKernelGGL(k_build_diag, dim3((unsigned)L.n_diag_tiles), dim3(256), 0, s, a, c->d_cl, c->d_tiles, c->X, c->Kd);
  hipLaunchKernelGGL(k_build_coupling, dim3((unsigned)L.n_c_tiles), dim3(256), 0, s, a, c->d_tiles + L.n_diag_tiles,
                     c->reps, c->C, L.ncr, L.r, (uint32_t)L.ldc);
  NUGPR_HIP(hipGetLastError());
  c->built = true;
  return NUGPR_OK;
}

int launch_export(nugpr_ctx* c, int what, int index, float* dst, int64_t ld, hipStream_t s) {
  const Layout& L = c->L;
  if (!dst) { set_error("dst is null"); return NUGPR_ERR_INVALID; }
  const float* src = nullptr;
  uint64_t lds = 0;
  int rows = 0, cols = 0, lower = 0;
  if (what >= 0 && what <= 2) {
    if (index < 0 || index >= L.nc) { set_error("cluster index out of range"); return NUGPR_ERR_INVALID; }
    const ClusterInfo& ci = L.cl[index];
    src = (what == 0 ? c->Kd : what == 1 ? c->Lf : c->G) + ci.koff;
    lds = ci.ld; rows = cols = (int)ci.b; lower = what != 0;
    if ((what == 0 && !c->built) || (what != 0 && !c->factored)) { set_error("nothing stored yet"); return NUGPR_ERR_STATE; }
  } else if (what == 3) {
    if (!c->built) { set_error("nothing stored yet"); return NUGPR_ERR_STATE; }
    src = c->C; lds = L.ldc; rows = cols = L.ncr;
  } else if (what == 4) {
    if (index < 0 || index >= L.nc) { set_error("cluster index out of range"); return NUGPR_ERR_INVALID; }
    src = c->Wd + (uint64_t)L.cl[index].row0 * L.ldw; lds = L.ldw; rows = (int)L.cl[index].b; cols = L.r;
  } else if (what == 5) {
    if (!c->factored) { set_error("nothing stored yet"); return NUGPR_ERR_STATE; }
    src = c->Bv; lds = L.T; rows = (int)L.n; cols = L.T;
  } else if (what == 6) {
    src = c->reps; lds = L.d; rows = L.ncr; cols = L.d;
  } else { set_error("unknown export selector"); return NUGPR_ERR_INVALID; }
  if (ld < cols) { set_error("ld smaller than the number of columns"); return NUGPR_ERR_INVALID; }
  hipLaunchKernelGGL(k_export, dim3(2048), dim3(256), 0, s, src, lds, dst, ld, rows, cols, lower);
  NUGPR_HIP(hipGetLastError());
  NUGPR_HIP(hipStreamSynchronize(s));
  return NUGPR_OK;
}

}  // namespace nugpr
