// Block assembly (Section 2.1 kernel, K_diag of Section 3.2, representative-point
// coupling of Section 3.3) and the theta-independent setup (representatives, basis W).
//
// Entries are STORED in fp32 but COMPUTED in fp64 and rounded once.  The loss is
// differenced over hyperparameter steps of 1e-3, and each probe's quadratic form
// z^T log(.) z weighs the entry errors by the (large) entries of L^-T z, so an entry error
// of a few fp32 ulps -- what an fp32 distance accumulation followed by the hardware exp
// gives -- shows up as 1e-4-level noise in the gradient.  On CDNA the fp64 vector FMA
// runs at the rate of the unpacked fp32 FMA, so the exact form costs no more than an fp32
// (hi, lo) split would: per pair and dimension one subtract, one multiply, one FMA.
//
// Squared distances use the direct difference form sum_k w_k (x_pk - x_qk)^2 on the
// vector ALUs; the |x|^2 + |x'|^2 - 2 x.x' contraction would put this on the matrix
// cores but cancels catastrophically.  The part of alpha + sigma^2 that the fp32 diagonal
// cannot hold is kept as a scalar and added by the matrix-vector product
// (StripPort::diag_add).
#include <cmath>
#include <vector>

#include "nugpr_internal.h"

namespace nugpr {

struct PairArgs {
  double w[MAX_D];      // log2(e) / (2 ell_k^2)
  double alpha;
  float diag_val;       // float(alpha + sigma^2)
  int32_t d;
};

// 2^(-a) for a >= 0 in fp64: a = n + f, |f| <= 1/2, 2^-f by its Taylor series in f ln 2
// (degree 10: relative error < 1e-13), scaled by 2^-n.
__device__ __forceinline__ double exp2_neg(double a) {
  const double n = rint(a);
  const double g = (n - a) * 0.69314718055994530942;      // -f ln 2, |g| <= 0.3466
  double p = 1.0 / 3628800.0;
  p = fma(p, g, 1.0 / 362880.0);
  p = fma(p, g, 1.0 / 40320.0);
  p = fma(p, g, 1.0 / 5040.0);
  p = fma(p, g, 1.0 / 720.0);
  p = fma(p, g, 1.0 / 120.0);
  p = fma(p, g, 1.0 / 24.0);
  p = fma(p, g, 1.0 / 6.0);
  p = fma(p, g, 0.5);
  p = fma(p, g, 1.0);
  p = fma(p, g, 1.0);
  const int e = n > 2000.0 ? -2000 : -(int)n;
  return ldexp(p, e);
}

// 64x64 tile of alpha * 2^(-sum_k w_k (xr_k - xc_k)^2); thread (ty, tx) holds a 4x4 patch.
// sXr / sXc: coordinates of the 64 row / column points widened to fp64, layout [k][64].
__device__ __forceinline__ void pair_tile(const PairArgs& a, const double (*sXr)[TILE], const double (*sXc)[TILE],
                                          int ty, int tx, float (&val)[4][4]) {
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
  for (int k = 0; k < a.d; ++k) {
    const double w = a.w[k];
    double r_[4], c_[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { r_[i] = sXr[k][4 * ty + i]; c_[i] = sXc[k][4 * tx + i]; }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const double df = r_[i] - c_[j];
        acc[i][j] = fma(w, df * df, acc[i][j]);
      }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) val[i][j] = (float)(a.alpha * exp2_neg(acc[i][j]));
}

__device__ __forceinline__ void load_points(const float* __restrict__ P, int d, int first, int valid,
                                            double (*sX)[TILE], int tid) {
  // sX[k][p] = P[(first + p) * d + k] for p < valid, else 0
  const int total = TILE * d;
  for (int idx = tid; idx < total; idx += 256) {
    const int p = idx / d, k = idx - p * d;
    sX[k][p] = p < valid ? (double)P[(uint64_t)(first + p) * d + k] : 0.0;
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

// dynamic LDS: two [d][64] fp64 coordinate panels, reused as a 64 x 65 fp32 transpose buffer
__host__ __device__ inline size_t pair_lds_bytes(int d) {
  const size_t panels = (size_t)2 * d * TILE * sizeof(double);
  const size_t transp = (size_t)TILE * (TILE + 1) * sizeof(float);
  return panels > transp ? panels : transp;
}

__global__ __launch_bounds__(256) void k_build_diag(const PairArgs a, const ClusterInfo* __restrict__ cl,
                                                    const uint64_t* __restrict__ tiles,
                                                    const float* __restrict__ X, float* __restrict__ Kd) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  double(*sXr)[TILE] = reinterpret_cast<double(*)[TILE]>(lds_raw);
  double(*sXc)[TILE] = sXr + a.d;
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
  float(*sT)[TILE + 1] = reinterpret_cast<float(*)[TILE + 1]>(lds_raw);   // reused once the tile is in registers
  const float dv = a.diag_val;
  store_tile(Kd + c.koff, c.ld, p0, q0, tr != tc, val, sT, ty, tx, tid,
             [b](int p, int q) { return p < b && q < b; },
             [b, dv](int p, float v) { return p < b ? dv : v; });
}

__global__ __launch_bounds__(256) void k_build_coupling(const PairArgs a, const uint64_t* __restrict__ tiles,
                                                        const float* __restrict__ reps, float* __restrict__ C,
                                                        int ncr, int r, uint32_t ldc) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  double(*sXr)[TILE] = reinterpret_cast<double(*)[TILE]>(lds_raw);
  double(*sXc)[TILE] = sXr + a.d;
  const uint64_t t = tiles[blockIdx.x];
  const int tr = (int)((t >> 16) & 0xffff), tc = (int)(t & 0xffff);
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int p0 = tr * TILE, q0 = tc * TILE;
  load_points(reps, a.d, p0, min(TILE, ncr - p0), sXr, tid);
  load_points(reps, a.d, q0, min(TILE, ncr - q0), sXc, tid);
  __syncthreads();
  float val[4][4];
  pair_tile(a, sXr, sXc, ty, tx, val);
  float(*sT)[TILE + 1] = reinterpret_cast<float(*)[TILE + 1]>(lds_raw);
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
template <typename ST>
__global__ void k_export(const ST* __restrict__ src, uint64_t lds, float* __restrict__ dst, int64_t ldd,
                         int rows, int cols, int lower_only) {
  const int64_t total = (int64_t)rows * cols;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int p = (int)(idx / cols), q = (int)(idx - (int64_t)p * cols);
    float v = (float)src[(uint64_t)p * lds + q];
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
  for (int k = 0; k < MAX_D; ++k) a.w[k] = 0.0;
  for (int k = 0; k < L.d; ++k) {
    const double ell = iso ? theta[0] : theta[k];
    a.w[k] = half_log2e / (ell * ell);
  }
  a.alpha = alpha;
  a.diag_val = (float)(alpha + sigma2);
  a.d = L.d;
  c->diag_residual = (float)((alpha + sigma2) - (double)a.diag_val);
  const size_t lds = pair_lds_bytes(L.d);
  hipLaunchKernelGGL(k_build_diag, dim3((unsigned)L.n_diag_tiles), dim3(256), lds, s, a, c->d_cl, c->d_tiles, c->X, c->Kd);
  hipLaunchKernelGGL(k_build_coupling, dim3((unsigned)L.n_c_tiles), dim3(256), lds, s, a, c->d_tiles + L.n_diag_tiles,
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
    src = nullptr; lds = L.T; rows = (int)L.n; cols = L.T;
  } else if (what == 6) {
    src = c->reps; lds = L.d; rows = L.ncr; cols = L.d;
  } else { set_error("unknown export selector"); return NUGPR_ERR_INVALID; }
  if (ld < cols) { set_error("ld smaller than the number of columns"); return NUGPR_ERR_INVALID; }
  if (what == 5 && c->acc64)
    hipLaunchKernelGGL((k_export<double>), dim3(2048), dim3(256), 0, s, (const double*)c->Bv, lds, dst, ld, rows, cols, lower);
  else
    hipLaunchKernelGGL((k_export<float>), dim3(2048), dim3(256), 0, s, what == 5 ? (const float*)c->Bv : src, lds, dst, ld,
                       rows, cols, lower);
  NUGPR_HIP(hipGetLastError());
  NUGPR_HIP(hipStreamSynchronize(s));
  return NUGPR_OK;
}

}  // namespace nugpr
