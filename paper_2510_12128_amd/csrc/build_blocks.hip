// Block assembly (Section 2.1 kernel, K_diag of Section 3.2, representative-point
// coupling of Section 3.3) and the theta-independent setup (representatives, basis W).
//
// Entries are STORED in fp32 but COMPUTED in fp64 and rounded once.  The loss is
// differenced over hyperparameter steps of 1e-3, and each probe's quadratic form
// z^T log(.) z weighs the entry errors by the (large) entries of L^-T z, so an entry error
// of a few fp32 ulps -- what an fp32 distance accumulation followed by the hardware exp
// gives -- shows up as 1e-4-level noise in the gradient.
//
// In fp64 the squared distance CAN be taken as |u|^2 + |v|^2 - 2 u.v (u, v the coordinates
// scaled by sqrt(w_k), w_k = log2(e) / (2 ell_k^2)): the cancellation costs ~1e-13 of the
// exponent, far below the fp32 rounding of the result.  That turns the O(b^2 d) part into a
// Gram matrix on the fp64 matrix cores (v_mfma_f64_16x16x4_f64) and leaves only the
// exponential (a degree-9 polynomial after range reduction) on the vector ALUs.
// The part of alpha + sigma^2 that the fp32 diagonal cannot hold is kept as a scalar and
// added by the matrix-vector product (StripPort::diag_add).
#include <algorithm>
#include <cmath>
#include <vector>

#include "nugpr_internal.h"

namespace nugpr {

typedef double v4d __attribute__((ext_vector_type(4)));

struct PairArgs {
  double sw[MAX_D];     // sqrt(log2(e) / (2 ell_k^2)): coordinate scale per dimension
  double alpha;
  float diag_val;       // float(alpha + sigma^2)
  int32_t d;
};

// 2^(-a) in fp64: a = n + f, |f| <= 1/2, 2^-f by its Taylor series in g = -f ln 2
// (degree 9 at |g| <= 0.347: relative error < 1e-11), scaled by 2^-n.
__device__ __forceinline__ double exp2_neg(double a) {
  const double n = rint(a);
  const double g = (n - a) * 0.69314718055994530942;
  double p = 1.0 / 362880.0;
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

// LDS layout (dynamic): two [kd][64] fp64 panels of scaled coordinates (kd = d rounded up to
// 4, the padding rows zero), two [64] fp64 squared norms, and a 64 x 65 fp32 staging tile.
__host__ __device__ inline int pair_kd(int d) { return (d + 3) & ~3; }
__host__ __device__ inline size_t pair_lds_bytes(int d) {
  return (size_t)2 * pair_kd(d) * TILE * sizeof(double) + 2 * TILE * sizeof(double) +
         (size_t)TILE * (TILE + 1) * sizeof(float);
}
constexpr int MAX_PT = MAX_D / 4;     // coordinates one thread holds for one 64-point panel

// Thread t holds coordinates k = (t % 4) + 4 e, e < kd / 4, of point t / 4 of a 64-point panel.
__device__ __forceinline__ void fetch_points(const float* __restrict__ P, int d, int kd, int first, int valid,
                                             int tid, float (&reg)[MAX_PT]) {
  const int p = tid >> 2, sub = tid & 3;
#pragma unroll
  for (int e = 0; e < MAX_PT; ++e) {
    const int k = sub + 4 * e;
    reg[e] = (e * 4 < kd && p < valid && k < d) ? P[(uint64_t)(first + p) * d + k] : 0.f;
  }
}

// sX[k][p] = sw[k] * x_pk (zero in the padding), sN[p] = sum_k sX[k][p]^2
__device__ __forceinline__ void commit_points(const PairArgs& a, int kd, const float (&reg)[MAX_PT],
                                              double (*sX)[TILE], double* sN, int tid) {
  const int p = tid >> 2, sub = tid & 3;
  double nrm = 0.0;
#pragma unroll
  for (int e = 0; e < MAX_PT; ++e) {
    if (e * 4 < kd) {
      const int k = sub + 4 * e;
      const double v = a.sw[k] * (double)reg[e];
      sX[k][p] = v;
      nrm = fma(v, v, nrm);
    }
  }
  nrm += __shfl_xor(nrm, 1);
  nrm += __shfl_xor(nrm, 2);
  if (sub == 0) sN[p] = nrm;
}

// 64 x 64 tile of alpha * 2^(-|u_r - v_c|^2): wave w owns rows 16w..16w+15; val[tj][i] is the
// entry at row 16w + (lane/16) + 4i, column 16 tj + lane%16 (the f64 16x16x4 accumulator layout).
__device__ __forceinline__ void pair_tile(const PairArgs& a, const double (*sXr)[TILE], const double (*sXc)[TILE],
                                          const double* sNr, const double* sNc, int wave, int lane,
                                          float (&val)[4][4]) {
  v4d acc[4];
#pragma unroll
  for (int tj = 0; tj < 4; ++tj) acc[tj] = (v4d){0.0, 0.0, 0.0, 0.0};
  const int m = lane & 15, kk = lane >> 4;
  const int kd = pair_kd(a.d);
  for (int ks = 0; ks < kd; ks += 4) {
    const double av = sXr[ks + kk][16 * wave + m];
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
      const double bv = sXc[ks + kk][16 * tj + m];
      acc[tj] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc[tj], 0, 0, 0);
    }
  }
#pragma unroll
  for (int tj = 0; tj < 4; ++tj) {
    const double nc = sNc[16 * tj + m];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double nr = sNr[16 * wave + kk + 4 * i];
      const double arg = fma(-2.0, acc[tj][i], nr + nc);
      val[tj][i] = (float)(a.alpha * exp2_neg(arg));
    }
  }
}

// Writes the staged tile (and its mirror image when off the diagonal of the tile grid) with
// 16-byte stores.  keep(p, q) decides which entries are stored as computed (the others
// become 0); diag(p, v) replaces diagonal entries.
template <class Keep, class DiagVal>
__device__ __forceinline__ void store_tile(float* __restrict__ out, uint32_t ld, int p0, int q0, bool mirror,
                                           const float (*sT)[TILE + 1], int tid, Keep keep, DiagVal diag) {
  const int r = tid >> 2, c0 = (tid & 3) * 16;     // this thread writes 16 consecutive entries of one row
  {
    const int p = p0 + r;
#pragma unroll
    for (int j4 = 0; j4 < 4; ++j4) {
      float v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int q = q0 + c0 + 4 * j4 + j;
        float x = keep(p, q) ? sT[r][c0 + 4 * j4 + j] : 0.f;
        if (p == q) x = diag(p, x);
        v[j] = x;
      }
      *reinterpret_cast<float4*>(out + (uint64_t)p * ld + q0 + c0 + 4 * j4) = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
  if (mirror) {
    const int q = q0 + r;                          // row of the mirrored tile
#pragma unroll
    for (int j4 = 0; j4 < 4; ++j4) {
      float v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int p = p0 + c0 + 4 * j4 + j;
        v[j] = keep(p, q) ? sT[c0 + 4 * j4 + j][r] : 0.f;
      }
      *reinterpret_cast<float4*>(out + (uint64_t)q * ld + p0 + c0 + 4 * j4) = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
}

// One work item = tile row `tr` of one square symmetric matrix (a cluster's K_ii, or the
// coupling C) and the run of tile columns tc0..tc1-1 (<= tr): the row panel's coordinates
// are staged once, the column panels stream through with the next one prefetched in
// registers while the current tile is computed, staged and written (with its mirror).
// item = cluster << 48 | tr << 32 | tc0 << 16 | tc1.
template <bool COUPLING>
__global__ __launch_bounds__(256) void k_build_panel(const PairArgs a, const ClusterInfo* __restrict__ cl,
                                                     const uint64_t* __restrict__ items,
                                                     const float* __restrict__ P, float* __restrict__ out_base,
                                                     int ncr, int r, uint32_t ldc) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const int d = a.d, kd = pair_kd(d);
  double(*sXr)[TILE] = reinterpret_cast<double(*)[TILE]>(lds_raw);
  double(*sXc)[TILE] = sXr + kd;
  double* sNr = reinterpret_cast<double*>(sXc + kd);
  double* sNc = sNr + TILE;
  float(*sT)[TILE + 1] = reinterpret_cast<float(*)[TILE + 1]>(sNc + TILE);

  const uint64_t it = items[blockIdx.x];
  const int ci = (int)(it >> 48), tr = (int)((it >> 32) & 0xffff), tc0 = (int)((it >> 16) & 0xffff),
            tc1 = (int)(it & 0xffff);
  int first, total;
  uint32_t ld;
  float* out;
  if (COUPLING) {
    first = 0; total = ncr; ld = ldc; out = out_base;
  } else {
    const ClusterInfo c = cl[ci];
    first = (int)c.row0; total = (int)c.b; ld = c.ld; out = out_base + c.koff;
  }
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int p0 = tr * TILE;
  float reg[MAX_PT];
  fetch_points(P, d, kd, first + p0, min(TILE, total - p0), tid, reg);
  commit_points(a, kd, reg, sXr, sNr, tid);
  fetch_points(P, d, kd, first + tc0 * TILE, min(TILE, total - tc0 * TILE), tid, reg);
  const float dv = a.diag_val;
  for (int tc = tc0; tc < tc1; ++tc) {
    const int q0 = tc * TILE;
    commit_points(a, kd, reg, sXc, sNc, tid);
    __syncthreads();
    if (tc + 1 < tc1) fetch_points(P, d, kd, first + q0 + TILE, min(TILE, total - q0 - TILE), tid, reg);
    float val[4][4];
    pair_tile(a, sXr, sXc, sNr, sNc, wave, lane, val);
#pragma unroll
    for (int tj = 0; tj < 4; ++tj)
#pragma unroll
      for (int i = 0; i < 4; ++i) sT[16 * wave + (lane >> 4) + 4 * i][16 * tj + (lane & 15)] = val[tj][i];
    __syncthreads();
    if (COUPLING) {
      // only blocks between DIFFERENT clusters enter K' (eq. (odsplit)): same-cluster entries are 0
      store_tile(out, ld, p0, q0, tr != tc, sT, tid,
                 [total, r](int p, int q) { return p < total && q < total && (p / r) != (q / r); },
                 [](int, float v) { return v; });
    } else {
      store_tile(out, ld, p0, q0, tr != tc, sT, tid,
                 [total](int p, int q) { return p < total && q < total; },
                 [total, dv](int p, float v) { return p < total ? dv : v; });
    }
  }
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
  // tile list of the diagonal blocks (used when the inverse factor is mirrored) and the
  // row-panel work items of the two assembly launches, longest first
  std::vector<uint64_t> tiles;
  tiles.reserve(2 * L.n_diag_tiles + L.n_c_tiles);
  for (int i = 0; i < L.nc; ++i)
    for (uint32_t tr = 0; tr < L.cl[i].nt; ++tr)
      for (uint32_t tc = 0; tc <= tr; ++tc) tiles.push_back(((uint64_t)i << 32) | ((uint64_t)tr << 16) | tc);
  constexpr uint32_t MAXT = 16;          // tiles per work item
  auto panel_items = [&](uint32_t nt, uint64_t ci, std::vector<uint64_t>& v) {
    for (uint32_t tr = 0; tr < nt; ++tr)
      for (uint32_t t0 = 0; t0 <= tr; t0 += MAXT)
        v.push_back((ci << 48) | ((uint64_t)tr << 32) | ((uint64_t)t0 << 16) | std::min<uint32_t>(t0 + MAXT, tr + 1));
  };
  auto by_length = [](uint64_t x, uint64_t y) {
    return ((x & 0xffff) - ((x >> 16) & 0xffff)) > ((y & 0xffff) - ((y >> 16) & 0xffff));
  };
  std::vector<uint64_t> pd, pc;
  for (int i = 0; i < L.nc; ++i) panel_items(L.cl[i].nt, (uint64_t)i, pd);
  panel_items((uint32_t)(L.ldc / TILE), 0, pc);
  std::stable_sort(pd.begin(), pd.end(), by_length);
  std::stable_sort(pc.begin(), pc.end(), by_length);
  c->n_pan_diag = (int)pd.size();
  c->n_pan_c = (int)pc.size();
  c->d_pan_diag = c->d_tiles + tiles.size();
  c->d_pan_c = c->d_pan_diag + pd.size();
  tiles.insert(tiles.end(), pd.begin(), pd.end());
  tiles.insert(tiles.end(), pc.begin(), pc.end());
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
  for (int k = 0; k < MAX_D; ++k) a.sw[k] = 0.0;
  for (int k = 0; k < L.d; ++k) {
    const double ell = iso ? theta[0] : theta[k];
    a.sw[k] = std::sqrt(half_log2e) / ell;
  }
  a.alpha = alpha;
  a.diag_val = (float)(alpha + sigma2);
  a.d = L.d;
  c->diag_residual = (float)((alpha + sigma2) - (double)a.diag_val);
  const size_t lds = pair_lds_bytes(L.d);
  hipLaunchKernelGGL((k_build_panel<false>), dim3((unsigned)c->n_pan_diag), dim3(256), lds, s, a, c->d_cl, c->d_pan_diag,
                     c->X, c->Kd, 0, 1, 0u);
  hipLaunchKernelGGL((k_build_panel<true>), dim3((unsigned)c->n_pan_c), dim3(256), lds, s, a, c->d_cl, c->d_pan_c,
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
