// Batched preconditioned CG (Sections 3.1-3.2; the vector operations of Tables 1-2) and
// the two operator applications it alternates: the block-low-rank product K' D and the
// block-Jacobi preconditioner M^-1 R.
//
// All T columns advance in lock step.  Vector blocks are n x T row-major, fp64 or fp32
// according to the context's arithmetic mode (VT below); every reduction that feeds a CG
// coefficient (the paper's batched dot products) is accumulated in fp64 in a fixed order:
// per-workgroup partial sums, then one small kernel that adds them, computes alpha / beta
// per column and updates the convergence mask on the device.  The host reads back one
// 16-byte flag record per iteration (O(1) traffic, Section 4).
#include <algorithm>
#include <cmath>
#include <cstring>

#include "nugpr_internal.h"

namespace nugpr {

// ---------------------------------------------------------------------------
// per-column dot products: partial[which][block][col] = sum over the block's rows
// ---------------------------------------------------------------------------
template <int NP, typename VT>
__global__ __launch_bounds__(256) void k_dot(const VT* __restrict__ A0, const VT* __restrict__ B0,
                                             const VT* __restrict__ A1, const VT* __restrict__ B1,
                                             int64_t n, int T, double* __restrict__ partial) {
  __shared__ double red[NP][256];
  const int rpp = 256 / T;                      // rows per pass
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
      s0 = fma((double)A0[idx], (double)B0[idx], s0);
      if (NP > 1) s1 = fma((double)A1[idx], (double)B1[idx], s1);
    }
  }
  red[0][tid] = s0;
  if (NP > 1) red[NP - 1][tid] = s1;
  __syncthreads();
  if (tid < T) {
    for (int w = 0; w < NP; ++w) {
      double s = 0.0;
      for (int k = 0; k < rpp; ++k) s += red[w][k * T + tid];
      partial[((int64_t)w * gridDim.x + blockIdx.x) * MAX_COLS + tid] = s;
    }
  }
}

// sum over the 64 lanes of a wave by register shuffles, fixed pairing (lane, lane + 32), (lane, lane + 16), ..;
// lane 0 holds the result
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

__device__ __forceinline__ double sum_partials(const double* __restrict__ partial, int nblocks, int col,
                                               double* red, int tid) {
  // 256 threads cooperate on one column at a time, fixed order: strided partial sums per thread, shuffles
  // inside each wave, then the four wave totals through LDS
  double s = 0.0;
  for (int b = tid; b < nblocks; b += 256) s += partial[(int64_t)b * MAX_COLS + col];
  s = wave_sum(s);
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  const double r = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  return r;
}

// The three scalar kernels run one workgroup per column (grid = T); the cross-column
// bookkeeping (how many columns are still active, did any meet negative curvature) is
// gathered by the last workgroup of the stop test (k_pcg_check).

// start of a solve: ||b||^2 and rho_0 = <r_0, z_0>
__global__ __launch_bounds__(256) void k_pcg_begin(PcgState* __restrict__ st, const double* __restrict__ partial,
                                                   int nblocks) {
  __shared__ double red[256];
  const int tid = threadIdx.x, c = blockIdx.x;
  const double bb = sum_partials(partial, nblocks, c, red, tid);
  const double rz = sum_partials(partial + (int64_t)nblocks * MAX_COLS, nblocks, c, red, tid);
  if (tid == 0) {
    const bool act = bb > 0.0 && rz == rz;
    st->bnorm2[c] = bb;
    st->rho[c] = rz;
    st->rho0[c] = rz;
    st->alpha[c] = 0.0;
    st->beta[c] = 0.0;
    st->active[c] = act ? 1 : 0;
    st->iters[c] = 0;
    st->converged[c] = (bb == 0.0) ? 1 : 0;
    st->indef[c] = 0;
  }
}

// the same from the values kept with the factor (which = 0: [y | L Z], 1: the probe block)
__global__ void k_pcg_begin_known(PcgState* __restrict__ st, int which, int T) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= T) return;
  const double bb = st->known_bb[which][c], rz = st->known_rz[which][c];
  const bool act = bb > 0.0 && rz == rz;
  st->bnorm2[c] = bb;
  st->rho[c] = rz;
  st->rho0[c] = rz;
  st->alpha[c] = 0.0;
  st->beta[c] = 0.0;
  st->active[c] = act ? 1 : 0;
  st->iters[c] = 0;
  st->converged[c] = (bb == 0.0) ? 1 : 0;
  st->indef[c] = 0;
}

__global__ __launch_bounds__(256) void k_store_known(PcgState* __restrict__ st, const double* __restrict__ partial,
                                                     int nblocks, int which) {
  __shared__ double red[256];
  const int tid = threadIdx.x, c = blockIdx.x;
  const double bb = sum_partials(partial, nblocks, c, red, tid);
  const double rz = sum_partials(partial + (int64_t)nblocks * MAX_COLS, nblocks, c, red, tid);
  if (tid == 0) { st->known_bb[which][c] = bb; st->known_rz[which][c] = rz; }
}

// alpha_c = rho_c / <d, K'd>_c for the active columns
__global__ __launch_bounds__(256) void k_pcg_alpha(PcgState* __restrict__ st, const double* __restrict__ partial,
                                                   int nblocks, int iter, double* __restrict__ alog) {
  __shared__ double red[256];
  const int tid = threadIdx.x, c = blockIdx.x;
  const double dq = sum_partials(partial, nblocks, c, red, tid);
  if (tid == 0) {
    double a = 0.0;
    if (st->active[c]) {
      if (dq > 0.0) a = st->rho[c] / dq;
      else { st->indef[c] = 1; st->active[c] = 0; }      // <d, K'd> <= 0 (or NaN)
    }
    st->alpha[c] = a;
    alog[(int64_t)iter * MAX_COLS + c] = a;
  }
}

// after the update: stop test on ||r_c|| (columns that meet it are frozen).  The workgroup that finishes
// last gathers the cross-column bookkeeping (how many columns are still active, did any meet negative
// curvature) and publishes it to the host: the flags, a system-scope fence, then the sequence number.
__global__ __launch_bounds__(256) void k_pcg_check(PcgState* __restrict__ st, const double* __restrict__ partial,
                                                   int nblocks, int iter, double tol2, int T,
                                                   HostFlags* __restrict__ out, uint64_t seq) {
  __shared__ double red[256];
  __shared__ int last;
  const int tid = threadIdx.x, c = blockIdx.x;
  const double rr = sum_partials(partial, nblocks, c, red, tid);
  if (tid == 0) {
    if (st->active[c]) {
      st->iters[c] = iter + 1;
      if (rr <= tol2 * st->bnorm2[c]) {
        st->active[c] = 0;
        st->converged[c] = 1;
      } else if (!(rr == rr)) {                // NaN residual: stop this column
        st->active[c] = 0;
        st->indef[c] = 1;
      }
    }
    __threadfence();
    last = (atomicAdd(&st->check_count, 1) == T - 1);
  }
  __syncthreads();
  if (last && tid == 0) {
    __threadfence();
    int n_active = 0, indef = 0;
    for (int k = 0; k < T; ++k) {
      n_active += *reinterpret_cast<volatile int32_t*>(&st->active[k]);
      indef |= *reinterpret_cast<volatile int32_t*>(&st->indef[k]);
    }
    st->check_count = 0;
    st->n_active = n_active;
    st->indefinite = indef;
    out->n_active = n_active;
    out->indefinite = indef;
    out->bad_cluster = st->bad_cluster;
    __threadfence_system();
    *reinterpret_cast<volatile uint64_t*>(&out->seq) = seq;
  }
}

// beta_c = <r, z>_new / rho_c for the columns that go on
__global__ __launch_bounds__(256) void k_pcg_beta(PcgState* __restrict__ st, const double* __restrict__ partial,
                                                  int nblocks, int iter, double* __restrict__ blog) {
  __shared__ double red[256];
  const int tid = threadIdx.x, c = blockIdx.x;
  const double rz = sum_partials(partial, nblocks, c, red, tid);
  if (tid == 0) {
    double bta = 0.0;
    if (st->active[c]) {
      if (!(rz > 0.0)) {                     // preconditioned residual lost positivity (or NaN)
        st->active[c] = 0;
        st->indef[c] = 1;
      } else {
        bta = rz / st->rho[c];
        st->rho[c] = rz;
      }
    }
    st->beta[c] = bta;
    blog[(int64_t)iter * MAX_COLS + c] = bta;
  }
}

// X += D diag(alpha); R -= Q diag(alpha)   (alpha stays in fp64: rounding it to fp32 would scale the whole
// step coherently).  In the first step of a solve X starts from zero and R from Rin = b, neither of which is
// read or written before.  The update is fused with the two reductions that follow it: partial[0] = per-workgroup sums of r_new^2
// (the stop test) and, when B is given, partial[1] = sums of b x_new (the quadratic form of the end-of-solve
// report).  Rows are split among the workgroups as in k_dot, so the sums are those k_dot would produce.
template <typename VT>
__global__ __launch_bounds__(256) void k_update_xr_dots(VT* __restrict__ X, VT* R, const VT* Rin,
                                                        const VT* __restrict__ D, const VT* __restrict__ Q,
                                                        const VT* __restrict__ B, const PcgState* __restrict__ st,
                                                        int64_t n, int T, int first, double* __restrict__ partial) {
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
    const double a = st->alpha[col];
    for (int64_t r = r0 + myrow; r < r1; r += rpp) {
      const int64_t idx = r * T + col;
      const VT xn = first ? (VT)(a * (double)D[idx]) : (VT)fma(a, (double)D[idx], (double)X[idx]);
      const VT rn = (VT)fma(-a, (double)Q[idx], (double)Rin[idx]);
      X[idx] = xn;
      R[idx] = rn;
      s0 = fma((double)rn, (double)rn, s0);
      if (B) s1 = fma((double)B[idx], (double)xn, s1);
    }
  }
  red[0][tid] = s0;
  red[1][tid] = s1;
  __syncthreads();
  if (tid < T) {
    for (int w = 0; w < 2; ++w) {
      double sacc = 0.0;
      for (int k = 0; k < rpp; ++k) sacc += red[w][k * T + tid];
      partial[((int64_t)w * gridDim.x + blockIdx.x) * MAX_COLS + tid] = sacc;
    }
  }
}

// D = Z + D diag(beta) for active columns, 0 for stopped ones
template <typename VT>
__global__ __launch_bounds__(256) void k_update_d(VT* D, const VT* Din, const VT* __restrict__ Z,
                                                  const PcgState* __restrict__ st, int64_t n, int T) {
  const int rpp = 256 / T;
  const int tid = threadIdx.x;
  const int myrow = tid / T, col = tid - myrow * T;
  if (myrow >= rpp) return;
  const double bta = st->beta[col];
  const bool act = st->active[col] != 0;
  for (int64_t r = (int64_t)blockIdx.x * rpp + myrow; r < n; r += (int64_t)gridDim.x * rpp) {
    const int64_t idx = r * T + col;
    D[idx] = act ? (VT)fma(bta, (double)Din[idx], (double)Z[idx]) : (VT)0;
  }
}

// End-of-solve report, written by the device straight into pinned host memory: the per-column state,
// <b_c, x_c> summed from the per-workgroup partials (fixed order), and the first `rows` rows of the
// alpha / beta logs.  One workgroup per column (each sums its column; they share the copies); the
// workgroup that finishes last publishes the sequence number.
__global__ __launch_bounds__(256) void k_pcg_tail(PcgState* __restrict__ st, const double* __restrict__ partial,
                                                  int nblocks, int T, int want_bx, const double* __restrict__ alog,
                                                  const double* __restrict__ blog, int rows,
                                                  PcgState* __restrict__ h_state, double* __restrict__ h_bx,
                                                  double* __restrict__ h_alog, double* __restrict__ h_blog,
                                                  HostFlags* __restrict__ flags, uint64_t seq) {
  __shared__ double red[256];
  __shared__ int last;
  const int tid = threadIdx.x, c = blockIdx.x;
  if (want_bx) {
    const double v = sum_partials(partial, nblocks, c, red, tid);
    if (tid == 0) h_bx[c] = v;
  }
  const int words = (int)(sizeof(PcgState) / sizeof(int32_t));
  const int32_t* src = reinterpret_cast<const int32_t*>(st);
  int32_t* dst = reinterpret_cast<int32_t*>(h_state);
  for (int i = c * 256 + tid; i < words; i += 256 * T) dst[i] = src[i];
  const int cnt = rows * MAX_COLS;
  for (int i = c * 256 + tid; i < cnt; i += 256 * T) { h_alog[i] = alog[i]; h_blog[i] = blog[i]; }
  __threadfence_system();
  __syncthreads();
  if (tid == 0) last = (atomicAdd(&st->tail_count, 1) == T - 1);
  __syncthreads();
  if (last && tid == 0) {
    st->tail_count = 0;
    __threadfence_system();
    *reinterpret_cast<volatile uint64_t*>(&flags->tail_seq) = seq;
  }
}

// Waits until the device has stored `want` in a pinned sequence slot: a short poll (the usual case:
// microseconds after the kernel ends), then an ordinary stream synchronisation.
static int wait_seq(const volatile uint64_t* slot, uint64_t want, hipStream_t s) {
  for (int spin = 0; spin < 200000; ++spin) {
    if (*slot == want) return NUGPR_OK;
    __builtin_ia32_pause();
  }
  NUGPR_HIP(hipStreamSynchronize(s));
  if (*slot != want) { set_error("the device did not report the end of a solver step"); return NUGPR_ERR_HIP; }
  return NUGPR_OK;
}

// start of a solve on a caller's right-hand sides: X = 0, R = B and, when the first direction is known
// (Z0 not null), D = Z0.  (The alpha / beta logs need no clearing: every row the host reads is written
// during the solve.)
template <typename VT>
__global__ void k_pcg_init(VT* __restrict__ X, VT* __restrict__ R, const VT* __restrict__ B,
                           const VT* __restrict__ Z0, VT* __restrict__ D, int64_t count) {
  const int64_t i0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
  if (Z0) {
    for (int64_t i = i0; i < count; i += stride) { X[i] = (VT)0; R[i] = B[i]; D[i] = Z0[i]; }
  } else {
    for (int64_t i = i0; i < count; i += stride) { X[i] = (VT)0; R[i] = B[i]; }
  }
}

template <typename SRC, typename DST>
__global__ void k_convert(const SRC* __restrict__ src, DST* __restrict__ dst, int64_t count) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = (DST)src[i];
}

int to_internal(nugpr_ctx* c, const float* src, void* dst, int64_t count, hipStream_t s) {
  if (c->acc64) hipLaunchKernelGGL((k_convert<float, double>), dim3(1024), dim3(256), 0, s, src, (double*)dst, count);
  else NUGPR_HIP(hipMemcpyAsync(dst, src, (size_t)count * sizeof(float), hipMemcpyDeviceToDevice, s));
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

int from_internal(nugpr_ctx* c, const void* src, float* dst, int64_t count, hipStream_t s) {
  if (c->acc64) hipLaunchKernelGGL((k_convert<double, float>), dim3(1024), dim3(256), 0, s, (const double*)src, dst, count);
  else NUGPR_HIP(hipMemcpyAsync(dst, src, (size_t)count * sizeof(float), hipMemcpyDeviceToDevice, s));
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

// ---------------------------------------------------------------------------
// operator applications on internal vector blocks
// ---------------------------------------------------------------------------
static int run_project(nugpr_ctx* c, const void* D, int T, hipStream_t s, const float* D32 = nullptr);
// Q = a Q0 + b D with the reduction that follows a product in the solver (partial as in
// k_onehot_expand_dot; may be null)
template <typename VT>
__global__ __launch_bounds__(256) void k_lincomb_dot(VT* __restrict__ Q, const VT* __restrict__ Q0,
                                                     const VT* __restrict__ D, double a, double b, int64_t n, int T,
                                                     double* __restrict__ partial) {
  __shared__ double red[256];
  const int rpp = 256 / T;
  const int tid = threadIdx.x;
  const int myrow = tid / T, col = tid - myrow * T;
  const bool live = myrow < rpp;
  const int64_t rows_per_block = (n + gridDim.x - 1) / gridDim.x;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
  double s0 = 0.0;
  if (live) {
    for (int64_t p = r0 + myrow; p < r1; p += rpp) {
      const int64_t idx = p * T + col;
      const double d = (double)D[idx];
      const VT qn = (VT)fma(a, (double)Q0[idx], b * d);
      Q[idx] = qn;
      s0 = fma(d, (double)qn, s0);
    }
  }
  red[tid] = s0;
  __syncthreads();
  if (partial && tid < T) {
    double sacc = 0.0;
    for (int k = 0; k < rpp; ++k) sacc += red[k * T + tid];
    partial[(int64_t)blockIdx.x * MAX_COLS + tid] = sacc;
  }
}

static int run_expand(nugpr_ctx* c, void* Q, int T, hipStream_t s, const void* D = nullptr, double* dq_partial = nullptr,
                      float* Q32 = nullptr);

int run_matvec(nugpr_ctx* c, const void* D, void* Q, int T, hipStream_t s, double* dq_partial, bool* dq_done,
               const float* D32, float* Q32) {
  const Layout& L = c->L;
  int rc;
  const uint64_t ppart = (uint64_t)L.ncr * T;
  // S_j = W_j^T D_j (dense W: in column slabs of W_j^T that are then added up); the projection of z_0, the
  // first direction of every solve on the context's own right-hand sides, is kept with the factor
  const bool s_known = D == c->Z0v && T == L.T && c->z0_ready && !D32;
  // The first direction again, on the blocks whose product with it is kept (base loss of a train step): the
  // operator is s K_0 + shift I for some other (s, shift), and the product a combination of what is kept.
  const bool shortcuts = !(c->params.flags & NUGPR_NO_SHORTCUTS);
  if (s_known && shortcuts && c->q0_gen == c->build_gen && Q != c->Q0v) {
    const double a = c->op_scale / c->q0_scale, b = c->op_shift - a * c->q0_shift;
    const int nb = L.n_dot_blocks;
    if (c->acc64) hipLaunchKernelGGL((k_lincomb_dot<double>), dim3(nb), dim3(256), 0, s, (double*)Q, (const double*)c->Q0v, (const double*)D, a, b, (int64_t)L.n, T, dq_partial);
    else hipLaunchKernelGGL((k_lincomb_dot<float>), dim3(nb), dim3(256), 0, s, (float*)Q, (const float*)c->Q0v, (const float*)D, a, b, (int64_t)L.n, T, dq_partial);
    NUGPR_HIP(hipGetLastError());
    if (dq_done) *dq_done = dq_partial != nullptr;
    c->stats.products_reused += 1;
    return NUGPR_OK;
  }
  c->stats.products += 1;
  if (!s_known && (rc = run_project(c, D, T, s, D32))) return rc;
  // only the launch with one column group in fp64 mode reads the lower tiles of the K_ii and of C alone
  if (!(c->acc64 && T >= 2 && T <= 17) && ((rc = ensure_kd_upper(c, s)) || (rc = ensure_c_upper(c, s)))) return rc;
  // Q_i = K_ii D_i   and   P = C_offdiag S (column slabs), one launch
  StripPort k0{}, k1{};
  k0.A = c->Kd; k0.in = D; k0.out = Q; k0.nin = 1; k0.scale = c->op_scale; k0.diag_add = c->op_shift;
  k1.A = c->C; k1.in = s_known ? c->S0v : c->Spart; k1.nin = 1; k1.out = c->Ppart; k1.out_part_stride = ppart; k1.scale = c->op_scale;
  const bool timed = c->prof_on && (size_t)(2 * c->prof_used + 1) < c->prof_ev.size();
  if (timed) NUGPR_HIP(hipEventRecord(c->prof_ev[2 * c->prof_used], s));
  if ((rc = launch_strip(c->tab_KC, k0, k1, T, c->acc64, s))) return rc;
  if (timed) {
    NUGPR_HIP(hipEventRecord(c->prof_ev[2 * c->prof_used + 1], s));
    c->prof_used += 1;
  }
  if (L.compensate) {                     // the fp32 residual of C - lambda_0 I, added slab by slab
    StripPort k2 = k1;
    k2.A = c->Clo; k2.accumulate = 1;
    if ((rc = launch_strip(c->tab_C, k2, k2, T, c->acc64, s))) return rc;
  }
  if (L.nsP > 1 && (rc = launch_sum_parts(c->Ppart, c->Ppart, (int64_t)ppart, L.nsP, ppart, c->acc64, s))) return rc;
  // Q_i += W_i P_i (and, on request, the partial sums of <d, q> in the same pass)
  const bool fuse = dq_partial && c->onehot;
  if (dq_done) *dq_done = fuse;
  if ((rc = run_expand(c, Q, T, s, fuse ? D : nullptr, fuse ? dq_partial : nullptr, Q32))) return rc;
  if (s_known && shortcuts && c->build_gen == c->factor_gen && c->q0_gen != c->build_gen) {
    const size_t bytes = (size_t)L.n * T * (c->acc64 ? sizeof(double) : sizeof(float));
    NUGPR_HIP(hipMemcpyAsync(c->Q0v, Q, bytes, hipMemcpyDeviceToDevice, s));
    c->q0_gen = c->build_gen;
    c->q0_scale = c->op_scale;
    c->q0_shift = c->op_shift;
  }
  return NUGPR_OK;
}

// out = a * x  (elementwise over a vector block)
template <typename VT>
__global__ void k_scaled_copy(VT* __restrict__ out, const VT* __restrict__ x, double a, int64_t count) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
    out[i] = (VT)(a * (double)x[i]);
}

// q = q + 4 a + d: the last step of Q(A) d = A(A d) + 4 A d + d (eq. (PQ)), with a = A d and q = A a on entry
template <typename VT>
__global__ void k_pade_q_combine(VT* __restrict__ q, const VT* __restrict__ a, const VT* __restrict__ d, int64_t count) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
    q[i] = (VT)((double)q[i] + 4.0 * (double)a[i] + (double)d[i]);
}

template <typename VT>
static int scaled_copy(void* out, const void* x, double a, int64_t count, hipStream_t s) {
  hipLaunchKernelGGL((k_scaled_copy<VT>), dim3(1024), dim3(256), 0, s, (VT*)out, (const VT*)x, a, count);
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

// One-hot basis (every point belongs to exactly one representative): S = W^T D is the sum of the rows of
// D over each representative's points, taken in ascending point order; Q += W P adds row assign[p] of P to
// row p.  Neither streams the dense W.
// ST: type of the block that is read.  Dwide (may be null): every point belongs to exactly one representative,
// so the gather visits every row of D once and can leave a copy of it in the solver's own type on the way
// (the widening of a caller's fp32 block, which the strip kernels then read, costs no pass of its own).
template <typename VT, typename ST>
__global__ __launch_bounds__(256) void k_onehot_project(const ST* __restrict__ D, VT* __restrict__ Dwide,
                                                        const int32_t* __restrict__ rep_ptr,
                                                        const int32_t* __restrict__ rep_pts, VT* __restrict__ S,
                                                        int ncr, int T) {
  const int rpp = 256 / T;
  const int tid = threadIdx.x;
  const int myrow = tid / T, col = tid - myrow * T;
  if (myrow >= rpp) return;
  for (int a = blockIdx.x * rpp + myrow; a < ncr; a += gridDim.x * rpp) {
    double s = 0.0;
    const int q1 = rep_ptr[a + 1];
    // eight gathers in flight at a time; the additions stay in ascending point order
    for (int q = rep_ptr[a]; q < q1; q += 8) {
      int idx[8];
      double v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) idx[j] = rep_pts[q + j < q1 ? q + j : q1 - 1];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (double)D[(int64_t)idx[j] * T + col];
      if (Dwide) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (q + j < q1) Dwide[(int64_t)idx[j] * T + col] = (VT)v[j];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) s += q + j < q1 ? v[j] : 0.0;
    }
    S[(int64_t)a * T + col] = (VT)s;
  }
}

// out = Q + W P: out is Q itself, or the caller's fp32 block (the narrowing then costs no pass of its own)
template <typename VT, typename OT>
__global__ __launch_bounds__(256) void k_onehot_expand(const VT* Q, const VT* __restrict__ P,
                                                       const int32_t* __restrict__ assign, int64_t n, int T,
                                                       OT* out) {
  const int rpp = 256 / T;
  const int tid = threadIdx.x;
  const int myrow = tid / T, col = tid - myrow * T;
  if (myrow >= rpp) return;
  for (int64_t p = (int64_t)blockIdx.x * rpp + myrow; p < n; p += (int64_t)gridDim.x * rpp) {
    const int64_t idx = p * T + col;
    out[idx] = (OT)((double)Q[idx] + (double)P[(int64_t)assign[p] * T + col]);
  }
}

// the same with the reduction that follows a product in the solver: partial = per-workgroup sums of d q_new
// per column, rows split among the workgroups as in k_dot
template <typename VT>
__global__ __launch_bounds__(256) void k_onehot_expand_dot(VT* __restrict__ Q, const VT* __restrict__ P,
                                                           const int32_t* __restrict__ assign,
                                                           const VT* __restrict__ D, int64_t n, int T,
                                                           double* __restrict__ partial) {
  __shared__ double red[256];
  const int rpp = 256 / T;
  const int tid = threadIdx.x;
  const int myrow = tid / T, col = tid - myrow * T;
  const bool live = myrow < rpp;
  const int64_t rows_per_block = (n + gridDim.x - 1) / gridDim.x;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
  double s0 = 0.0;
  if (live) {
    for (int64_t p = r0 + myrow; p < r1; p += rpp) {
      const int64_t idx = p * T + col;
      const VT qn = (VT)((double)Q[idx] + (double)P[(int64_t)assign[p] * T + col]);
      Q[idx] = qn;
      s0 = fma((double)D[idx], (double)qn, s0);
    }
  }
  red[tid] = s0;
  __syncthreads();
  if (tid < T) {
    double sacc = 0.0;
    for (int k = 0; k < rpp; ++k) sacc += red[k * T + tid];
    partial[(int64_t)blockIdx.x * MAX_COLS + tid] = sacc;
  }
}

static int elementwise_grid(int64_t n, int T);

// S = W^T D into the first slab of Spart (summed over the column slabs when W is dense).  D32 (one-hot basis,
// fp64 mode only): the block is read from this fp32 array and its widened copy is written to D on the way.
static int run_project(nugpr_ctx* c, const void* D, int T, hipStream_t s, const float* D32) {
  const Layout& L = c->L;
  if (D32 && !(c->onehot && c->acc64)) { set_error("internal: fused widening needs the one-hot basis in fp64 mode"); return NUGPR_ERR_INVALID; }
  if (c->onehot) {
    const int grid = elementwise_grid(L.ncr, T);
    if (D32) hipLaunchKernelGGL((k_onehot_project<double, float>), dim3(grid), dim3(256), 0, s, D32, (double*)const_cast<void*>(D), c->rep_ptr, c->rep_pts, (double*)c->Spart, L.ncr, T);
    else if (c->acc64) hipLaunchKernelGGL((k_onehot_project<double, double>), dim3(grid), dim3(256), 0, s, (const double*)D, (double*)nullptr, c->rep_ptr, c->rep_pts, (double*)c->Spart, L.ncr, T);
    else hipLaunchKernelGGL((k_onehot_project<float, float>), dim3(grid), dim3(256), 0, s, (const float*)D, (float*)nullptr, c->rep_ptr, c->rep_pts, (float*)c->Spart, L.ncr, T);
    NUGPR_HIP(hipGetLastError());
    return NUGPR_OK;
  }
  int rc;
  const uint64_t spart = (uint64_t)L.ncr * T;
  StripPort s0{};
  s0.A = c->Wt; s0.in = D; s0.out = c->Spart; s0.nin = 1; s0.out_part_stride = spart;
  if ((rc = launch_strip(c->tab_WtD, s0, s0, T, c->acc64, s))) return rc;
  if (L.nsS > 1 && (rc = launch_sum_parts(c->Spart, c->Spart, (int64_t)spart, L.nsS, spart, c->acc64, s))) return rc;
  return NUGPR_OK;
}

// Q += W P with P the first slab of Ppart; with Q32 (one-hot basis, fp64 mode) the sum goes to that fp32 array instead
static int run_expand(nugpr_ctx* c, void* Q, int T, hipStream_t s, const void* D, double* dq_partial, float* Q32) {
  const Layout& L = c->L;
  if (Q32 && !(c->onehot && c->acc64 && !dq_partial)) { set_error("internal: fused narrowing needs the one-hot basis in fp64 mode"); return NUGPR_ERR_INVALID; }
  if (c->onehot && dq_partial) {
    const int nb = L.n_dot_blocks;
    if (c->acc64) hipLaunchKernelGGL((k_onehot_expand_dot<double>), dim3(nb), dim3(256), 0, s, (double*)Q, (const double*)c->Ppart, c->assign, (const double*)D, (int64_t)L.n, T, dq_partial);
    else hipLaunchKernelGGL((k_onehot_expand_dot<float>), dim3(nb), dim3(256), 0, s, (float*)Q, (const float*)c->Ppart, c->assign, (const float*)D, (int64_t)L.n, T, dq_partial);
    NUGPR_HIP(hipGetLastError());
    return NUGPR_OK;
  }
  if (c->onehot) {
    const int grid = elementwise_grid(L.n, T);
    if (Q32) hipLaunchKernelGGL((k_onehot_expand<double, float>), dim3(grid), dim3(256), 0, s, (const double*)Q, (const double*)c->Ppart, c->assign, (int64_t)L.n, T, Q32);
    else if (c->acc64) hipLaunchKernelGGL((k_onehot_expand<double, double>), dim3(grid), dim3(256), 0, s, (const double*)Q, (const double*)c->Ppart, c->assign, (int64_t)L.n, T, (double*)Q);
    else hipLaunchKernelGGL((k_onehot_expand<float, float>), dim3(grid), dim3(256), 0, s, (const float*)Q, (const float*)c->Ppart, c->assign, (int64_t)L.n, T, (float*)Q);
    NUGPR_HIP(hipGetLastError());
    return NUGPR_OK;
  }
  StripPort w0{};
  w0.A = c->Wd; w0.in = c->Ppart; w0.nin = 1; w0.out = Q; w0.accumulate = 1;
  return launch_strip(c->tab_WP, w0, w0, T, c->acc64, s);
}

// Q += scale * W (C_offdiag (W^T D)): the low-rank part of the product on its own
static int run_lowrank_accumulate(nugpr_ctx* c, const void* D, void* Q, int T, hipStream_t s) {
  const Layout& L = c->L;
  int rc;
  const uint64_t ppart = (uint64_t)L.ncr * T;
  if (!(c->acc64 && T >= 2 && T <= 17) && (rc = ensure_c_upper(c, s))) return rc;
  if ((rc = run_project(c, D, T, s))) return rc;
  StripPort k1{};
  k1.A = c->C; k1.in = c->Spart; k1.nin = 1; k1.out = c->Ppart; k1.out_part_stride = ppart; k1.scale = c->op_scale;
  if ((rc = launch_strip(c->tab_C, k1, k1, T, c->acc64, s))) return rc;
  if (L.compensate) {
    StripPort k2 = k1;
    k2.A = c->Clo; k2.accumulate = 1;
    if ((rc = launch_strip(c->tab_C, k2, k2, T, c->acc64, s))) return rc;
  }
  if (L.nsP > 1 && (rc = launch_sum_parts(c->Ppart, c->Ppart, (int64_t)ppart, L.nsP, ppart, c->acc64, s))) return rc;
  return run_expand(c, Q, T, s);
}

// out = A D with A = Y K' Y^T, Y = L^-1 (the paper's R^-T K' R^-1, eq. (RKR)).  Scratch: Vv, Uv.
// While the stored blocks are the ones that were factored, K_diag = s L L^T + shift I for the
// operator in force (eqs. (linear1)-(linear3)), so A D = s D + Y (shift U + s W C W^T U), U = Y^T D,
// and the block-diagonal matrix is not streamed at all.
int run_split_op(nugpr_ctx* c, const void* D, void* out, int T, hipStream_t s) {
  int rc;
  const int64_t cnt = c->L.n * T;
  StripPort up{};
  up.A = c->G; up.in = D; up.out = c->Vv; up.nin = 1;
  if ((rc = launch_strip(c->tab_upG, up, up, T, c->acc64, s))) return rc;                 // U = Y^T D
  const bool identity = c->build_gen == c->factor_gen && !c->general_route &&
                        !(c->params.flags & (NUGPR_NO_SHORTCUTS | NUGPR_PRECOND_COMPENSATED));
  StripPort lo{};
  lo.A = c->G; lo.in = c->Uv; lo.out = out; lo.nin = 1;
  if (!identity) {
    if ((rc = run_matvec(c, c->Vv, c->Uv, T, s))) return rc;                              // K' U
  } else {
    rc = c->acc64 ? scaled_copy<double>(c->Uv, c->Vv, c->op_shift, cnt, s) : scaled_copy<float>(c->Uv, c->Vv, c->op_shift, cnt, s);
    if (rc) return rc;
    if ((rc = run_lowrank_accumulate(c, c->Vv, c->Uv, T, s))) return rc;
    rc = c->acc64 ? scaled_copy<double>(out, D, c->op_scale, cnt, s) : scaled_copy<float>(out, D, c->op_scale, cnt, s);
    if (rc) return rc;
    lo.accumulate = 1;
  }
  return launch_strip(c->tab_lowG, lo, lo, T, c->acc64, s);                               // Y (.)
}

// Q = (A^2 + 4 A + I) D, eq. (PQ).  Scratch: Zv (holds A D), and what run_split_op uses.
static int run_pade_q(nugpr_ctx* c, const void* D, void* Q, int T, hipStream_t s) {
  int rc;
  if ((rc = run_split_op(c, D, c->Zv, T, s))) return rc;
  if ((rc = run_split_op(c, c->Zv, Q, T, s))) return rc;
  const int64_t cnt = c->L.n * T;
  if (c->acc64)
    hipLaunchKernelGGL((k_pade_q_combine<double>), dim3(1024), dim3(256), 0, s, (double*)Q, (const double*)c->Zv, (const double*)D, cnt);
  else
    hipLaunchKernelGGL((k_pade_q_combine<float>), dim3(1024), dim3(256), 0, s, (float*)Q, (const float*)c->Zv, (const float*)D, cnt);
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

int run_precond(nugpr_ctx* c, const void* R, void* Z, int T, hipStream_t s) {
  int rc;
  c->stats.precond_applies += 1;
  StripPort a{};
  a.A = c->G; a.in = R; a.out = c->Vv; a.nin = 1;
  if ((rc = launch_strip(c->tab_lowG, a, a, T, c->acc64, s))) return rc;
  StripPort b{};
  b.A = c->G; b.in = c->Vv; b.out = Z; b.nin = 1;
  return launch_strip(c->tab_upG, b, b, T, c->acc64, s);
}

static int elementwise_grid(int64_t n, int T) {
  const int rpp = 256 / T;
  int64_t g = (n + rpp - 1) / rpp;
  return (int)std::min<int64_t>(g, 4096);
}

template <typename VT>
static int dot2_t(nugpr_ctx* c, const VT* A0, const VT* B0, const VT* A1, const VT* B1, int T, double* out0,
                  double* out1, hipStream_t s) {
  const Layout& L = c->L;
  const int nb = L.n_dot_blocks;
  hipLaunchKernelGGL((k_dot<2, VT>), dim3(nb), dim3(256), 0, s, A0, B0, A1, B1, (int64_t)L.n, T, c->dotpart);
  NUGPR_HIP(hipGetLastError());
  NUGPR_HIP(hipMemcpyAsync(c->h_buf, c->dotpart, (size_t)2 * nb * MAX_COLS * sizeof(double), hipMemcpyDeviceToHost, s));
  NUGPR_HIP(hipStreamSynchronize(s));
  for (int col = 0; col < T; ++col) {
    double a0 = 0.0, a1 = 0.0;
    for (int b = 0; b < nb; ++b) {
      a0 += c->h_buf[(size_t)b * MAX_COLS + col];
      a1 += c->h_buf[((size_t)nb + b) * MAX_COLS + col];
    }
    out0[col] = a0;
    out1[col] = a1;
  }
  return NUGPR_OK;
}

// <A0, B0> and <A1, B1> per column, one synchronisation
int run_dot2(nugpr_ctx* c, const void* A0, const void* B0, const void* A1, const void* B1, int T, double* out0,
             double* out1, hipStream_t s) {
  if (c->acc64) return dot2_t<double>(c, (const double*)A0, (const double*)B0, (const double*)A1, (const double*)B1, T, out0, out1, s);
  return dot2_t<float>(c, (const float*)A0, (const float*)B0, (const float*)A1, (const float*)B1, T, out0, out1, s);
}

template <typename VT>
static int pcg_t(nugpr_ctx* c, const VT* B, VT* X, int T, int32_t* iters, double* alpha, double* beta,
                 int* max_it_used, hipStream_t s, PcgExtras* extras, int system) {
  const Layout& L = c->L;
  const int64_t n = L.n;
  const int nb = L.n_dot_blocks;
  const int eg = elementwise_grid(n, T);
  const double tol2 = c->params.tol * c->params.tol;
  const int max_iter = c->params.max_iter;
  int rc;
  VT *R = (VT*)c->Rv, *Z = (VT*)c->Zv, *D = (VT*)c->Dv, *Q = (VT*)c->Qv;
  // Without a preconditioner (the Pade system, already preconditioned) z = r throughout.
  const bool plain = system == PCG_PADE_Q;
  const VT* Zr = plain ? R : Z;
  // Solves on the two right-hand-side blocks the context owns start from values kept with the factor:
  // z_0 = M^-1 b (or b itself for the Pade system), <b, b> and <b, z_0>.  Nothing is initialised then:
  // the first update reads b in the place of r and writes x without reading it, and the first direction
  // is z_0 where it lies.
  const bool own = T == L.T && c->z0_ready && (const void*)B == (plain ? (const void*)c->Pv : (const void*)c->Bv);
  const VT* Dcur = D;                    // the direction the operator is applied to
  if (own) {
    hipLaunchKernelGGL(k_pcg_begin_known, dim3(1), dim3(64), 0, s, c->d_state, plain ? 1 : 0, T);
    Dcur = plain ? B : (const VT*)c->Z0v;
  } else {
    // x_0 = 0, r_0 = b, d_0 = z_0 = M^-1 r_0 written straight into D
    hipLaunchKernelGGL((k_pcg_init<VT>), dim3(1024), dim3(256), 0, s, X, R, B, plain ? B : (const VT*)nullptr, D, n * T);
    if (!plain && (rc = run_precond(c, R, D, T, s))) return rc;
    hipLaunchKernelGGL((k_dot<2, VT>), dim3(nb), dim3(256), 0, s, (const VT*)R, (const VT*)R, (const VT*)R, (const VT*)D, n, T, c->dotpart);
    hipLaunchKernelGGL(k_pcg_begin, dim3(T), dim3(256), 0, s, c->d_state, c->dotpart, nb);
  }
  NUGPR_HIP(hipGetLastError());
  bool first = own;
  int it = 0;
  bool indefinite = false;
  // The first iteration is issued without asking the device whether any column is active: columns
  // that start inactive (zero right-hand side) are skipped by every kernel on their own flag, and
  // the host learns the count at the first stop test.
  c->h_flags->n_active = 1;
  const size_t cnt = (size_t)max_iter * MAX_COLS;
  PcgState* hs = reinterpret_cast<PcgState*>(c->h_buf + 2 * cnt);
  double* hdot = c->h_buf + 2 * cnt + (sizeof(PcgState) + sizeof(double) - 1) / sizeof(double);
  const bool want_logs = alpha || beta;
  // The end-of-solve report (k_pcg_tail) is issued INSIDE the iteration that is expected to be the last
  // one, right behind its stop test, so that it is already on the host when the stop test says "done";
  // a solve that ends earlier or later than the previous one of its kind gets the report after the loop.
  const int expect = c->expect_iters[plain ? 1 : 0];
  // (its <b, x> sums were left in the second partial set by the update kernel of the same iteration)
  auto issue_tail = [&](int rows, bool bx_ready) -> int {
    if (extras && !bx_ready)
      hipLaunchKernelGGL((k_dot<2, VT>), dim3(nb), dim3(256), 0, s, B, (const VT*)X, B, (const VT*)X, n, T, c->dotpart);
    c->tail_seq += 1;
    hipLaunchKernelGGL(k_pcg_tail, dim3(T), dim3(256), 0, s, c->d_state, c->dotpart + (size_t)nb * MAX_COLS, nb, T, extras ? 1 : 0, c->alog,
                       c->blog, want_logs ? rows : 0, hs, hdot, c->h_buf, c->h_buf + cnt, c->h_flags, c->tail_seq);
    NUGPR_HIP(hipGetLastError());
    return NUGPR_OK;
  };
  bool tail_current = false;
  while (it < max_iter && c->h_flags->n_active > 0) {
    bool dq_done = false;
    if ((rc = plain ? run_pade_q(c, Dcur, Q, T, s) : run_matvec(c, Dcur, Q, T, s, c->dotpart, &dq_done))) return rc;
    if (!dq_done)
      hipLaunchKernelGGL((k_dot<1, VT>), dim3(nb), dim3(256), 0, s, Dcur, (const VT*)Q, Dcur, (const VT*)Q, n, T, c->dotpart);
    hipLaunchKernelGGL(k_pcg_alpha, dim3(T), dim3(256), 0, s, c->d_state, c->dotpart, nb, it, c->alog);
    // the update, fused with ||r||^2 for the stop test and, in the iteration expected to be the last, <b, x>
    const bool report = it + 1 >= expect || it + 1 >= max_iter;
    hipLaunchKernelGGL((k_update_xr_dots<VT>), dim3(nb), dim3(256), 0, s, X, R, first ? B : (const VT*)R, Dcur,
                       (const VT*)Q, (report && extras) ? B : (const VT*)nullptr, c->d_state, n, T, first ? 1 : 0,
                       c->dotpart);
    first = false;
    // stop test first: when every column has converged the preconditioner apply is not needed
    c->flag_seq += 1;
    hipLaunchKernelGGL(k_pcg_check, dim3(T), dim3(256), 0, s, c->d_state, c->dotpart, nb, it, tol2, T, c->h_flags,
                       c->flag_seq);
    NUGPR_HIP(hipGetLastError());
    tail_current = false;
    if (report) {
      if ((rc = issue_tail(it + 1, true))) return rc;
      tail_current = true;
    }
    if ((rc = wait_seq(&c->h_flags->seq, c->flag_seq, s))) return rc;
    const int j = it++;
    if (c->h_flags->indefinite) indefinite = true;
    if (c->h_flags->n_active == 0 || it >= max_iter) break;
    if (!plain && (rc = run_precond(c, R, Z, T, s))) return rc;
    hipLaunchKernelGGL((k_dot<1, VT>), dim3(nb), dim3(256), 0, s, (const VT*)R, Zr, (const VT*)R, Zr, n, T, c->dotpart);
    hipLaunchKernelGGL(k_pcg_beta, dim3(T), dim3(256), 0, s, c->d_state, c->dotpart, nb, j, c->blog);
    hipLaunchKernelGGL((k_update_d<VT>), dim3(eg), dim3(256), 0, s, D, Dcur, Zr, c->d_state, n, T);
    NUGPR_HIP(hipGetLastError());
    Dcur = D;
  }
  c->expect_iters[plain ? 1 : 0] = it > 0 ? it : 1;
  c->stats.pcg_solves += 1;
  c->stats.pcg_iterations += it;
  c->stats.pcg_iterations_max = std::max<int64_t>(c->stats.pcg_iterations_max, it);
  if (!tail_current && (rc = issue_tail(it, false))) return rc;
  if ((rc = wait_seq(&c->h_flags->tail_seq, c->tail_seq, s))) return rc;
  bool all_conv = true;
  int mx = 0;
  for (int col = 0; col < T; ++col) {
    if (iters) iters[col] = hs->iters[col];
    mx = std::max(mx, hs->iters[col]);
    if (!hs->converged[col]) all_conv = false;
    if (hs->indef[col]) indefinite = true;
  }
  if (max_it_used) *max_it_used = mx;
  if (extras) {
    for (int col = 0; col < T; ++col) {
      extras->bx[col] = hdot[col];
      extras->rho0[col] = hs->rho0[col];
    }
  }
  if (alpha || beta) {
    const double* ha = c->h_buf;
    for (int j = 0; j < max_iter; ++j)
      for (int col = 0; col < T; ++col) {                 // rows past the last iteration were never written: zero
        if (alpha) alpha[(size_t)j * T + col] = j < it ? ha[(size_t)j * MAX_COLS + col] : 0.0;
        // (no beta follows the last iteration)
        if (beta) beta[(size_t)j * T + col] = j < it - 1 ? ha[cnt + (size_t)j * MAX_COLS + col] : 0.0;
      }
  }
  // NaN / Inf among the coordinates of the last assembly (found by its scaling kernel), or in a right-hand
  // side: the latter shows in the first dot products of its column, <b, b> and <b, M^-1 b>
  if (c->assembly_mark != 0 && hs->nonfinite_mark == c->assembly_mark) return NUGPR_NOT_FINITE;
  for (int col = 0; col < T; ++col)
    if (!std::isfinite(hs->bnorm2[col]) || !std::isfinite(hs->rho0[col])) return NUGPR_NOT_FINITE;
  if (indefinite) return NUGPR_INDEFINITE;
  return all_conv ? NUGPR_OK : NUGPR_NOT_CONVERGED;
}

template <typename VT>
static int store_known_t(nugpr_ctx* c, hipStream_t s) {
  const Layout& L = c->L;
  const int nb = L.n_dot_blocks;
  const VT *B = (const VT*)c->Bv, *Z0 = (const VT*)c->Z0v, *P = (const VT*)c->Pv;
  hipLaunchKernelGGL((k_dot<2, VT>), dim3(nb), dim3(256), 0, s, B, B, B, Z0, (int64_t)L.n, L.T, c->dotpart);
  hipLaunchKernelGGL(k_store_known, dim3(L.T), dim3(256), 0, s, c->d_state, c->dotpart, nb, 0);
  if (L.t > 0) {
    hipLaunchKernelGGL((k_dot<2, VT>), dim3(nb), dim3(256), 0, s, P, P, P, P, (int64_t)L.n, L.T, c->dotpart);
    hipLaunchKernelGGL(k_store_known, dim3(L.T), dim3(256), 0, s, c->d_state, c->dotpart, nb, 1);
  }
  NUGPR_HIP(hipGetLastError());
  // W^T z_0
  int rc = run_project(c, c->Z0v, L.T, s);
  if (rc) return rc;
  NUGPR_HIP(hipMemcpyAsync(c->S0v, c->Spart, (size_t)L.ncr * L.T * sizeof(VT), hipMemcpyDeviceToDevice, s));
  return NUGPR_OK;
}

// <b, b> and <b, z_0> of the context's own right-hand-side blocks, kept in the device state (called by the
// factorisation once B, z_0 = M^-1 B and the probe block exist)
int store_known_starts(nugpr_ctx* c, hipStream_t s) {
  return c->acc64 ? store_known_t<double>(c, s) : store_known_t<float>(c, s);
}

int run_pcg(nugpr_ctx* c, const void* B, void* X, int T, int32_t* iters, double* alpha, double* beta,
            int* max_it_used, hipStream_t s, PcgExtras* extras, int system) {
  if (c->acc64) return pcg_t<double>(c, (const double*)B, (double*)X, T, iters, alpha, beta, max_it_used, s, extras, system);
  return pcg_t<float>(c, (const float*)B, (float*)X, T, iters, alpha, beta, max_it_used, s, extras, system);
}

}  // namespace nugpr
