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
//
// Two kernels per assembly:
//   k_scale_points  writes the scaled coordinates once, in fp64, in the order the matrix
//                   cores read their operands (groups of 16 points, coordinate-major inside a
//                   group), and the squared norms;
//   k_build_tile    one workgroup = one 64 x 64 tile of a lower triangle.  Each wave owns a
//                   16-column slice: operands come from the scaled array (512-byte contiguous
//                   loads, served by L2), the mirror image is stored straight from registers
//                   and the tile itself through a wave-private LDS staging area, both with
//                   16-byte stores.
#include <algorithm>
#include <cmath>
#include <type_traits>
#include <vector>

#include "nugpr_internal.h"

namespace nugpr {

typedef double v4d __attribute__((ext_vector_type(4)));

struct ScaleArgs {
  double sw[MAX_D];     // sqrt(log2(e) / (2 ell_k^2)): coordinate scale per dimension
  int32_t d;
};

__host__ __device__ inline int pair_kd(int d) { return (d + 3) & ~3; }

// Scaled coordinates of the point with padded row number pr live at
//   S[((pr / 16) * kd + k) * 16 + pr % 16],  k < kd = d rounded up to 4 (padding zero),
// so the 64 lanes (m = lane % 16, kk = lane / 16) of a wave read the operand of MFMA step ks
// for the 16 points of a group as ONE contiguous 512-byte run: element (4 ks + kk) * 16 + m.
// Four threads share a point (coordinates k = sub + 4 e); rows past the end of a cluster are
// written as zeros.  grid.y = cluster (or 0 for the representatives), 64 points per block.
__global__ __launch_bounds__(256) void k_scale_points(const ScaleArgs a, const ClusterInfo* __restrict__ cl,
                                                      const float* __restrict__ P, double* __restrict__ S,
                                                      double* __restrict__ N, int single_total, int single_ld,
                                                      PcgState* __restrict__ st, int mark) {
  uint32_t first, total, ld, prow;
  if (cl) {
    const ClusterInfo c = cl[blockIdx.y];
    first = c.row0; total = c.b; ld = c.ld; prow = c.prow;
  } else {
    first = 0; total = (uint32_t)single_total; ld = (uint32_t)single_ld; prow = 0;
  }
  const uint32_t pl = blockIdx.x * 64 + (threadIdx.x >> 2);
  if (pl >= ld) return;                       // whole groups of four threads leave together
  const int sub = threadIdx.x & 3, d = a.d, kd = pair_kd(d);
  const uint32_t pr = prow + pl;
  double* __restrict__ dst = S + ((uint64_t)(pr >> 4) * kd) * 16 + (pr & 15);
  double nrm = 0.0;
  for (int k = sub; k < kd; k += 4) {
    const double v = (pl < total && k < d) ? a.sw[k] * (double)P[(uint64_t)(first + pl) * d + k] : 0.0;
    dst[(uint64_t)k * 16] = v;
    nrm = fma(v, v, nrm);
  }
  nrm += __shfl_xor(nrm, 1);
  nrm += __shfl_xor(nrm, 2);
  if (sub == 0) {
    N[pr] = nrm;
    if (!(nrm < INFINITY)) st->nonfinite_mark = mark;       // NaN or Inf among this point's coordinates
  }
}

// 2^f on [-1/2, 1/2]: degree-6 interpolant at the Chebyshev nodes (near-minimax), relative error
// < 2.6e-9, a twentieth of the fp32 rounding that follows
constexpr int EXP2_TERMS = 7;
static const double EXP2_COEF[EXP2_TERMS] = {1.0, 0.69314720670283259, 0.2402265092228876, 0.055503272266703242,
                                             0.009618056678524561, 0.0013400428177608545, 0.00015461444698568769};

struct PanelArgs {
  double coef[EXP2_TERMS];   // alpha times the coefficients of 2^f
  float diag_val;       // diagonal entries: float(alpha + sigma^2); coupling under compensation: float(alpha - lambda_0)
  int keep_same;        // coupling: keep the entries between representatives of one cluster (compensation)
  int mirror;           // also store the mirror image of the tiles below the diagonal
  // two matrices from one pass (PAIR instantiations): the exponent of side s is e + g[s] * w, where e is the
  // exponent at the lengthscales the points were scaled with and w is the squared difference of the scaled
  // coordinate pair_dim, or e itself when pair_dim < 0 (one lengthscale for all coordinates)
  double g[2];
  int pair_dim;
  int32_t kd;           // coordinates per point in the scaled array (multiple of 4)
};

constexpr int ST_LD = 20;            // row stride of the staging area (floats): rows stay 16-byte aligned

// alpha * 2^a for a <= 0 (up to rounding), rounded once to fp32.
// a = n + f with n = rint(a) by the 1.5 * 2^52 trick (n also lands, in two's complement, in the low word
// of the sum) and f = a - n in [-1/2, 1/2]; alpha 2^f by a degree-6 polynomial whose coefficients arrive
// already multiplied by alpha; the factor 2^n is applied to the fp32 value (exact, except where the
// result is subnormal or vanishes, as the true value does).  Arguments below -900 are taken as -900.
// Only full-rate vector instructions are used.
// W values at a time, step by step across all of them: a dependent fp64 instruction can issue only
// every other slot, so W independent chains keep the vector ALU busy where one leaves it half idle.
template <int W>
__device__ __forceinline__ void kernel_values(const double (&arg)[W], const double (&co)[EXP2_TERMS], float (&out)[W]) {
  constexpr double MAGIC = 6755399441055744.0;            // 1.5 * 2^52
  double a[W], big[W], f[W], p[W];
#pragma unroll
  for (int j = 0; j < W; ++j) a[j] = fmax(arg[j], -900.0);
#pragma unroll
  for (int j = 0; j < W; ++j) big[j] = a[j] + MAGIC;
#pragma unroll
  for (int j = 0; j < W; ++j) f[j] = a[j] - (big[j] - MAGIC);
#pragma unroll
  for (int j = 0; j < W; ++j) p[j] = fma(co[6], f[j], co[5]);
#pragma unroll
  for (int k = 4; k >= 0; --k)
#pragma unroll
    for (int j = 0; j < W; ++j) p[j] = fma(p[j], f[j], co[k]);
#pragma unroll
  for (int j = 0; j < W; ++j) out[j] = ldexpf((float)p[j], __double2loint(big[j]));
}

// One workgroup = one 64 x 64 tile (tr, tc), tc <= tr, of one square symmetric matrix (a cluster's
// K_ii, or the coupling C) and its mirror image.
//
// Wave w computes columns 16 w .. 16 w + 15 with four 16 x 16 fp64 MFMA accumulators (one per
// 16-row group); the row operands of the tile are shared through LDS, the column operands go
// straight into registers.  The rows of a group are fed to the matrix cores in the order
// 0,4,8,12,1,5,.. so that a lane ends up with FOUR CONSECUTIVE rows of one column: that is a
// 16-byte piece of the mirror image, stored straight from registers.  The tile itself needs the
// other orientation and goes through a wave-private LDS staging area (16-byte reads and stores).
//
// Why one tile per workgroup and nothing cleverer: on this chip the fp64 matrix instructions run
// at the rate of the vector ALU and do not overlap with it, and a wave that alternates arithmetic
// with bursts of stores stalls on the store path; long-lived workgroups that walk along a tile row
// measured 30 % slower than the sum of their parts.  Short workgroups leave the overlap to the
// hardware: while some wait for operands or drain their stores, others compute (seven fit on a
// compute unit: registers are capped for that, and the staging area holds one 16-row group at a time).  Consecutive workgroups take neighbouring tiles of a row, so the row
// operands they share stay in L2.  The exponential uses full-rate instructions only, and the masks
// run on the tiles that need them.
// NKS = kd / 4 when positive; NKS = 0 handles any kd with a loop over the coordinate groups.
//
// PAIR: the two matrices of a central difference in one lengthscale, ell_k e^{+h} and ell_k e^{-h}, from one
// pass.  Their exponents differ from the one at ell_k by a multiple of the squared difference in coordinate
// k alone, so the matrix instructions (40 % of the pass) and the operand traffic are shared; only the
// exponential and the stores are done twice.  Side 0 goes to out_base, side 1 to out_base2, same layout.
template <bool COUPLING, int NKS, bool PAIR>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(PAIR ? 5 : 6, 7)))
void k_build_tile(const PanelArgs a, const BuildItem* __restrict__ items, const double* __restrict__ S,
                  const double* __restrict__ N, float* __restrict__ out_base, int r, float* __restrict__ out_base2) {
  extern __shared__ __attribute__((aligned(16))) double sA[];      // 4 * kd * 16 doubles: row operands
  __shared__ __attribute__((aligned(32))) double sNr[TILE];
  __shared__ __attribute__((aligned(16))) float sT[4][16 * ST_LD];      // per wave: one 16-row group in transit

  const BuildItem cur = items[blockIdx.x];
  const int tr = cur.tr, tc = cur.tc0;
  const int total = (int)cur.total;
  const uint32_t ld = cur.ld, prow = cur.prow;
  float* __restrict__ out = out_base + cur.out_off;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: lives in a scalar register
  const int m = lane & 15, kk = lane >> 4;
  const int kd = a.kd, nks = NKS > 0 ? NKS : kd / 4;
  const int p0 = tr * TILE, q0 = tc * TILE;
  const uint64_t gstride = (uint64_t)kd * 16;                 // doubles per group of 16 points
  const int lofs = kk * 16 + m;                               // this lane's element of a 4-coordinate step
  // row operand: matrix row m of a group carries point 4 (m % 4) + m / 4, so accumulator
  // component i of lane (kk, m) is point 4 kk + i of the group, column m
  const int aofs = kk * 16 + 4 * (m & 3) + (m >> 2);

  // every load of the tile is issued before the first wait: one round trip to memory
  constexpr int NB = NKS > 0 ? NKS : 1;
  const uint32_t qg = prow + (uint32_t)q0 + 16 * wave;         // first of this wave's 16 column points
  const double* __restrict__ Sc = S + (uint64_t)(qg >> 4) * gstride + lofs;
  double bv[NB];
  if (NKS > 0) {
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) bv[ks] = Sc[ks * 64];
  }
  const double nc = (N + qg)[(uint32_t)m];
  double vc = 0.0;                                             // coordinate pair_dim of this lane's column point
  if (PAIR && a.pair_dim >= 0) vc = (S + (uint64_t)(qg >> 4) * gstride)[(uint32_t)(a.pair_dim * 16 + m)];
  {
    constexpr int NCA = NKS > 0 ? NKS : MAX_D / 4;              // row operand elements per thread (4 kd 16 / 256)
    const double* __restrict__ Sg = S + (uint64_t)((prow + p0) >> 4) * gstride;
    const int n_a = 4 * (int)gstride;
    double ra[NCA];
    const double rr = (N + (prow + p0))[(uint32_t)(tid & (TILE - 1))];
#pragma unroll
    for (int j = 0; j < NCA; ++j)                 // (byte offsets in 32 bits: n_a is at most 4096)
      ra[j] = *reinterpret_cast<const double*>(reinterpret_cast<const char*>(Sg) +
                                               (uint32_t)(min(tid + 256 * j, n_a - 1) << 3));
    if (tid < TILE) sNr[tid] = rr;
    // the row operands (4 groups x kd coordinates x 16 points, already in operand order), doubled
#pragma unroll
    for (int j = 0; j < NCA; ++j)
      if (tid + 256 * j < n_a) sA[tid + 256 * j] = 2.0 * ra[j];
  }
  __syncthreads();

  // the accumulators start at -(|x_p|^2 + |x_q|^2) and the row operands carry a factor 2: what comes
  // out is -|x_p - x_q|^2 in the scaled coordinates, the exponent of 2 for the entry
  v4d acc[4];
#pragma unroll
  for (int ti = 0; ti < 4; ++ti) {
    const double4 nr = *reinterpret_cast<const double4*>(&sNr[16 * ti + 4 * kk]);
    acc[ti] = (v4d){-nr.x - nc, -nr.y - nc, -nr.z - nc, -nr.w - nc};
  }
  if (NKS > 0) {
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
      for (int ti = 0; ti < 4; ++ti)
        acc[ti] = __builtin_amdgcn_mfma_f64_16x16x4f64(sA[(ti * NKS + ks) * 64 + aofs], bv[ks], acc[ti], 0, 0, 0);
  } else {
    for (int ks = 0; ks < nks; ++ks) {
      const double b = Sc[ks * 64];
#pragma unroll
      for (int ti = 0; ti < 4; ++ti)
        acc[ti] = __builtin_amdgcn_mfma_f64_16x16x4f64(sA[(ti * nks + ks) * 64 + aofs], b, acc[ti], 0, 0, 0);
    }
  }

  const float dv = a.diag_val;
  float* __restrict__ sTw = &sT[wave][0];
  // staging of one 16-row group: this lane writes rows 4 kk + i, column m; it reads row lane / 4,
  // columns 4 (lane % 4) .. + 3 for the store of the tile's own rows
  float* __restrict__ st_w = sTw + (4 * kk) * ST_LD + m;
  const float4* __restrict__ st_r = reinterpret_cast<const float4*>(sTw + (lane >> 2) * ST_LD + 4 * (lane & 3));
  const uint64_t ld64 = ld;
  const int q = q0 + 16 * wave + m;
  // Blocked storage (blocked_index): strip tr, column blocks 2 tc and 2 tc + 1 hold the tile, each as eight
  // 16 x 16 fragments of 1 KiB.  The tile itself: row group ti, this wave's 16 columns = fragment
  // (ti, wave % 2) of block 2 tc + wave / 2; lane l holds row l / 4, columns 4 (l % 4) .. + 3: float4 number l
  // (wave-uniform base + a 32-bit lane offset: the store takes the base from scalar registers)
  float* __restrict__ od = out + (uint64_t)tr * TILE * ld64 + (uint64_t)(2 * tc + (wave >> 1)) * (TILE * BLK_COLS) +
                           (wave & 1) * FRAG;
  const uint32_t od_lane = 4u * (uint32_t)lane;
  // its mirror image (strip tc): rows 16 wave + m, columns 16 ti + 4 kk .. + 3 of the tile = fragment
  // (wave, ti % 2) of block 2 tr + ti / 2, row m, columns 4 kk ..; a tile on the diagonal is its own mirror
  // image, entry for entry, and is simply written twice
  float* __restrict__ om = out + (uint64_t)tc * TILE * ld64 + (uint64_t)(2 * tr) * (TILE * BLK_COLS) +
                           (2 * wave) * FRAG;
  const uint32_t om_lane = (uint32_t)(m * 16 + 4 * kk);

  // second matrix of a pair: same offsets from the other base
  const int64_t side_off = PAIR ? (int64_t)(out_base2 - out_base) : 0;
  // the sixteen entries of this lane, one 16-row group at a time: masked (EDGE) or not
  auto entries = [&](auto edge_c) {
    constexpr bool EDGE = decltype(edge_c)::value;
#pragma unroll
    for (int ti = 0; ti < 4; ++ti) {
      double w[4] = {0.0, 0.0, 0.0, 0.0};
      if (PAIR) {
        if (a.pair_dim >= 0) {
          // the row points 4 kk .. 4 kk + 3 of this group, coordinate pair_dim (staged doubled)
          const double2* __restrict__ ur = reinterpret_cast<const double2*>(&sA[(ti * kd + a.pair_dim) * 16 + 4 * kk]);
          const double2 u01 = ur[0], u23 = ur[1];
          const double d0 = fma(0.5, u01.x, -vc), d1 = fma(0.5, u01.y, -vc), d2 = fma(0.5, u23.x, -vc),
                       d3 = fma(0.5, u23.y, -vc);
          w[0] = d0 * d0; w[1] = d1 * d1; w[2] = d2 * d2; w[3] = d3 * d3;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) w[i] = acc[ti][i];
        }
      }
#pragma unroll
      for (int side = 0; side < (PAIR ? 2 : 1); ++side) {
        float x[4];
        double arg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) arg[i] = PAIR ? fma(a.g[side], w[i], acc[ti][i]) : acc[ti][i];
        kernel_values<4>(arg, a.coef, x);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = 16 * ti + 4 * kk + i;
          if (EDGE) {
            const int p = p0 + row;
            bool keep = p < total && q < total;
            if (COUPLING) {
              // only blocks between DIFFERENT clusters enter K' (eq. (odsplit)): same-cluster entries are 0
              // (all of C, with alpha - lambda_0 on its diagonal, under the compensation of eq. (krep))
              keep = keep && (a.keep_same || (p / r) != (q / r));
              x[i] = keep ? x[i] : 0.f;
              if (a.keep_same && p == q && p < total) x[i] = dv;
            } else {
              x[i] = keep ? x[i] : 0.f;
              if (p == q && p < total) x[i] = dv;
            }
          }
          st_w[i * ST_LD] = x[i];
        }
        if (a.mirror || tr == tc)
          *reinterpret_cast<float4*>(om + side * side_off + (ti >> 1) * (TILE * BLK_COLS) + (ti & 1) * FRAG + om_lane) =
              make_float4(x[0], x[1], x[2], x[3]);
        // The staging rows are wave-private and the LDS serves one wave's accesses in order: the read below
        // sees this group's writes, and the next group's writes come after it.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const float4 rowv = *st_r;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        *reinterpret_cast<float4*>(od + side * side_off + (2 * ti) * FRAG + od_lane) = rowv;
      }
    }
  };
  // tiles that can hold dropped or replaced entries: on the diagonal, at the ragged end, or (coupling)
  // overlapping a same-cluster block of r x r representatives (q0 <= p0)
  const bool edge = tr == tc || p0 + TILE > total || q0 + TILE > total ||
                    (COUPLING && (q0 + TILE - 1) / r >= p0 / r);
  if (edge) entries(std::true_type());
  else entries(std::false_type());
}

// What fp32 storage of the compensated coupling matrix drops (eq. (krep)): every entry of
// C - lambda_0 I is evaluated once more in plain fp64 from the representatives and the stored fp32 value
// is subtracted; the difference, in fp32, is the second term of a two-term representation of the entry.
// The matrix is small here (n_c r <= 512).
struct CouplingArgs {
  double inv_ell[MAX_D];
  double alpha, lambda0;
  int n, d;
  uint32_t ld;
};
__global__ __launch_bounds__(256) void k_coupling_residual(CouplingArgs a, const float* __restrict__ reps,
                                                           const float* __restrict__ Chi, float* __restrict__ Clo) {
  const uint64_t idx = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (uint64_t)a.ld * a.ld) return;
  const int i = (int)(idx / a.ld), j = (int)(idx - (uint64_t)i * a.ld);
  float lo = 0.f;
  if (i < a.n && j < a.n) {
    double q = 0.0;
    for (int k = 0; k < a.d; ++k) {
      const double t = ((double)reps[(uint64_t)i * a.d + k] - (double)reps[(uint64_t)j * a.d + k]) * a.inv_ell[k];
      q = fma(t, t, q);
    }
    double v = a.alpha * exp(-0.5 * q);
    if (i == j) v -= a.lambda0;
    lo = (float)(v - (double)Chi[blocked_index(a.ld, i, j)]);
  }
  Clo[blocked_index(a.ld, i, j)] = lo;             // same blocked storage as the matrix it completes
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
                                                 float* __restrict__ Wt, int32_t* __restrict__ assign, int r, int d,
                                                 uint32_t ldw) {
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
  assign[p] = (int32_t)blockIdx.y * r + best;
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
                         int rows, int cols, int lower_only, int blocked) {
  const int64_t total = (int64_t)rows * cols;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int p = (int)(idx / cols), q = (int)(idx - (int64_t)p * cols);
    float v = (float)src[blocked ? blocked_index((uint32_t)lds, p, q) : (uint64_t)p * lds + q];
    if (lower_only && q > p) v = 0.f;
    dst[(int64_t)p * ldd + q] = v;
  }
}

int launch_setup(nugpr_ctx* c, const float* user_reps, const float* user_W, hipStream_t s) {
  const Layout& L = c->L;
  // tile list of the diagonal blocks (used when the inverse factor is mirrored) and the
  // work items of the two assembly launches
  std::vector<uint64_t> tiles;
  tiles.reserve(L.n_diag_tiles);
  for (int i = 0; i < L.nc; ++i)
    for (uint32_t tr = 0; tr < L.cl[i].nt; ++tr)
      for (uint32_t tc = 0; tc <= tr; ++tc) tiles.push_back(((uint64_t)i << 32) | ((uint64_t)tr << 16) | tc);
  // one assembly work item per tile of the lower triangles, neighbours along a tile row next to each other
  auto panel_items = [&](uint32_t nt, uint64_t out_off, uint32_t prow, uint32_t total, uint32_t ld,
                         std::vector<BuildItem>& v) {
    for (uint32_t tr = 0; tr < nt; ++tr)
      for (uint32_t tc = 0; tc <= tr; ++tc) {
        BuildItem b{};
        b.out_off = out_off; b.prow = prow; b.total = total; b.ld = ld;
        b.tr = (uint16_t)tr; b.tc0 = (uint16_t)tc; b.tc1 = (uint16_t)(tc + 1);
        v.push_back(b);
      }
  };
  std::vector<BuildItem> pd, pc;
  // last cluster first: the blocks written last are the ones the product reads first (cluster 0 upwards),
  // while they are still in the memory-side cache
  for (int i = L.nc - 1; i >= 0; --i) panel_items(L.cl[i].nt, L.cl[i].koff, L.cl[i].prow, L.cl[i].b, L.cl[i].ld, pd);
  panel_items((uint32_t)(L.ldc / TILE), 0, 0, (uint32_t)L.ncr, (uint32_t)L.ldc, pc);
  c->n_pan_diag = (int)pd.size();
  c->n_pan_c = (int)pc.size();
  c->d_pan_diag = reinterpret_cast<BuildItem*>(c->d_tiles + tiles.size());
  c->d_pan_c = c->d_pan_diag + pd.size();
  NUGPR_HIP(hipMemcpyAsync(c->d_tiles, tiles.data(), tiles.size() * sizeof(uint64_t), hipMemcpyHostToDevice, s));
  NUGPR_HIP(hipMemcpyAsync(c->d_pan_diag, pd.data(), pd.size() * sizeof(BuildItem), hipMemcpyHostToDevice, s));
  NUGPR_HIP(hipMemcpyAsync(c->d_pan_c, pc.data(), pc.size() * sizeof(BuildItem), hipMemcpyHostToDevice, s));
  NUGPR_HIP(hipStreamSynchronize(s));   // the host vectors are about to go out of scope
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
    hipLaunchKernelGGL(k_build_W, grid, dim3(256), 0, s, c->d_cl, c->X, c->reps, c->Wd, c->Wt, c->assign, L.r, L.d,
                       (uint32_t)L.ldw);
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

// pair_param < 0: one assembly at theta.  Otherwise theta holds the centre of a central difference in
// lengthscale pair_param with step h on its logarithm: ell e^{+h} goes to the blocks in force (Kd, C),
// ell e^{-h} to the spare ones (Kd2, C2); theta_built / theta_spare record which is which.
static int build_impl(nugpr_ctx* c, const double* theta, hipStream_t s, bool need_upper, int pair_param, double h,
                      double value_plus, double value_minus) {
  const Layout& L = c->L;
  if (!theta) { set_error("theta is null"); return NUGPR_ERR_INVALID; }
  for (int i = 0; i < L.p; ++i)
    if (!(theta[i] > 0.0) || !std::isfinite(theta[i])) { set_error("theta entries must be finite and > 0"); return NUGPR_ERR_INVALID; }
  const bool iso = (c->params.flags & NUGPR_ISOTROPIC) != 0;
  const double alpha = theta[L.p - 2], sigma2 = theta[L.p - 1];
  ScaleArgs sa;
  const double half_log2e = 0.5 * 1.4426950408889634074;
  for (int k = 0; k < MAX_D; ++k) sa.sw[k] = 0.0;
  for (int k = 0; k < L.d; ++k) {
    const double ell = iso ? theta[0] : theta[k];
    sa.sw[k] = std::sqrt(half_log2e) / ell;
  }
  sa.d = L.d;
  PanelArgs a;
  for (int k = 0; k < EXP2_TERMS; ++k) a.coef[k] = alpha * EXP2_COEF[k];
  a.diag_val = (float)(alpha + sigma2);
  a.mirror = need_upper ? 1 : 0;
  a.kd = pair_kd(L.d);
  a.keep_same = 0;
  a.g[0] = a.g[1] = 0.0;
  a.pair_dim = -1;
  const bool pair = pair_param >= 0;
  if (pair) {
    if (L.compensate || pair_param >= L.p - 2) { set_error("pair assembly: not a lengthscale, or compensation is on"); return NUGPR_ERR_INVALID; }
    // squared scaled distances go with ell^-2: factors e^{-2h} and e^{+2h}
    const double gp = std::expm1(-2.0 * h), gm = std::expm1(2.0 * h);
    if (iso) { a.g[0] = gp; a.g[1] = gm; a.pair_dim = -1; }             // exponent e (1 + g)
    else { a.g[0] = -gp; a.g[1] = -gm; a.pair_dim = pair_param; }       // exponent e - g (u_k - v_k)^2, e = -|u - v|^2
  }
  c->diag_residual = (float)((alpha + sigma2) - (double)a.diag_val);
  PanelArgs ac = a;                                  // the coupling launch
  // the upper tiles of C can be left out only if its strips pair up in the product (and nothing else reads them)
  const bool need_c_upper = need_upper || L.compensate || !c->c_paired;
  ac.mirror = need_c_upper ? 1 : 0;
  const bool host_lambda = L.compensate && L.ncr <= COMPENSATE_HOST_MAX;
  if (L.compensate && !host_lambda) {
    // large coupling: the matrix is assembled with a zero diagonal first, lambda_0 comes from an eigenvalue
    // iteration on the assembled matrix (below), and the diagonal alpha - lambda_0 is written last
    ac.keep_same = 1;
    ac.diag_val = 0.f;
  }
  if (host_lambda) {
    // lambda_0 = smallest eigenvalue of the representatives' kernel matrix (eq. (krep)), fp64 on the host
    const int N = L.ncr;
    std::vector<double> Cm((size_t)N * N);
    const double* R = c->h_reps.data();
    for (int i = 0; i < N; ++i)
      for (int j = 0; j <= i; ++j) {
        double q = 0.0;
        for (int k = 0; k < L.d; ++k) {
          const double t = (R[(size_t)i * L.d + k] - R[(size_t)j * L.d + k]) / (iso ? theta[0] : theta[k]);
          q += t * t;
        }
        Cm[(size_t)i * N + j] = Cm[(size_t)j * N + i] = alpha * std::exp(-0.5 * q);
      }
    double lam0 = 0.0;
    if (sym_smallest_eigenvalue(Cm, N, &lam0)) { set_error("lambda_0: eigen-solve did not converge"); return NUGPR_ERR_INVALID; }
    c->lambda0 = lam0;
    c->lambda0_steps = 0;
    ac.keep_same = 1;
    ac.diag_val = (float)(alpha - lam0);
  }
  c->assembly_mark = c->assembly_mark >= 0x7ffffff0 ? 1 : c->assembly_mark + 1;
  hipLaunchKernelGGL(k_scale_points, dim3((unsigned)L.ntmax, (unsigned)L.nc), dim3(256), 0, s, sa, c->d_cl, c->X, c->Xs,
                     c->Xn, 0, 0, c->d_state, c->assembly_mark);
  hipLaunchKernelGGL(k_scale_points, dim3((unsigned)(L.ldc / TILE), 1u), dim3(256), 0, s, sa,
                     (const ClusterInfo*)nullptr, c->reps, c->Rs, c->Rn, L.ncr, L.ldc, c->d_state, c->assembly_mark);
  const dim3 gd((unsigned)c->n_pan_diag), gc((unsigned)c->n_pan_c), blk(256);
  const size_t lds = (size_t)4 * a.kd * 16 * sizeof(double);      // row operands of one tile
#define NUGPR_TILES(NKS)                                                                                         \
  do {                                                                                                           \
    if (pair) {                                                                                                  \
      hipLaunchKernelGGL((k_build_tile<true, NKS, true>), gc, blk, lds, s, ac, c->d_pan_c, c->Rs, c->Rn, c->C, L.r, c->C2);      \
      hipLaunchKernelGGL((k_build_tile<false, NKS, true>), gd, blk, lds, s, a, c->d_pan_diag, c->Xs, c->Xn, c->Kd, 1, c->Kd2);   \
    } else {                                                                                                     \
      hipLaunchKernelGGL((k_build_tile<true, NKS, false>), gc, blk, lds, s, ac, c->d_pan_c, c->Rs, c->Rn, c->C, L.r, (float*)nullptr);    \
      hipLaunchKernelGGL((k_build_tile<false, NKS, false>), gd, blk, lds, s, a, c->d_pan_diag, c->Xs, c->Xn, c->Kd, 1, (float*)nullptr); \
    }                                                                                                            \
  } while (0)
  switch (a.kd / 4) {        // the dimensions of the usual workloads get their own instantiation
    case 1: NUGPR_TILES(1); break;
    case 2: NUGPR_TILES(2); break;
    case 5: NUGPR_TILES(5); break;
    default: NUGPR_TILES(0); break;
  }
#undef NUGPR_TILES
  NUGPR_HIP(hipGetLastError());
  if (L.compensate) {
    CouplingArgs ca;
    for (int k = 0; k < MAX_D; ++k) ca.inv_ell[k] = k < L.d ? 1.0 / (iso ? theta[0] : theta[k]) : 0.0;
    // (large coupling: the diagonal is zero for now, in both terms)
    ca.alpha = alpha; ca.lambda0 = host_lambda ? c->lambda0 : alpha; ca.n = L.ncr; ca.d = L.d; ca.ld = (uint32_t)L.ldc;
    const unsigned blocks = (unsigned)(((uint64_t)L.ldc * L.ldc + 255) / 256);
    hipLaunchKernelGGL(k_coupling_residual, dim3(blocks), dim3(256), 0, s, ca, c->reps, c->C, c->Clo);
    NUGPR_HIP(hipGetLastError());
    if (!host_lambda) {
      double lam0 = 0.0;
      int steps = 0;
      int rc = coupling_lambda_min(c, theta, s, &lam0, &steps);
      if (rc) return rc;
      c->lambda0 = lam0;
      c->lambda0_steps = steps;
      if ((rc = coupling_set_diag(c, alpha - lam0, s))) return rc;
    }
  }
  c->theta_built.assign(theta, theta + L.p);
  c->theta_spare.clear();
  if (pair) {
    c->theta_spare = c->theta_built;
    c->theta_built[pair_param] = value_plus;      // the caller's own values of ell e^{+h} and ell e^{-h}
    c->theta_spare[pair_param] = value_minus;
  }
  if (pair) c->lf_valid = false;              // the second matrix of the pair has just overwritten the Cholesky factor
  c->spare_upper_valid = pair && need_upper;
  c->c_upper_valid = need_c_upper;
  c->spare_c_upper_valid = pair && need_c_upper;
  c->op_scale = 1.0;
  c->op_shift = (double)c->diag_residual;
  c->built = true;
  c->kd_upper_valid = need_upper;
  c->build_gen += 1;
  c->stats.assembly_passes += 1;
  c->stats.matrices_assembled += pair ? 2 : 1;
  return NUGPR_OK;
}

int launch_build(nugpr_ctx* c, const double* theta, hipStream_t s, bool need_upper) {
  return build_impl(c, theta, s, need_upper, -1, 0.0, 0.0, 0.0);
}

int launch_build_pair(nugpr_ctx* c, const double* theta, int param, double h, double value_plus, double value_minus,
                      hipStream_t s, bool need_upper) {
  return build_impl(c, theta, s, need_upper, param, h, value_plus, value_minus);
}

int swap_pair(nugpr_ctx* c) {
  if (c->theta_spare.empty()) { set_error("no spare blocks to switch to"); return NUGPR_ERR_STATE; }
  std::swap(c->Kd, c->Kd2);
  std::swap(c->C, c->C2);
  c->theta_built.swap(c->theta_spare);
  c->theta_spare.clear();               // the blocks left behind are not used again
  c->kd_upper_valid = c->spare_upper_valid;
  c->c_upper_valid = c->spare_c_upper_valid;
  c->build_gen += 1;
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
    if (what == 1 && !c->lf_valid) {
      set_error("the Cholesky factor's storage has since been reused by a lengthscale pair assembly (nugpr_train_step); "
                "call nugpr_precond_factor again");
      return NUGPR_ERR_STATE;
    }
    if (what == 0) {
      const int rc = ensure_kd_upper(c, s);
      if (rc) return rc;
    }
  } else if (what == 3) {
    if (!c->built) { set_error("nothing stored yet"); return NUGPR_ERR_STATE; }
    {
      const int rc = ensure_c_upper(c, s);
      if (rc) return rc;
    }
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
    hipLaunchKernelGGL((k_export<double>), dim3(2048), dim3(256), 0, s, (const double*)c->Bv, lds, dst, ld, rows, cols, lower, 0);
  else
    hipLaunchKernelGGL((k_export<float>), dim3(2048), dim3(256), 0, s, what == 5 ? (const float*)c->Bv : src, lds, dst, ld,
                       rows, cols, lower, what <= 3 ? 1 : 0);     // K_ii, L_i, L_i^-1 and C are stored blocked
  NUGPR_HIP(hipGetLastError());
  NUGPR_HIP(hipStreamSynchronize(s));
  return NUGPR_OK;
}

}  // namespace nugpr
