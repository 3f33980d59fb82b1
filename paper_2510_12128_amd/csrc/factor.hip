// Block-Jacobi preconditioner (Section 3.2, eq. (cholesky factorization)): batched
// Cholesky K_ii = L_i L_i^T of every diagonal block, the explicit inverses L_i^-1 (the
// paper applies the factor as an explicit inverse followed by batched products, Table 2),
// log det of the preconditioner, and the right-hand sides B = [y | L Z].
//
// Everything is tiled in 64 x 64 fp32 tiles whose products run on the matrix cores
// (v_mfma_f32_16x16x4_f32, four waves per tile, each 32 x 32).
//   Cholesky: left-looking over tile columns.  Step k: every tile (m, k), m >= k, gets
//     A[m,k] - sum_{j<k} L[m,j] L[k,j]^T in one batched launch over clusters (most of
//     the sum one step ahead, see k_potrf_update); the workgroup that owns the diagonal
//     tile factors and inverts it in registers; a second launch multiplies the tiles
//     below by that inverse.
//   Inverse: the binary-tree identity
//     [L11 0; L21 L22]^-1 = [Y11 0; -Y22 L21 Y11, Y22]
//     applied bottom-up over tile ranges, two batched products per level
//     (T = L21 Y11, kept transposed in the still unused upper triangle; Y21 = -Y22 T).
//   The inverse is finally mirrored into the upper triangle so that both halves of the
//   preconditioner apply, tril(G) r and triu(G) v, stream row-major strips.
// log det of the preconditioner is taken from the STORED inverse, -2 sum log Y_pp, so the
// split of eq. (logdet) holds exactly for the operator PCG really applies.
#include <climits>
#include <cmath>

#include "nugpr_internal.h"

namespace nugpr {

typedef float v4f __attribute__((ext_vector_type(4)));
constexpr int KS = 32;          // contraction depth per LDS stage (two 16-deep halves per thread)
constexpr int SP = KS + 1;      // padded LDS row

struct Frag {          // one thread's share of a 64 x 32 operand stage: four elements of each 16-deep half
  float v[8];
};

// Logical operand Op[r][k]; memory is element (r, k) (TRANS = false) or (k, r) of a matrix stored in blocks of
// 16 x 16 fragments (blocked_index): the four elements a thread loads are consecutive in a fragment row, and the
// 64 threads of a wave load one whole fragment, 1 KiB in one piece.
// tri: 0 none, 1 keep k <= r, 2 keep k >= r (r, k are coordinates inside the same square block).
template <bool TRANS>
__device__ __forceinline__ Frag fetch(const float* __restrict__ base, uint32_t ld, int r0, int k0, int rmax,
                                      int tri, int tid) {
  Frag f;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    float* v = f.v + 4 * h;
    if (!TRANS) {
      const int r = r0 + (tid >> 2), k = k0 + 16 * h + (tid & 3) * 4;
      if (r < rmax) {
        const float4 x = *reinterpret_cast<const float4*>(base + blocked_index(ld, r, k));
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
      } else {
        v[0] = v[1] = v[2] = v[3] = 0.f;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (tri == 1 && k + j > r) v[j] = 0.f;
        if (tri == 2 && k + j < r) v[j] = 0.f;
      }
    } else {
      const int k = k0 + 16 * h + (tid >> 4), r = r0 + (tid & 15) * 4;
      const float4 x = *reinterpret_cast<const float4*>(base + blocked_index(ld, k, r));
      v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (r + j >= rmax) v[j] = 0.f;
        if (tri == 1 && k > r + j) v[j] = 0.f;
        if (tri == 2 && k < r + j) v[j] = 0.f;
      }
    }
  }
  return f;
}

template <bool TRANS>
__device__ __forceinline__ void commit(float (*s)[SP], const Frag& f, int tid) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    if (!TRANS) {
      const int r = tid >> 2, k = 16 * h + (tid & 3) * 4;
#pragma unroll
      for (int j = 0; j < 4; ++j) s[r][k + j] = f.v[4 * h + j];
    } else {
      const int k = 16 * h + (tid >> 4), r = (tid & 15) * 4;
#pragma unroll
      for (int j = 0; j < 4; ++j) s[r + j][k] = f.v[4 * h + j];
    }
  }
}

struct Operand {
  const float* base;
  uint32_t ld;
  int r0;      // first logical row of the 64-row tile
  int rmax;    // rows >= rmax read as zero
  int tri;
};

// acc[i][j] += OpA[64 x K] * OpB[64 x K]^T over k in [k0, k1), k0/k1 multiples of 32 (all callers pass tile boundaries).
// The operands enter the matrix instruction in swapped roles (OpB as its row operand), which transposes the
// 16 x 16 result inside the registers: lane l holds C[row l & 15][columns 4 (l >> 4) .. + 3], four consecutive
// columns of one row, i.e. 16 bytes of a row-major fragment, and the 64 lanes of a wave one whole fragment
// (1 KiB in one piece): tiles are read and written with one 16-byte access per lane and fragment.
template <bool TA, bool TB>
__device__ __forceinline__ void tile_gemm(v4f (&acc)[2][2], const Operand& A, const Operand& B, int k0, int k1,
                                          float (*sA)[SP], float (*sB)[SP], int tid) {
  const int wave = tid >> 6, lane = tid & 63;
  const int wy = wave >> 1, wx = wave & 1;
  const int m = lane & 15, kk = lane >> 4;
  if (k0 >= k1) return;
  Frag fa = fetch<TA>(A.base, A.ld, A.r0, k0, A.rmax, A.tri, tid);
  Frag fb = fetch<TB>(B.base, B.ld, B.r0, k0, B.rmax, B.tri, tid);
  for (int k = k0; k < k1; k += KS) {
    __syncthreads();
    commit<TA>(sA, fa, tid);
    commit<TB>(sB, fb, tid);
    __syncthreads();
    if (k + KS < k1) {
      fa = fetch<TA>(A.base, A.ld, A.r0, k + KS, A.rmax, A.tri, tid);
      fb = fetch<TB>(B.base, B.ld, B.r0, k + KS, B.rmax, B.tri, tid);
    }
#pragma unroll
    for (int ks = 0; ks < KS / 4; ++ks) {
      const float a0 = sA[wy * 32 + m][4 * ks + kk];
      const float a1 = sA[wy * 32 + 16 + m][4 * ks + kk];
      const float b0 = sB[wx * 32 + m][4 * ks + kk];
      const float b1 = sB[wx * 32 + 16 + m][4 * ks + kk];
      acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(b0, a0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(b1, a0, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(b0, a1, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(b1, a1, acc[1][1], 0, 0, 0);
    }
  }
}

__device__ __forceinline__ void zero_acc(v4f (&acc)[2][2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};
}

// visit every accumulator element with its (row, col) inside the 64 x 64 tile
template <class F>
__device__ __forceinline__ void for_each_acc(v4f (&acc)[2][2], int tid, F f) {
  const int wave = tid >> 6, lane = tid & 63;
  const int wy = wave >> 1, wx = wave & 1;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        f(wy * 32 + 16 * i + (lane & 15), wx * 32 + 16 * j + 4 * (lane >> 4) + v, acc[i][j][v]);
}
// the same, four consecutive columns at a time: f(row, first column (a multiple of 4), the four values)
template <class F>
__device__ __forceinline__ void for_each_acc4(v4f (&acc)[2][2], int tid, F f) {
  const int wave = tid >> 6, lane = tid & 63;
  const int wy = wave >> 1, wx = wave & 1;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) f(wy * 32 + 16 * i + (lane & 15), wx * 32 + 16 * j + 4 * (lane >> 4), acc[i][j]);
}

// Blocked storage seen tile by tile: element (r, q) of the 64 x 64 tile (tr, tc) of a square block lies at
// tile_base(ld, tr, tc) + tile_offset(r, q) (= blocked_index(ld, 64 tr + r, 64 tc + q)).  The base is uniform over a
// workgroup and computed once; the offset is a few 32-bit shifts, and with the accumulator coordinates of
// for_each_acc most of it is a compile-time constant.
__device__ __forceinline__ uint64_t tile_base(uint32_t ld, int tr, int tc) {
  return (uint64_t)tr * TILE * ld + (uint64_t)tc * (2 * TILE * BLK_COLS);
}
__device__ __forceinline__ uint32_t tile_offset(int r, int q) {
  return (uint32_t)((q >> 5) * (TILE * BLK_COLS) + (((r >> 4) * 2 + ((q & 31) >> 4)) * FRAG) + (r & 15) * 16 + (q & 15));
}

// Workgroup -> (cluster, item) for a launch of `per` items for each of `nc` clusters: a 1-D grid of
// die_grid(per, nc) workgroups.  Workgroups go round-robin to the 8 dies, each with an L2 of its own: with
// the cluster as the slow index of a plain grid the tiles of one cluster, which all read the same panel,
// would be spread over every die and the panel fetched eight times.  With nc > 0 die d takes the clusters
// d, d + 8, .. one after the other (the grid is rounded up to whole groups of 8 clusters; workgroups that
// fall past the last cluster return at once).  That ties a cluster's work to one die: with clusters of
// very different sizes the dies would finish far apart, and the host then passes -nc for the plain order
// (cluster = slow index), which spreads every cluster over all dies (configuration 5: 302 against 353 ms).
constexpr int NUM_DIES = 8;
static inline unsigned die_grid(int per, int nc) {
  const int n = nc < 0 ? -nc : nc;
  return (unsigned)per * NUM_DIES * ((n + NUM_DIES - 1) / NUM_DIES);
}
__device__ __forceinline__ bool die_local_item(int per, int nc, int& cluster, int& item, int id = (int)blockIdx.x) {
  if (nc < 0) {
    cluster = id / per;
    item = id % per;
    return cluster < -nc;
  }
  const int die = id % NUM_DIES, slot = id / NUM_DIES;
  cluster = die + NUM_DIES * (slot / per);
  item = slot % per;
  return cluster < nc;
}

// ---------------------------------------------------------------------------
// Cholesky, step k
// ---------------------------------------------------------------------------
// Left-looking, with the bulk of every tile's update done one step ahead.  The launch of step k has two
// kinds of workgroups:
//   diagonal  tile (k, k): subtract the contribution of column k - 1 (the only one that was not final when the
//             bulk of this tile was computed), then factor and invert the tile
//   row m > k two tiles of the same block row, one after the other:
//             finish (m, k): subtract the contribution of column k - 1, as above;
//             bulk (m, k + 1): L <- A - sum over the columns < k, all final by now
// The factorisation of the diagonal tile is serial and keeps one workgroup per cluster busy for tens of
// microseconds; with the long products of the NEXT column in the same launch the rest of the chip has work
// meanwhile, where a launch that only finished column k would idle behind its diagonal tiles.
// Grid order = start order (workgroups are handed out in index order, a few thousand take tens of
// microseconds): the diagonal tiles of all clusters first, since the launch cannot end before they do.  Finish
// and bulk of a block row share a workgroup because, as workgroups of their own, the short finish ones either
// delay the start of the long ones or wait behind them for a free slot: measured 25 us per launch.
__global__ __launch_bounds__(256) void k_potrf_update(const ClusterInfo* __restrict__ cl, const float* Kd,
                                                      float* Lf, float* __restrict__ G, int k,
                                                      int n_rows, int grid_diag, int nc, PcgState* __restrict__ st) {
  // the operand stages and, once the products are done, the tile on its way into the registers of the
  // factorisation (then its exchange buffers) share one piece of LDS: 16.5 KB per workgroup
  static_assert(2 * TILE * SP >= TILE * (TILE + 1), "the tile to be factored must fit in the operand stages");
  __shared__ __attribute__((aligned(16))) float stage[2 * TILE * SP];
  float (*sA)[SP] = reinterpret_cast<float (*)[SP]>(stage);
  float (*sB)[SP] = reinterpret_cast<float (*)[SP]>(stage + TILE * SP);
  float (*sT)[TILE + 1] = reinterpret_cast<float (*)[TILE + 1]>(stage);
  const int id = (int)blockIdx.x;
  const bool diag = id < grid_diag;
  int ci, item;
  if (diag) {
    if (!die_local_item(1, nc, ci, item, id)) return;
  } else {
    if (!die_local_item(n_rows, nc, ci, item, id - grid_diag)) return;
    item += 1;
  }
  const ClusterInfo c = cl[ci];
  const int mt = k + item;                     // block row of this workgroup
  if (mt >= (int)c.nt) return;
  const int tid = threadIdx.x;
  const int b = (int)c.b;
  const float* A = Kd + c.koff;
  float* L = Lf + c.koff;
  v4f acc[2][2];
  zero_acc(acc);
  Operand oa{L, c.ld, mt * TILE, b, 0};
  Operand ob{L, c.ld, k * TILE, b, 0};
  if (k > 0) tile_gemm<false, false>(acc, oa, ob, (k - 1) * TILE, k * TILE, sA, sB, tid);
  // what the products are subtracted from: the assembled block, or the bulk result of the step before
  const float* base = k == 0 ? A : L;
  if (!diag) {
    {
      const uint64_t tb = tile_base(c.ld, mt, k);
      const float* bt = base + tb;
      float* lt = L + tb;
      for_each_acc4(acc, tid, [&](int r, int q, const v4f& v) {
        const uint32_t at = tile_offset(r, q);
        const float4 x = *reinterpret_cast<const float4*>(bt + at);
        *reinterpret_cast<float4*>(lt + at) = make_float4(x.x - v[0], x.y - v[1], x.z - v[2], x.w - v[3]);
      });
    }
    zero_acc(acc);
    Operand oc{L, c.ld, (k + 1) * TILE, b, 0};
    if (k > 0) tile_gemm<false, false>(acc, oa, oc, 0, k * TILE, sA, sB, tid);
    {
      const uint64_t tb = tile_base(c.ld, mt, k + 1);
      const float* at_ = A + tb;
      float* lt = L + tb;
      for_each_acc4(acc, tid, [&](int r, int q, const v4f& v) {
        const uint32_t at = tile_offset(r, q);
        const float4 x = *reinterpret_cast<const float4*>(at_ + at);
        *reinterpret_cast<float4*>(lt + at) = make_float4(x.x - v[0], x.y - v[1], x.z - v[2], x.w - v[3]);
      });
    }
    return;
  }
  // ---- diagonal tile: factor and invert it; rows/cols past the cluster end behave as identity ----
  // This workgroup is the critical path of the whole launch (the next launch needs its result) and shares its
  // compute unit with workgroups that keep the matrix cores busy, which slows every instruction it issues: so
  // the tile lives in REGISTERS and a pivot costs one LDS round trip and one barrier.  Wave w owns the columns
  // 16 w .. 16 w + 15 of all 64 rows, lane i the row i: a[u] = A[i][16 w + u], y[u] = Y[i][16 w + u].
  // Elimination without square roots (A = Lu D Lu^T, Lu unit lower) applied to [A | I]:
  //   pivot j:  m_i = a_ij / d_j (i > j);  a_ic -= m_i a_cj (c > j);  y_ic -= m_i y_jc (c <= j)
  // leaves a_ic = (Lu D)_ic below the diagonal, d on it, and Y = Lu^-1; then L = Lu D^1/2, L^-1 = D^-1/2 Lu^-1.
  // Per pivot the owners publish column j of A (one value per row) and row j of Y in LDS, double-buffered so
  // that one barrier per pivot is enough.
  __syncthreads();                              // every wave is done reading the operand stages
  const int valid = min(TILE, b - k * TILE);
  const float* bkk = base + tile_base(c.ld, k, k);
  for_each_acc4(acc, tid, [&](int r, int q, const v4f& v) {
    const float4 b4 = *reinterpret_cast<const float4*>(bkk + tile_offset(r, q));
    const float x[4] = {b4.x - v[0], b4.y - v[1], b4.z - v[2], b4.w - v[3]};
#pragma unroll
    for (int u = 0; u < 4; ++u) sT[r][q + u] = (r >= valid || q + u >= valid) ? (r == q + u ? 1.f : 0.f) : x[u];
  });
  __syncthreads();
  const int w = tid >> 6, i = tid & 63;
  float a[16], y[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    a[u] = sT[i][16 * w + u];
    y[u] = (16 * w + u == i) ? 1.f : 0.f;
  }
  __syncthreads();                              // sT is dead from here on: its memory holds the exchange buffers
  float* colbuf = stage;                        // [2][64]  column j of A, by row
  float* rowbuf = stage + 2 * TILE;             // [2][64]  row j of Y
  float* dvec = stage + 4 * TILE;               // [64]     the pivots d_j
  bool bad = false;
#pragma unroll 1
  for (int jb = 0; jb < 4; ++jb) {
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      const int j = 16 * jb + jj;
      float* cb = colbuf + (j & 1) * TILE;
      float* rb = rowbuf + (j & 1) * TILE;
      if (w == jb) cb[i] = a[jj];
      if (i == j) {
#pragma unroll
        for (int u = 0; u < 16; u += 4) *reinterpret_cast<float4*>(rb + 16 * w + u) = make_float4(y[u], y[u + 1], y[u + 2], y[u + 3]);
      }
      __syncthreads();
      float dj = cb[j];
      if (!(dj > 0.f) || !(dj < INFINITY)) { bad = true; dj = 1.f; }
      if (tid == 0) dvec[j] = dj;
      const float mi = i > j ? cb[i] / dj : 0.f;
      if (w > jb) {                             // all 16 columns of this wave lie right of the pivot
#pragma unroll
        for (int u = 0; u < 16; u += 4) {
          const float4 cj = *reinterpret_cast<const float4*>(cb + 16 * w + u);
          a[u] = fmaf(-mi, cj.x, a[u]); a[u + 1] = fmaf(-mi, cj.y, a[u + 1]);
          a[u + 2] = fmaf(-mi, cj.z, a[u + 2]); a[u + 3] = fmaf(-mi, cj.w, a[u + 3]);
        }
      } else if (w == jb) {
#pragma unroll
        for (int u = jj + 1; u < 16; ++u) a[u] = fmaf(-mi, cb[16 * w + u], a[u]);
      }
      if (w <= jb) {                            // Y_j is zero right of column j
#pragma unroll
        for (int u = 0; u < 16; u += 4) {
          const float4 yj = *reinterpret_cast<const float4*>(rb + 16 * w + u);
          y[u] = fmaf(-mi, yj.x, y[u]); y[u + 1] = fmaf(-mi, yj.y, y[u + 1]);
          y[u + 2] = fmaf(-mi, yj.z, y[u + 2]); y[u + 3] = fmaf(-mi, yj.w, y[u + 3]);
        }
      }
    }
  }
  __syncthreads();                              // dvec complete
  if (bad && tid == 0) atomicMin(&st->bad_cluster, ci);
  // L_ic = a_ic / sqrt(d_c) (c < i), sqrt(d_i) on the diagonal;  (L^-1)_ic = y_ic / sqrt(d_i) (c <= i)
  const float rsi = 1.f / sqrtf(dvec[i]);
  float* Y = G + c.koff;
  const uint64_t at = tile_base(c.ld, k, k) + tile_offset(i, 16 * w);     // one fragment row: 16 floats
#pragma unroll
  for (int u = 0; u < 16; u += 4) {
    float lo[4], yo[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int cc = 16 * w + u + v;
      const float sc = sqrtf(dvec[cc]);
      lo[v] = cc < i ? a[u + v] / sc : (cc == i ? sc : 0.f);
      yo[v] = cc <= i ? y[u + v] * rsi : 0.f;
    }
    *reinterpret_cast<float4*>(L + at + u) = make_float4(lo[0], lo[1], lo[2], lo[3]);
    *reinterpret_cast<float4*>(Y + at + u) = make_float4(yo[0], yo[1], yo[2], yo[3]);
  }
}

// tiles below the diagonal: L[m,k] <- L[m,k] * inv(L[k,k])^T
__global__ __launch_bounds__(256) void k_potrf_trsm(const ClusterInfo* __restrict__ cl, float* __restrict__ Lf,
                                                    const float* __restrict__ G, int k, int per, int nc) {
  __shared__ __attribute__((aligned(16))) float sA[TILE][SP];
  __shared__ __attribute__((aligned(16))) float sB[TILE][SP];
  int ci, item;
  if (!die_local_item(per, nc, ci, item)) return;
  const ClusterInfo c = cl[ci];
  const int mt = k + 1 + item;
  if (mt >= (int)c.nt) return;
  const int tid = threadIdx.x;
  float* L = Lf + c.koff;
  const float* Y = G + c.koff;
  v4f acc[2][2];
  zero_acc(acc);
  Operand oa{L, c.ld, mt * TILE, (int)c.b, 0};
  Operand ob{Y, c.ld, k * TILE, (int)c.ld, 1};          // Y_kk[c][j], lower triangular
  tile_gemm<false, false>(acc, oa, ob, k * TILE, (k + 1) * TILE, sA, sB, tid);
  __syncthreads();
  float* lt = L + tile_base(c.ld, mt, k);
  for_each_acc4(acc, tid, [&](int r, int q, const v4f& v) {
    *reinterpret_cast<float4*>(lt + tile_offset(r, q)) = make_float4(v[0], v[1], v[2], v[3]);
  });
}

// ---------------------------------------------------------------------------
// triangular inverse, one tree level (half = tiles per child)
// ---------------------------------------------------------------------------
// stage 1: T = L21 * Y11, stored transposed in the mirror block (upper triangle of G)
__global__ __launch_bounds__(256) void k_trtri_stage1(const ClusterInfo* __restrict__ cl, const float* __restrict__ Lf,
                                                      float* __restrict__ G, int half, int per, int nc) {
  __shared__ __attribute__((aligned(16))) float stage[2 * TILE * SP];   // operand stages, then the tile on its way to the mirror block
  float (*sA)[SP] = reinterpret_cast<float (*)[SP]>(stage);
  float (*sB)[SP] = reinterpret_cast<float (*)[SP]>(stage + TILE * SP);
  float (*sT)[TILE + 1] = reinterpret_cast<float (*)[TILE + 1]>(stage);
  int ci, item;
  if (!die_local_item(per, nc, ci, item)) return;
  const ClusterInfo c = cl[ci];
  const int node = item / (half * half), within = item % (half * half);
  const int start = node * 2 * half, mid = start + half;
  const int tm = mid + within / half, tn = start + within % half;
  if (mid >= (int)c.nt || tm >= (int)c.nt) return;
  const int tid = threadIdx.x;
  const float* L = Lf + c.koff;
  float* Y = G + c.koff;
  v4f acc[2][2];
  zero_acc(acc);
  Operand oa{L, c.ld, tm * TILE, (int)c.b, 0};          // L21[m][k]
  Operand ob{Y, c.ld, tn * TILE, (int)c.ld, 2};         // OpB[n][k] = Y11[k][n], nonzero for k >= n
  tile_gemm<false, true>(acc, oa, ob, tn * TILE, mid * TILE, sA, sB, tid);
  __syncthreads();                              // every wave is done reading the operand stages
  for_each_acc(acc, tid, [&](int r, int q, float v) { sT[r][q] = v; });
  __syncthreads();
  // mirror block: rows = columns of T (tile tn), columns = rows of T (tile tm)

  float* yt = Y + tile_base(c.ld, tn, tm);
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int q = idx >> 6, r = idx & 63;
    yt[tile_offset(q, r)] = sT[r][q];
  }
}

// stage 2: Y21 = -Y22 * T
__global__ __launch_bounds__(256) void k_trtri_stage2(const ClusterInfo* __restrict__ cl, float* __restrict__ G,
                                                      int half, int per, int nc) {
  __shared__ __attribute__((aligned(16))) float sA[TILE][SP];
  __shared__ __attribute__((aligned(16))) float sB[TILE][SP];
  int ci, item;
  if (!die_local_item(per, nc, ci, item)) return;
  const ClusterInfo c = cl[ci];
  const int node = item / (half * half), within = item % (half * half);
  const int start = node * 2 * half, mid = start + half;
  const int tm = mid + within / half, tn = start + within % half;
  if (mid >= (int)c.nt || tm >= (int)c.nt) return;
  const int tid = threadIdx.x;
  float* Y = G + c.koff;
  v4f acc[2][2];
  zero_acc(acc);
  Operand oa{Y, c.ld, tm * TILE, (int)c.b, 1};          // Y22[m][k], nonzero for k <= m
  Operand ob{Y, c.ld, tn * TILE, (int)c.ld, 0};         // OpB[n][k] = T[k][n], read from the mirror block
  tile_gemm<false, false>(acc, oa, ob, mid * TILE, (tm + 1) * TILE, sA, sB, tid);
  float* yt = Y + tile_base(c.ld, tm, tn);
  for_each_acc4(acc, tid, [&](int r, int q, const v4f& v) {
    *reinterpret_cast<float4*>(yt + tile_offset(r, q)) = make_float4(-v[0], -v[1], -v[2], -v[3]);
  });
}

// upper triangle <- transpose of the lower triangle (tile list of the assembly kernels)
__global__ __launch_bounds__(256) void k_mirror(const ClusterInfo* __restrict__ cl, const uint64_t* __restrict__ tiles,
                                                float* __restrict__ G) {
  __shared__ float sT[TILE][TILE + 1];
  const uint64_t t = tiles[blockIdx.x];
  const int ci = (int)(t >> 32), tr = (int)((t >> 16) & 0xffff), tc = (int)(t & 0xffff);
  const ClusterInfo c = cl[ci];
  float* Y = G + c.koff;
  const int tid = threadIdx.x;

  const float* ys = Y + tile_base(c.ld, tr, tc);
  float* yd = Y + tile_base(c.ld, tc, tr);
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;
    sT[r][q] = ys[tile_offset(r, q)];
  }
  __syncthreads();
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;      // element (r, q) of the destination tile
    if (tr != tc || q > r) yd[tile_offset(r, q)] = sT[q][r];
  }
}

// upper tiles of one square blocked matrix of nt x nt tiles <- transposes of the lower ones (1-D grid of nt * nt)
__global__ __launch_bounds__(256) void k_mirror_square(float* __restrict__ M, uint32_t ld, int nt) {
  __shared__ float sT[TILE][TILE + 1];
  const int tr = (int)(blockIdx.x / (unsigned)nt), tc = (int)(blockIdx.x % (unsigned)nt);
  if (tc >= tr) return;
  const int tid = threadIdx.x;
  const float* ms = M + tile_base(ld, tr, tc);
  float* md = M + tile_base(ld, tc, tr);
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;
    sT[r][q] = ms[tile_offset(r, q)];
  }
  __syncthreads();
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;
    md[tile_offset(r, q)] = sT[q][r];
  }
}

int ensure_c_upper(nugpr_ctx* c, hipStream_t s) {
  if (c->c_upper_valid || !c->built) return NUGPR_OK;
  const int nt = c->L.ldc / TILE;
  hipLaunchKernelGGL(k_mirror_square, dim3((unsigned)nt * (unsigned)nt), dim3(256), 0, s, c->C, (uint32_t)c->L.ldc, nt);
  NUGPR_HIP(hipGetLastError());
  c->c_upper_valid = true;
  return NUGPR_OK;
}

bool kd_lower_suffices(const nugpr_ctx* c) {
  // fp64 mode with 2..17 columns (one column group): the producer / consumer strip kernel pairs the tiles of
  // the symmetric blocks.  The Pade route also solves single columns, which read whole strips.
  return c->acc64 && c->L.T >= 2 && c->L.T <= 17 && !(c->params.flags & NUGPR_LOGDET_PADE);
}

int ensure_kd_upper(nugpr_ctx* c, hipStream_t s) {
  if (c->kd_upper_valid || !c->built) return NUGPR_OK;
  hipLaunchKernelGGL(k_mirror, dim3((unsigned)c->L.n_diag_tiles), dim3(256), 0, s, c->d_cl, c->d_tiles, c->Kd);
  NUGPR_HIP(hipGetLastError());
  c->kd_upper_valid = true;
  return NUGPR_OK;
}

// log det of the preconditioner of one cluster from the stored inverse diagonal
__global__ __launch_bounds__(256) void k_logdet(const ClusterInfo* __restrict__ cl, const float* __restrict__ G,
                                                double* __restrict__ out) {
  __shared__ double red[256];
  const ClusterInfo c = cl[blockIdx.x];
  const float* Y = G + c.koff;
  double s = 0.0;
  for (uint32_t p = threadIdx.x; p < c.b; p += 256) s += log((double)Y[blocked_index(c.ld, p, p)]);
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = -2.0 * red[0];
}

__global__ void k_reset_bad(PcgState* st) { st->bad_cluster = INT_MAX; }

// V = [0 | Z] (n x T) from the probes (n x t)
template <typename VT>
__global__ void k_probes_to_block(const float* __restrict__ Z, VT* __restrict__ V, int64_t n, int t) {
  const int T = t + 1;
  const int64_t total = n * T;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int64_t p = idx / T;
    const int col = (int)(idx - p * T);
    V[idx] = col == 0 ? (VT)0 : (VT)Z[p * t + col - 1];
  }
}

template <typename VT>
__global__ void k_set_col0(VT* __restrict__ B, const float* __restrict__ y, int64_t n, int T) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n; p += (int64_t)gridDim.x * blockDim.x)
    B[p * T] = (VT)y[p];
}

// Diagonal blocks of the compensated matrix (eq. (kypp)) with the one-hot basis: tile (tr, tc), tc <= tr, of
// cluster ci gets  K_ii[p][q] + Cc[a(p)][a(q)],  a(p) = the row of the coupling matrix that point p belongs to and
// Cc = C - lambda_0 I as stored (same-cluster entries kept, float(alpha - lambda_0) on the diagonal).  Reads the
// lower triangle of Cc element-wise (row >= column), which every storage mode keeps.  One workgroup per tile of
// the assembly's tile list; writes the spare blocks, where the factorisation then runs in place.
__global__ __launch_bounds__(256) void k_compensated_blocks(const ClusterInfo* __restrict__ cl,
                                                            const uint64_t* __restrict__ tiles,
                                                            const float* __restrict__ Kd, float* __restrict__ out,
                                                            const float* __restrict__ Cc, uint32_t ldc,
                                                            const int32_t* __restrict__ assign) {
  __shared__ int32_t ar[TILE], ac[TILE];
  const uint64_t t = tiles[blockIdx.x];
  const int ci = (int)(t >> 32), tr = (int)((t >> 16) & 0xffff), tc = (int)(t & 0xffff);
  const ClusterInfo c = cl[ci];
  const int tid = threadIdx.x;
  if (tid < TILE) {
    const uint32_t p = (uint32_t)(tr * TILE + tid);
    ar[tid] = p < c.b ? assign[c.row0 + p] : -1;
  } else if (tid < 2 * TILE) {
    const uint32_t q = (uint32_t)(tc * TILE + tid - TILE);
    ac[tid - TILE] = q < c.b ? assign[c.row0 + q] : -1;
  }
  __syncthreads();
  const uint64_t tb = tile_base(c.ld, tr, tc);
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;
    const uint32_t at = tile_offset(r, q);
    float v = Kd[c.koff + tb + at];
    const int a = ar[r], b = ac[q];
    if (a >= 0 && b >= 0) v += Cc[blocked_index(ldc, (uint32_t)max(a, b), (uint32_t)min(a, b))];
    out[c.koff + tb + at] = v;
  }
}

int launch_factor(nugpr_ctx* c, hipStream_t s) {
  const Layout& L = c->L;
  // clusters of similar size: one die per cluster; otherwise every cluster over all dies (see die_local_item)
  uint64_t tiles_sum = 0;
  for (const ClusterInfo& ci : L.cl) tiles_sum += ci.nt;
  const bool even = (uint64_t)L.ntmax * (uint64_t)L.nc * 4 <= tiles_sum * 5;
  const int ncm = even ? L.nc : -L.nc;
  c->Lf = c->Kd2;                 // the factor goes into the spare blocks (see nugpr_ctx::lf_valid)
  c->lf_valid = true;
  // what is factored: the assembled K_ii, or (NUGPR_PRECOND_COMPENSATED) the diagonal blocks of K'' formed in the
  // spare blocks, where the factorisation then runs in place (every tile is read before it is written)
  const float* Afac = c->Kd;
  if (c->params.flags & NUGPR_PRECOND_COMPENSATED) {
    if (!c->onehot) { set_error("NUGPR_PRECOND_COMPENSATED needs the default one-hot basis"); return NUGPR_ERR_STATE; }
    hipLaunchKernelGGL(k_compensated_blocks, dim3((unsigned)L.n_diag_tiles), dim3(256), 0, s, c->d_cl, c->d_tiles, c->Kd,
                       c->Kd2, c->C, (uint32_t)L.ldc, c->assign);
    Afac = c->Kd2;
  }
  hipLaunchKernelGGL(k_reset_bad, dim3(1), dim3(1), 0, s, c->d_state);
  for (int k = 0; k < L.ntmax; ++k) {
    const int n_rows = L.ntmax - k - 1;         // block rows below the diagonal tile
    const unsigned grid_diag = die_grid(1, ncm), grid_rows = n_rows > 0 ? die_grid(n_rows, ncm) : 0u;
    hipLaunchKernelGGL(k_potrf_update, dim3(grid_diag + grid_rows), dim3(256), 0, s, c->d_cl, Afac, c->Lf, c->G, k,
                       n_rows, (int)grid_diag, ncm, c->d_state);
    if (k + 1 < L.ntmax)
      hipLaunchKernelGGL(k_potrf_trsm, dim3(die_grid(L.ntmax - k - 1, ncm)), dim3(256), 0, s, c->d_cl, c->Lf, c->G, k,
                         L.ntmax - k - 1, ncm);
  }
  for (int half = 1; half < L.ntmax; half *= 2) {
    const int nodes = (L.ntmax + 2 * half - 1) / (2 * half);
    const int per = half * half * nodes;
    dim3 grid(die_grid(per, ncm));
    hipLaunchKernelGGL(k_trtri_stage1, grid, dim3(256), 0, s, c->d_cl, c->Lf, c->G, half, per, ncm);
    hipLaunchKernelGGL(k_trtri_stage2, grid, dim3(256), 0, s, c->d_cl, c->G, half, per, ncm);
  }
  hipLaunchKernelGGL(k_mirror, dim3((unsigned)L.n_diag_tiles), dim3(256), 0, s, c->d_cl, c->d_tiles, c->G);
  hipLaunchKernelGGL(k_logdet, dim3(L.nc), dim3(256), 0, s, c->d_cl, c->G, c->d_logdet);
  NUGPR_HIP(hipGetLastError());
  // right-hand sides B = [y | L Z]
  if (L.t > 0) {
    if (c->acc64)
      hipLaunchKernelGGL((k_probes_to_block<double>), dim3(1024), dim3(256), 0, s, c->probes, (double*)c->Pv, (int64_t)L.n, L.t);
    else
      hipLaunchKernelGGL((k_probes_to_block<float>), dim3(1024), dim3(256), 0, s, c->probes, (float*)c->Pv, (int64_t)L.n, L.t);
    StripPort p0{};
    p0.A = c->Lf; p0.in = c->Pv; p0.out = c->Bv; p0.nin = 1;
    int rc = launch_strip(c->tab_lowL, p0, p0, L.T, c->acc64, s);
    if (rc) return rc;
  }
  if (c->acc64) hipLaunchKernelGGL((k_set_col0<double>), dim3(1024), dim3(256), 0, s, (double*)c->Bv, c->y, (int64_t)L.n, L.T);
  else hipLaunchKernelGGL((k_set_col0<float>), dim3(1024), dim3(256), 0, s, (float*)c->Bv, c->y, (int64_t)L.n, L.T);
  NUGPR_HIP(hipGetLastError());
  // z_0 = M^-1 B of every later solve on these right-hand sides (x_0 = 0, so r_0 = B whatever theta is)
  c->z0_ready = false;
  int rc = run_precond(c, c->Bv, c->Z0v, L.T, s);
  if (rc) return rc;
  if ((rc = store_known_starts(c, s))) return rc;
  c->z0_ready = true;
  c->factor_gen = c->build_gen;
  c->stats.factorisations += 1;
  return NUGPR_OK;
}

}  // namespace nugpr
