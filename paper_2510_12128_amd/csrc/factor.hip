// Block-Jacobi preconditioner (Section 3.2, eq. (cholesky factorization)): batched
// Cholesky K_ii = L_i L_i^T of every diagonal block, the explicit inverses L_i^-1 (the
// paper applies the factor as an explicit inverse followed by batched products, Table 2),
// log det of the preconditioner, and the right-hand sides B = [y | L Z].
//
// Everything is tiled in 64 x 64 fp32 tiles whose products run on the matrix cores
// (v_mfma_f32_16x16x4_f32, four waves per tile, each 32 x 32).
//   Cholesky: left-looking over tile columns.  Step k: every tile (m, k), m >= k, gets
//     A[m,k] - sum_{j<k} L[m,j] L[k,j]^T in one batched launch over clusters; the
//     workgroup that owns the diagonal tile factors it in LDS and also writes its
//     inverse; a second launch multiplies the tiles below by that inverse.
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
      acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1, acc[1][1], 0, 0, 0);
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
        f(wy * 32 + 16 * i + 4 * (lane >> 4) + v, wx * 32 + 16 * j + (lane & 15), acc[i][j][v]);
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
//   finish  tile (m, k), m >= k: subtract the contribution of column k - 1, the only one that was not final
//           when the bulk was computed; the workgroup of the diagonal tile then factors and inverts it in LDS
//   bulk    tile (m, k + 1), m >= k + 1: L <- A - sum over the columns < k, all final by now
// The factorisation of the diagonal tile is serial and keeps one workgroup per cluster busy for tens of
// microseconds; with the long products of the NEXT column in the same launch the rest of the chip has work
// meanwhile, where a launch that only finished column k would idle behind its diagonal tiles.
// Grid: the finish workgroups of all clusters first (n_finish per cluster), then the bulk ones.
__global__ __launch_bounds__(256) void k_potrf_update(const ClusterInfo* __restrict__ cl, const float* __restrict__ Kd,
                                                      float* __restrict__ Lf, float* __restrict__ G, int k,
                                                      int n_finish, int n_bulk, int grid_finish, int nc,
                                                      PcgState* __restrict__ st) {
  // the operand stages and, once the products are done, the tile being factored share one piece of LDS
  // (34 KB per workgroup with the inverse: four workgroups per compute unit instead of three)
  static_assert(2 * TILE * SP >= TILE * (TILE + 1), "the factored tile must fit in the operand stages");
  __shared__ __attribute__((aligned(16))) float stage[2 * TILE * SP];
  __shared__ float sI[TILE][TILE + 1];
  float (*sA)[SP] = reinterpret_cast<float (*)[SP]>(stage);
  float (*sB)[SP] = reinterpret_cast<float (*)[SP]>(stage + TILE * SP);
  float (*sT)[TILE + 1] = reinterpret_cast<float (*)[TILE + 1]>(stage);
  const bool bulk = (int)blockIdx.x >= grid_finish;
  int ci, item;
  if (!die_local_item(bulk ? n_bulk : n_finish, nc, ci, item, bulk ? (int)blockIdx.x - grid_finish : (int)blockIdx.x)) return;
  const ClusterInfo c = cl[ci];
  const int col = bulk ? k + 1 : k;            // tile column this workgroup works on
  const int mt = col + item;
  if (mt >= (int)c.nt) return;
  const int tid = threadIdx.x;
  const int b = (int)c.b;
  const float* A = Kd + c.koff;
  float* L = Lf + c.koff;
  v4f acc[2][2];
  zero_acc(acc);
  Operand oa{L, c.ld, mt * TILE, b, 0};
  Operand ob{L, c.ld, col * TILE, b, 0};
  if (bulk) tile_gemm<false, false>(acc, oa, ob, 0, k * TILE, sA, sB, tid);
  else if (k > 0) tile_gemm<false, false>(acc, oa, ob, (k - 1) * TILE, k * TILE, sA, sB, tid);
  // what the products are subtracted from: the assembled block, or the bulk result of the step before
  const float* base = (bulk || k == 0) ? A : L;
  if (bulk || mt != k) {
    for_each_acc(acc, tid, [&](int r, int q, float v) {
      const uint64_t at = blocked_index(c.ld, mt * TILE + r, col * TILE + q);
      L[at] = base[at] - v;
    });
    return;
  }
  // ---- diagonal tile: factor in LDS; rows/cols past the cluster end behave as identity ----
  __syncthreads();                              // every wave is done reading the operand stages
  const int valid = min(TILE, b - k * TILE);
  for_each_acc(acc, tid, [&](int r, int q, float v) {
    float x = base[blocked_index(c.ld, k * TILE + r, k * TILE + q)] - v;
    if (r >= valid || q >= valid) x = (r == q) ? 1.f : 0.f;
    sT[r][q] = x;
  });
  __syncthreads();
  // Right-looking elimination with ONE barrier per pivot: column j is left unscaled (its entries are read as
  // a_ij a_cj / d_j by the update) and the division by sqrt(d_j) is applied to all columns in a pass at the
  // end; d_j = sT[j][j] is final once pivot j - 1 has been processed and is not touched afterwards.
  bool bad = false;
  for (int j = 0; j < TILE - 1; ++j) {
    float dj = sT[j][j];
    if (!(dj > 0.f) || !(dj < INFINITY)) { bad = true; dj = 1.f; }
    const float rd = 1.f / dj;
    const int i = tid >> 2;                // trailing update, row i, columns j < cc <= i
    if (i > j) {
      const float lij = sT[i][j] * rd;
      for (int cc = j + 1 + (tid & 3); cc <= i; cc += 4) sT[i][cc] = fmaf(-lij, sT[cc][j], sT[i][cc]);
    }
    __syncthreads();
  }
  {
    const float dl = sT[TILE - 1][TILE - 1];
    if (!(dl > 0.f) || !(dl < INFINITY)) bad = true;
  }
  __syncthreads();
  // scaling pass: L_ij = a_ij / sqrt(d_j), L_jj = sqrt(d_j) (non-positive pivots behave as 1, as above);
  // the diagonal is read before anything is written
  {
    const int i = tid >> 2;
    float col[TILE / 4];
#pragma unroll
    for (int u = 0; u < TILE / 4; ++u) {
      const int j = 4 * u + (tid & 3);
      float dj = sT[j][j];
      if (!(dj > 0.f) || !(dj < INFINITY)) dj = 1.f;
      const float sj = sqrtf(dj);
      col[u] = j < i ? sT[i][j] / sj : (j == i ? sj : 0.f);
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < TILE / 4; ++u) {
      const int j = 4 * u + (tid & 3);
      if (j <= i) sT[i][j] = col[u];
    }
  }
  __syncthreads();
  if (bad && tid == 0) atomicMin(&st->bad_cluster, ci);
  // ---- inverse of the lower-triangular tile: column cc by forward substitution, four lanes per column
  // sharing each row's sum (lanes 4 cc .. 4 cc + 3 sit in one wave) ----
  {
    const int cc = tid >> 2, part = tid & 3;
    if (part == 0) {
      for (int i = 0; i < cc; ++i) sI[i][cc] = 0.f;
      sI[cc][cc] = 1.f / sT[cc][cc];
    }
    for (int i = cc + 1; i < TILE; ++i) {
      // the four lanes of a column run the same iterations, so the shuffles stay inside active lanes; the
      // column's earlier entries were written by this wave, whose LDS accesses are served in order
      float sacc = 0.f;
      for (int j = cc + part; j < i; j += 4) sacc = fmaf(sT[i][j], sI[j][cc], sacc);
      sacc += __shfl_xor(sacc, 1);
      sacc += __shfl_xor(sacc, 2);
      if (part == 0) sI[i][cc] = -sacc / sT[i][i];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  }
  __syncthreads();
  float* Y = G + c.koff;
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;
    const uint64_t at = blocked_index(c.ld, k * TILE + r, k * TILE + q);
    L[at] = (q <= r) ? sT[r][q] : 0.f;
    Y[at] = (q <= r) ? sI[r][q] : 0.f;
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
  for_each_acc(acc, tid, [&](int r, int q, float v) { L[blocked_index(c.ld, mt * TILE + r, k * TILE + q)] = v; });
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

  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int q = idx >> 6, r = idx & 63;
    Y[blocked_index(c.ld, tn * TILE + q, tm * TILE + r)] = sT[r][q];
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
  for_each_acc(acc, tid, [&](int r, int q, float v) { Y[blocked_index(c.ld, tm * TILE + r, tn * TILE + q)] = -v; });
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

  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;
    sT[r][q] = Y[blocked_index(c.ld, tr * TILE + r, tc * TILE + q)];
  }
  __syncthreads();
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;      // element (r, q) of the destination tile
    if (tr != tc || q > r) Y[blocked_index(c.ld, tc * TILE + r, tr * TILE + q)] = sT[q][r];
  }
}

// upper tiles of one square blocked matrix of nt x nt tiles <- transposes of the lower ones (1-D grid of nt * nt)
__global__ __launch_bounds__(256) void k_mirror_square(float* __restrict__ M, uint32_t ld, int nt) {
  __shared__ float sT[TILE][TILE + 1];
  const int tr = (int)(blockIdx.x / (unsigned)nt), tc = (int)(blockIdx.x % (unsigned)nt);
  if (tc >= tr) return;
  const int tid = threadIdx.x;
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;
    sT[r][q] = M[blocked_index(ld, tr * TILE + r, tc * TILE + q)];
  }
  __syncthreads();
  for (int idx = tid; idx < TILE * TILE; idx += 256) {
    const int r = idx >> 6, q = idx & 63;
    M[blocked_index(ld, tc * TILE + r, tr * TILE + q)] = sT[q][r];
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

int launch_factor(nugpr_ctx* c, hipStream_t s) {
  const Layout& L = c->L;
  // clusters of similar size: one die per cluster; otherwise every cluster over all dies (see die_local_item)
  uint64_t tiles_sum = 0;
  for (const ClusterInfo& ci : L.cl) tiles_sum += ci.nt;
  const bool even = (uint64_t)L.ntmax * (uint64_t)L.nc * 4 <= tiles_sum * 5;
  const int ncm = even ? L.nc : -L.nc;
  c->Lf = c->Kd2;                 // the factor goes into the spare blocks (see nugpr_ctx::lf_valid)
  c->lf_valid = true;
  hipLaunchKernelGGL(k_reset_bad, dim3(1), dim3(1), 0, s, c->d_state);
  for (int k = 0; k < L.ntmax; ++k) {
    const int n_finish = L.ntmax - k, n_bulk = L.ntmax - k - 1;
    const unsigned grid_finish = die_grid(n_finish, ncm), grid_bulk = n_bulk > 0 ? die_grid(n_bulk, ncm) : 0u;
    hipLaunchKernelGGL(k_potrf_update, dim3(grid_finish + grid_bulk), dim3(256), 0, s, c->d_cl, c->Kd, c->Lf, c->G, k,
                       n_finish, n_bulk, (int)grid_finish, ncm, c->d_state);
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
