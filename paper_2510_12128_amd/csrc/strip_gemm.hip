// Strip GEMM: the product of a stored fp32 matrix strip (64 rows,
// any number of columns) with a tall-skinny vector block of T <= 33 columns.
//
// Every matrix of the hot path is applied through this one kernel:
//   K_ii D_i, C S (coupling), W_i^T D_i, W_i P_i        -- the block-low-rank product
//                                                          K' D of eq. (odsplit), Section 3.3
//   tril(L_i^-1) R_i, triu(L_i^-T) V_i                   -- the block-Jacobi preconditioner,
//                                                          applied as explicit inverses (Table 2)
//   tril(L_i) Z_i                                        -- probe right-hand sides
//
// Two kernels share the tiling and the arithmetic and differ in how the matrix reaches the
// matrix cores:
//   k_strip       the fp32 mode and single-column products: every wave loads its own matrix
//                 rows into registers (described next);
//   k_strip_ring  the fp64 mode with two or more columns, i.e. every launch of the training
//                 path: a fifth wave streams matrix tiles and vector slabs into an LDS ring
//                 with LDS-direct loads while four waves consume them, and the tiles of a
//                 symmetric block are read once for the two strips they serve (its own
//                 description stands in front of it, further down).
//
// Common design (gfx950, wave64): a workgroup owns a strip of 64 matrix rows, each of four
// consumer waves 16 of them, and walks along the rows in chunks of 64 columns with 16-byte
// loads, for all T columns at once.  Lane (m, kg) of a wave holds float4
// A[row m][c + 16 s + 4 kg ..]; the four components feed four 16x16x4 MFMAs, whose
// contraction index is the kg of the lane, so the column permutation inside a 16-column
// group is absorbed by reading the matching rows of the vector block from LDS (stored as
// 4-vectors over 4 consecutive rows).  Columns 1..T-1 (the probes) go through the matrix
// cores in groups of 16; column 0 (y) rides on the vector ALUs from the same registers, so
// T = 17 costs one MFMA group, not two.
// k_strip: the vector block chunk is double-buffered in LDS; the matrix chunk lives in ONE
// register set: slot s is reloaded with the next chunk's data right after it has been
// consumed, so each load has a full chunk period to land while few registers are live, and
// occupancy hides the rest of the HBM latency.
//
// Two arithmetic modes, same data movement:
//   ACC64 = true   vector blocks are fp64; the fp32 matrix entries are widened in
//                  registers and contracted with v_mfma_f64_16x16x4_f64: products and
//                  sums carry no fp32 rounding at all.
//   ACC64 = false  vector blocks are fp32; v_mfma_f32_16x16x4_f32 in four short
//                  independent chains per column group that are folded into fp64 sums
//                  after every chunk.
// The CG coefficients and the SLQ estimate are Rayleigh quotients of these products
// scaled by n, so rounding in the running sums enters the loss at first order; the fp64
// mode removes it, the fp32 mode keeps it near sqrt(b) * 1e-7 per output entry.
#include <algorithm>
#include <type_traits>

#include "nugpr_internal.h"

namespace nugpr {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

template <bool ACC64> struct VecT { typedef float type; };
template <> struct VecT<true> { typedef double type; };

struct alignas(32) Quad64 { double x, y, z, w; };
struct alignas(16) Quad32 { float x, y, z, w; };

// row of the 16x16 accumulator tile held in component i of lane `lane`:
// f32 16x16x4 keeps rows 4*(lane/16) + i, f64 16x16x4 keeps rows (lane/16) + 4*i
template <bool ACC64>
__device__ __forceinline__ int acc_row(int lane, int i) {
  return ACC64 ? (lane >> 4) + 4 * i : 4 * (lane >> 4) + i;
}

constexpr int CHUNK = 64;              // columns per pipeline stage
constexpr int NL = CHUNK / 16;         // float4 loads per lane per chunk
constexpr int NPRE = 1;                // register sets of matrix chunks in flight per wave (1 or 2)

// At least two waves per SIMD: with at most 256 registers a wave the compiler keeps the MFMA
// accumulators in ordinary vector registers instead of copying them in and out of the
// accumulation registers around every chunk.
template <int NG, bool ACC64>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_strip(const StripArgs a) {
  typedef typename VecT<ACC64>::type VT;
  typedef typename std::conditional<ACC64, Quad64, Quad32>::type QuadT;
  constexpr int NCOLM = NG > 0 ? 16 * NG : 1;    // columns handled by the matrix cores
  constexpr int NE = (CHUNK * (16 * NG + 1) + 255) / 256;   // staged vector elements per thread
  constexpr int NGA = NG > 0 ? NG : 1;
  __shared__ QuadT sB[2][(CHUNK / 4) * NCOLM];
  __shared__ QuadT sY[2][CHUNK / 4];

  const StripItem it = a.items[blockIdx.x];
  const StripPort& pt = a.port[it.port];
  const VT* __restrict__ vin = static_cast<const VT*>(pt.in);
  const int T = a.T;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int m = lane & 15, kg = lane >> 4;
  const int nrows = (int)it.nrows;
  const int lr = wave * 16 + m;                               // local row this lane loads
  const int lrc = lr < nrows ? lr : nrows - 1;
  // this lane's four matrix elements of 16-column step s of the chunk that starts at column cc
  // (row-major, or 64 x 32 blocks: see blocked_index; cc is a multiple of 64)
  const float* __restrict__ Arow = pt.A + it.a_off + (uint64_t)lrc * (uint64_t)it.lda + 4 * kg;
  // blocked: fragment (row group, s % 2) of block cc / 32 + s / 2, row lrc % 16, columns 4 kg ..
  const float* __restrict__ Ablk = pt.A + it.a_off + (uint64_t)((lrc >> 4) * 2) * FRAG + (lrc & 15) * 16 + 4 * kg;
  const bool blocked = it.blocked != 0;
  auto Aaddr = [&](const int cc, const int s) -> const float* {
    return blocked ? Ablk + (uint64_t)((cc >> 5) + (s >> 1)) * (TILE * BLK_COLS) + (s & 1) * FRAG : Arow + cc + 16 * s;
  };
  const int c_begin = (int)it.c_begin, c_end = (int)it.c_end;
  const int nchunks = c_end > c_begin ? (c_end - c_begin + CHUNK - 1) / CHUNK : 0;
  // columns this lane's row keeps: [q_lo, q_hi)
  const int diag = (int)it.row_in_block + lr;
  const int q_lo = it.mode == 2 ? diag : c_begin;
  const int q_hi = it.mode == 1 ? (diag + 1 < c_end ? diag + 1 : c_end) : c_end;
  // chunks that may hold dropped elements: the last one, and the one with the diagonal tile
  const int mask_from = it.mode == 1 ? (int)it.row_in_block : c_end - (c_end - c_begin) % CHUNK;
  const int mask_upto = it.mode == 2 ? (int)it.row_in_block + TILE : c_begin;

  // zero the LDS once: the padding columns of the MFMA operand are never written again
  {
    VT* z = reinterpret_cast<VT*>(&sB[0][0]);
    for (int i = tid; i < 2 * CHUNK * NCOLM; i += 256) z[i] = (VT)0;
  }
  __syncthreads();

  v4f acc32[NGA][4];       // fp32 mode: four chains per group, restarted every chunk
  v4d acc64[NGA][2];       // fp64 mode: two chains per group (hides the MFMA issue latency)
  double dacc[NGA][4];     // fp32 mode: fp64 running sums
  float accy32[4] = {0.f, 0.f, 0.f, 0.f};
  double daccy = 0.0;
#pragma unroll
  for (int g = 0; g < NGA; ++g) {
#pragma unroll
    for (int j = 0; j < 4; ++j) { acc32[g][j] = (v4f){0.f, 0.f, 0.f, 0.f}; dacc[g][j] = 0.0; }
    acc64[g][0] = (v4d){0.0, 0.0, 0.0, 0.0};
    acc64[g][1] = (v4d){0.0, 0.0, 0.0, 0.0};
  }

  // staging: thread `tid` moves flat elements e = tid + 256 k of the chunk's contiguous
  // (CHUNK x T) slab; rows past the item's last column are staged as zero
  const int nelem = CHUNK * T;
  auto load_in = [&](int c, VT (&reg)[NE]) {
    const VT* __restrict__ src = vin + (uint64_t)(it.in_row0 + (uint32_t)c) * (uint64_t)T;
    const int lim = min(nelem, (c_end - c) * T);       // >= T: chunk c starts before c_end
    // every lane loads (from a clamped address) so the loads sit in straight-line code and
    // the outstanding-load counter stays exact; lanes past the slab keep a zero instead
#pragma unroll
    for (int k = 0; k < NE; ++k) {
      const int e = tid + 256 * k;
      const VT v = src[e < lim ? e : lim - 1];
      reg[k] = e < lim ? v : (VT)0;
    }
  };
  auto store_in = [&](int buf, const VT (&reg)[NE]) {
#pragma unroll
    for (int k = 0; k < NE; ++k) {
      const int e = tid + 256 * k;
      if (e < nelem) {
        const int q = (T == 1) ? e : (int)__umulhi((uint32_t)e, a.magicT);
        const int col = e - q * T;
        if (col == 0) reinterpret_cast<VT*>(&sY[buf][q >> 2])[q & 3] = reg[k];
        else if (NG > 0) reinterpret_cast<VT*>(&sB[buf][(q >> 2) * NCOLM + (col - 1)])[q & 3] = reg[k];
      }
    }
  };

  // one 16-column step: 4 MFMAs per column group + the y column on the vector ALUs.
  // `slot` is the register the 16 columns came from; it is reloaded from `next` as soon as its
  // value has been consumed (widened in the fp64 mode, issued to the matrix cores in the
  // fp32 mode).  The scheduling barriers keep the compiler from moving the reload ahead of
  // that point, where it would need a second register set and a drain at the loop's end.
  auto step = [&](float4& slot, const float* __restrict__ next, const bool masked, const int q0, int buf, int s) {
    float4 av = slot;
    if (masked) {
      av.x = (q0 + 0 >= q_lo && q0 + 0 < q_hi) ? av.x : 0.f;
      av.y = (q0 + 1 >= q_lo && q0 + 1 < q_hi) ? av.y : 0.f;
      av.z = (q0 + 2 >= q_lo && q0 + 2 < q_hi) ? av.z : 0.f;
      av.w = (q0 + 3 >= q_lo && q0 + 3 < q_hi) ? av.w : 0.f;
    }
    if constexpr (ACC64) {
      const double ax = (double)av.x, ay = (double)av.y, az = (double)av.z, aw = (double)av.w;
      // empty statement that ties the reload's address to the widened values: the reload
      // cannot be issued before the old contents of the slot have been consumed
      int dep = 0;
      asm volatile("" : "+v"(dep) : "v"(ax), "v"(ay), "v"(az), "v"(aw));
      slot = *reinterpret_cast<const float4*>(next + dep);
      if (NG > 0) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const Quad64 bv = sB[buf][(4 * s + kg) * NCOLM + 16 * g + m];
          acc64[g][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(ax, bv.x, acc64[g][0], 0, 0, 0);
          acc64[g][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(ay, bv.y, acc64[g][1], 0, 0, 0);
          acc64[g][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(az, bv.z, acc64[g][0], 0, 0, 0);
          acc64[g][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(aw, bv.w, acc64[g][1], 0, 0, 0);
        }
      }
      const Quad64 yv = sY[buf][4 * s + kg];
      daccy = fma(ax, yv.x, daccy);
      daccy = fma(ay, yv.y, daccy);
      daccy = fma(az, yv.z, daccy);
      daccy = fma(aw, yv.w, daccy);
    } else {
      if (NG > 0) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const Quad32 bv = sB[buf][(4 * s + kg) * NCOLM + 16 * g + m];
          acc32[g][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.x, acc32[g][0], 0, 0, 0);
          acc32[g][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bv.y, acc32[g][1], 0, 0, 0);
          acc32[g][2] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, bv.z, acc32[g][2], 0, 0, 0);
          acc32[g][3] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, bv.w, acc32[g][3], 0, 0, 0);
        }
      }
      const Quad32 yv = sY[buf][4 * s + kg];
      accy32[0] = fmaf(av.x, yv.x, accy32[0]);
      accy32[1] = fmaf(av.y, yv.y, accy32[1]);
      accy32[2] = fmaf(av.z, yv.z, accy32[2]);
      accy32[3] = fmaf(av.w, yv.w, accy32[3]);
      __builtin_amdgcn_sched_barrier(0);
      slot = *reinterpret_cast<const float4*>(next);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // NPRE register sets hold the matrix chunks in flight: set (ch % NPRE) carries chunk ch
  // and slot s of it is reloaded with chunk ch + NPRE right after it has been read, so
  // the loads of NPRE chunks are outstanding while the matrix cores work on one.
  float4 areg[NPRE][NL];
  VT inreg[NE];
  const int c_last = c_begin + (nchunks - 1) * CHUNK;    // chunks past the end re-read the last one
  if (nchunks > 0) {
#pragma unroll
    for (int p = 0; p < NPRE; ++p) {
      const int cp = min(c_begin + p * CHUNK, c_last);
#pragma unroll
      for (int s = 0; s < NL; ++s) areg[p][s] = *reinterpret_cast<const float4*>(Aaddr(cp, s));
    }
    load_in(c_begin, inreg);
    store_in(0, inreg);
  }
  __syncthreads();

  auto chunk = [&](auto set_c, const int ch) {
    constexpr int SET = decltype(set_c)::value;
    const int buf = ch & 1;
    const int c = c_begin + ch * CHUNK;
    load_in(min(c + CHUNK, c_last), inreg);
    const int cn = min(c + NPRE * CHUNK, c_last);
    // chunk with elements outside the item's column range or on the wrong side of the diagonal
    const bool masked = (c >= mask_from || c < mask_upto);
#pragma unroll
    for (int s = 0; s < NL; ++s) step(areg[SET][s], Aaddr(cn, s), masked, c + 16 * s + 4 * kg, buf, s);
    if constexpr (!ACC64) {
      // fold this chunk's short chains into the fp64 sums and restart them
      if (NG > 0) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            dacc[g][i] += ((double)acc32[g][0][i] + (double)acc32[g][1][i]) +
                          ((double)acc32[g][2][i] + (double)acc32[g][3][i]);
#pragma unroll
          for (int j = 0; j < 4; ++j) acc32[g][j] = (v4f){0.f, 0.f, 0.f, 0.f};
        }
      }
      daccy += ((double)accy32[0] + (double)accy32[1]) + ((double)accy32[2] + (double)accy32[3]);
      accy32[0] = accy32[1] = accy32[2] = accy32[3] = 0.f;
    }
    store_in(buf ^ 1, inreg);
    __syncthreads();
  };
  if constexpr (NPRE == 1) {
    for (int ch = 0; ch < nchunks; ++ch) chunk(std::integral_constant<int, 0>(), ch);
  } else {
    static_assert(NPRE <= 2, "the chunk loop is unrolled by the number of register sets");
    // An odd chunk count is rounded up: the extra chunk starts at or past c_end, so it is a
    // masked chunk whose every element is dropped (it re-reads the last chunk's data).
    for (int ch = 0; ch < nchunks; ch += 2) {
      chunk(std::integral_constant<int, 0>(), ch);
      chunk(std::integral_constant<int, NPRE - 1>(), ch + 1);
    }
  }

  // ---- epilogue ----
  VT* __restrict__ out = static_cast<VT*>(pt.out) + (uint64_t)it.out_part * pt.out_part_stride;
  const double dadd = (double)it.diag_add * pt.diag_add;   // diagonal shift (incl. the part of the diagonal fp32 cannot hold)
  const bool add_diag = (dadd != 0.0);
  const double scale = pt.scale;
  if (NG > 0) {
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int col = 1 + 16 * g + m;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = wave * 16 + acc_row<ACC64>(lane, i);
        if (row < nrows && col < T) {
          double v = scale * (ACC64 ? (acc64[g][0][i] + acc64[g][1][i]) : dacc[g][i]);
          if (add_diag) v = fma(dadd, (double)vin[(uint64_t)(it.in_row0 + it.row_in_block + row) * T + col], v);
          const uint64_t idx = (uint64_t)(it.out_row0 + row) * T + col;
          if (pt.accumulate) v += (double)out[idx];
          out[idx] = (VT)v;
        }
      }
    }
  }
  daccy += __shfl_xor(daccy, 16);
  daccy += __shfl_xor(daccy, 32);
  if (kg == 0 && lr < nrows) {
    double v = scale * daccy;
    if (add_diag) v = fma(dadd, (double)vin[(uint64_t)(it.in_row0 + it.row_in_block + lr) * T], v);
    const uint64_t idx = (uint64_t)(it.out_row0 + lr) * T;
    if (pt.accumulate) v += (double)out[idx];
    out[idx] = (VT)v;
  }
}

// ---------------------------------------------------------------------------
// fp64 mode with T >= 2: producer / consumer version of the kernel above.
//
// A workgroup has FIVE waves.  Wave 4 only moves data: for every 64-column chunk it issues
// LDS-direct loads (global_load_lds_dwordx4: memory -> LDS, no registers) of the 64 x 64 matrix
// tile -- in exactly the per-lane order the consumers read it back, one 16-byte slot per lane
// and step -- and of the chunk's contiguous (64 x T) slab of the vector block, into a ring of
// STAGES buffers.  Waves 0..3 never touch global memory inside the loop: they read their
// slots and the vector rows from LDS and run the same arithmetic as k_strip.  One workgroup
// barrier per chunk hands a filled stage to the consumers and a drained one back to the
// loader, which keeps STAGES - 1 chunks (about 50 KB per workgroup) in flight however long
// the matrix cores are busy: the loads no longer wait for the wave that will use them.
// Chunks with dropped elements (ragged end, diagonal tile) zero the matrix entries AND
// the vector rows past the item's last column, so whatever follows a short slab in
// memory never reaches the sums.
// ---------------------------------------------------------------------------
constexpr uint32_t waitcnt_vm(uint32_t n) {      // s_waitcnt immediate: vmcnt(n), the other counters unconstrained
  return (n & 15u) | ((n >> 4) << 14) | 0x0F70u;
}

template <int NG, int RCH, int STAGES_>
struct RingCfg {
  static constexpr int NCOLM = 16 * NG;
  static constexpr int NSLAB = (RCH * (NCOLM + 1) * 8 + 1023) / 1024;      // 1 KiB loads covering a slab of fp64
  static constexpr int STAGES = STAGES_;
  static constexpr int NSTEP = RCH / 16;                                   // 16-column steps per chunk
  static constexpr int A_BYTES = RCH * 64 * 4;                             // 64 rows x RCH columns of fp32
  static constexpr int STAGE_BYTES = A_BYTES + NSLAB * 1024;
  static constexpr int LOADS = 4 * NSTEP + NSLAB;                                 // loader instructions per chunk
  static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + 512;             // + slack for reads of unused columns
};

// TC: the number of columns T when it is known at compile time (the usual widths: 16 or 32 probes + y), else
// 0.  With T a constant the LDS addresses of the vector rows a lane reads in a chunk differ from one base by
// constants that fit the instructions' offset fields; with T at run time they cost some thirty vector
// instructions per chunk, on a pipe that the matrix instructions already keep busy half of the time.
template <int NG, int RCH, int STAGES_, bool SYM, int TC>
__global__ __launch_bounds__(320) __attribute__((amdgpu_waves_per_eu(2))) void k_strip_ring(const StripArgs a) {
#if __HIP_DEVICE_COMPILE__
  typedef RingCfg<NG, RCH, STAGES_> Cfg;
  constexpr int NSTEP = Cfg::NSTEP;
  constexpr int STAGES = Cfg::STAGES;
  extern __shared__ __attribute__((aligned(16))) unsigned char ring[];

  const StripItem it = a.items[blockIdx.x];
  const StripPort& pt = a.port[it.port];
  const double* __restrict__ vin = static_cast<const double*>(pt.in);
  const int T = TC > 0 ? TC : a.T;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int m = lane & 15, kg = lane >> 4;
  const int nrows = (int)it.nrows;
  const int c_begin = (int)it.c_begin, c_end = (int)it.c_end;
  // Strips of a symmetric matrix (StripItem::blocked bit 1).  The item's columns are the tiles tb .. tb + nb - 1
  // of a square super-block whose rows are a group of `na` strips; the item is strip number jr of that group.
  // It visits its tiles in the rotating order p = (t - jr) mod max(na, nb), t = 0, 1, ..  A super-block on the
  // diagonal of the matrix (kind 0: a cluster's K_ii, or a diagonal block of C) takes tile p from the strip's
  // own rows when p <= jr and as the TRANSPOSE of the stored tile (tb + p, strip) when p > jr; one below the
  // diagonal (kind 1) always reads its own rows, one above it (kind 2) always the transposed tiles of its
  // mirror image.  The partner strip visits the same stored tile at the same step t, the two workgroups are
  // dealt to the same die and start together, so the two requests for the same 16 KiB meet in that die's L2
  // and HBM serves one: the lower triangle is streamed, the upper one never leaves memory.  Steps whose
  // tile lies past the item's last one (groups of unequal size) load a valid tile and drop it whole.
  const uint32_t fl = it.blocked;
  const bool sym = SYM && (fl & 2u) != 0;
  const int kind = (int)((fl >> 2) & 3u);
  const int j_abs = (int)(it.row_in_block >> 6);                      // the strip's index inside the matrix
  const int tb = c_begin >> 6, nb = (c_end - c_begin + TILE - 1) >> 6;
  const int na = (int)((fl >> 4) & 0x7ffu);                           // 0: the group is the item's own tile range
  const int jr = na ? (int)((fl >> 15) & 0x7ffu) : j_abs - tb;
  const int mrot = na > nb ? na : nb;
  const int nchunks = sym ? 2 * mrot : (c_end > c_begin ? (c_end - c_begin + RCH - 1) / RCH : 0);
  // chunk ch: c = first column of the product it covers (c_end: none, the chunk is dropped), c_addr = first
  // column of the tile that is loaded, p = that tile's number in the item; returns whether it is transposed
  auto locate = [&](const int ch, int& c, int& c_addr, int& p) {
    if (!sym) { c = c_addr = c_begin + ch * RCH; p = 0; return false; }
    p = (ch >> 1) - jr;
    p += p < 0 ? mrot : 0;
    const bool valid = p < nb;
    p = valid ? p : nb - 1;
    c_addr = c_begin + TILE * p + RCH * (ch & 1);
    c = valid ? c_addr : c_end;
    return kind == 2 || (kind == 0 && p > jr);
  };

  if (wave == 4) {
    // ---- loader ----
    // matrix: for consumer wave w and step s, lane (m, kg) fetches A[16 w + m][c + 16 s + 4 kg .. + 3]
    // (rows past the strip's last one re-read it; the padded leading dimension keeps the columns in bounds)
    // (blocked storage: a chunk of RCH = 32 columns is one block, and the operand of (w, s) one 1 KiB
    // fragment of it: float4 number 4 m + kg)
    static_assert(RCH == BLK_COLS, "the ring kernel reads one storage block per chunk");
    const bool blocked = it.blocked != 0;
    const float* __restrict__ Ab = pt.A + it.a_off + 4 * kg;
    const uint64_t cmul = blocked ? (uint64_t)TILE : 1u;        // a block of 32 columns starts 64 * 32 floats after the last
    const int smul = blocked ? FRAG : 16;                      // step s of a chunk: the next fragment / 16 columns on
    uint64_t rowoff[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int rw = min(16 * w + m, nrows - 1);
      rowoff[w] = blocked ? (uint64_t)((rw >> 4) * 2) * FRAG + (uint64_t)(rw & 15) * 16 : (uint64_t)rw * (uint64_t)it.lda;
    }
    const unsigned char* __restrict__ vbytes = reinterpret_cast<const unsigned char*>(vin);
    // transposed tiles: the operand of (w, s) is fragment (2 half + s, w % 2) of column block 2 j_abs + w / 2
    // of strip tb + p, whole (every fragment of the padded block exists); lane l fetches the piece (row
    // 4 ((l / 4) % 4) + l / 16, columns 4 (l % 4) .. + 3), which puts element (4 kg + i, m) of the fragment
    // at float 64 i + 16 kg + m: the consumers read their four values with unit stride across the wave
    const float* __restrict__ At = pt.A + it.a_off + (uint64_t)(2 * j_abs) * (TILE * BLK_COLS) +
                                   (((lane >> 2) & 3) * 4 + (lane >> 4)) * 16 + (lane & 3) * 4;
    auto issue = [&](const int ch) {
      int c, c_addr, p;
      const bool tr = locate(ch, c, c_addr, p);
      unsigned char* st = ring + (ch % STAGES) * Cfg::STAGE_BYTES;
      if (SYM && tr) {
        const float* __restrict__ Ap = At + (uint64_t)(tb + p - j_abs) * TILE * (uint64_t)it.lda + (ch & 1) * (4 * FRAG);
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
          for (int s = 0; s < NSTEP; ++s)
            __builtin_amdgcn_global_load_lds(Ap + (w >> 1) * (TILE * BLK_COLS) + (2 * s + (w & 1)) * FRAG,
                                             st + (w * NSTEP + s) * 1024, 16, 0, 0);
      } else {
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
          for (int s = 0; s < NSTEP; ++s)
            __builtin_amdgcn_global_load_lds(Ab + rowoff[w] + (uint64_t)c_addr * cmul + s * smul, st + (w * NSTEP + s) * 1024, 16, 0, 0);
      }
      // vector slab: rows in_row0 + c .., T columns, contiguous; 16-byte pieces past its last valid byte
      // re-read the last valid piece (the consumers drop those rows).  A chunk that lies wholly past the
      // last column (second half of a ragged last tile) reads the last row instead and is dropped whole.
      const int c_slab = min(c, c_end - 1);
      const uint64_t slab0 = (uint64_t)(it.in_row0 + (uint32_t)c_slab) * (uint64_t)T * 8u;
      const int valid = min(RCH, c_end - c_slab) * T * 8;               // > 0
      const int last_piece = ((valid - 1) >> 4) << 4;
#pragma unroll
      for (int i = 0; i < Cfg::NSLAB; ++i) {
        const int off = min((i * 64 + lane) * 16, last_piece);
        __builtin_amdgcn_global_load_lds(vbytes + slab0 + off, st + Cfg::A_BYTES + i * 1024, 16, 0, 0);
      }
    };
    for (int p = 0; p < STAGES - 1; ++p)
      if (p < nchunks) issue(p);
    for (int ch = 0; ch < nchunks; ++ch) {
      // chunk ch must have landed; the chunks issued after it may still be in flight.  Near the end fewer
      // chunks follow, so everything is waited for.
      if (STAGES > 2 && ch + STAGES - 2 <= nchunks - 1) __builtin_amdgcn_s_waitcnt(waitcnt_vm((STAGES - 2) * Cfg::LOADS));
      else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
      __builtin_amdgcn_s_barrier();
      // the consumers are done with chunk ch - 1: its stage takes chunk ch + STAGES - 1
      if (ch + STAGES - 1 < nchunks) issue(ch + STAGES - 1);
    }
    return;
  }

  // ---- consumers ----
  const int lr = wave * 16 + m;                               // local row of this lane's matrix slots
  const int diag = (int)it.row_in_block + lr;
  const int q_lo = it.mode == 2 ? diag : c_begin;
  const int q_hi = it.mode == 1 ? (diag + 1 < c_end ? diag + 1 : c_end) : c_end;
  const int rib = (int)it.row_in_block;

  v4d acc64[NG][2];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    acc64[g][0] = (v4d){0.0, 0.0, 0.0, 0.0};
    acc64[g][1] = (v4d){0.0, 0.0, 0.0, 0.0};
  }
  double daccy = 0.0;

  for (int ch = 0; ch < nchunks; ++ch) {
    int c, c_addr, p_tile;
    const bool tr = locate(ch, c, c_addr, p_tile);
    __builtin_amdgcn_s_barrier();                             // chunk ch is in its stage
    const unsigned char* st = ring + (ch % STAGES) * Cfg::STAGE_BYTES;
    const float4* __restrict__ sAw = reinterpret_cast<const float4*>(st) + wave * (64 * NSTEP) + lane;
    const float* __restrict__ sAt = reinterpret_cast<const float*>(st) + wave * (256 * NSTEP) + lane;
    const double* __restrict__ sV = reinterpret_cast<const double*>(st + Cfg::A_BYTES);
    // chunks that can hold dropped elements: past the last column, or touching the diagonal tile
    const bool masked = c + RCH > c_end || (it.mode == 1 && c + RCH > rib) || (it.mode == 2 && c < rib + TILE);
    const int kvalid = c_end - c;                             // vector rows of this chunk that exist
#pragma unroll
    for (int s = 0; s < NSTEP; ++s) {
      // the operand: float4 number `lane` of the (wave, s) fragment, or, for a transposed tile, four floats 64 apart
      // (the 16-byte read goes through a volatile pointer into LDS: otherwise the compiler merges the two
      // branches into four 4-byte reads at selected addresses, for both kinds of tile)
      float4 av;
      if (SYM && tr) {
        av = make_float4(sAt[s * 256], sAt[s * 256 + 64], sAt[s * 256 + 128], sAt[s * 256 + 192]);
      } else {
        typedef __attribute__((address_space(3))) const volatile v4f* lds_v4f;
        const v4f q = *(lds_v4f)(sAw + s * 64);
        av = make_float4(q[0], q[1], q[2], q[3]);
      }
      const int k0 = 16 * s + 4 * kg;                         // chunk-local column of av.x
      const double* __restrict__ vr = sV + k0 * T;
      double y[4], b[NG][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        y[j] = vr[j * T];
#pragma unroll
        for (int g = 0; g < NG; ++g) b[g][j] = vr[j * T + 1 + 16 * g + m];
      }
      if (masked) {
        const int q0 = c + k0;
        av.x = (q0 + 0 >= q_lo && q0 + 0 < q_hi) ? av.x : 0.f;
        av.y = (q0 + 1 >= q_lo && q0 + 1 < q_hi) ? av.y : 0.f;
        av.z = (q0 + 2 >= q_lo && q0 + 2 < q_hi) ? av.z : 0.f;
        av.w = (q0 + 3 >= q_lo && q0 + 3 < q_hi) ? av.w : 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = k0 + j < kvalid;
          y[j] = ok ? y[j] : 0.0;
#pragma unroll
          for (int g = 0; g < NG; ++g) b[g][j] = ok ? b[g][j] : 0.0;
        }
      }
      const double ax = (double)av.x, ay = (double)av.y, az = (double)av.z, aw = (double)av.w;
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        acc64[g][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(ax, b[g][0], acc64[g][0], 0, 0, 0);
        acc64[g][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(ay, b[g][1], acc64[g][1], 0, 0, 0);
        acc64[g][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(az, b[g][2], acc64[g][0], 0, 0, 0);
        acc64[g][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(aw, b[g][3], acc64[g][1], 0, 0, 0);
      }
      daccy = fma(ax, y[0], daccy);
      daccy = fma(ay, y[1], daccy);
      daccy = fma(az, y[2], daccy);
      daccy = fma(aw, y[3], daccy);
    }
    // every LDS read of this stage has returned before the barrier that lets the loader refill it
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }

  // ---- epilogue (as in k_strip) ----
  double* __restrict__ out = static_cast<double*>(pt.out) + (uint64_t)it.out_part * pt.out_part_stride;
  const double dadd = (double)it.diag_add * pt.diag_add;
  const bool add_diag = (dadd != 0.0);
  const double scale = pt.scale;
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int col = 1 + 16 * g + m;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = wave * 16 + acc_row<true>(lane, i);
      if (row < nrows && col < T) {
        double v = scale * (acc64[g][0][i] + acc64[g][1][i]);
        if (add_diag) v = fma(dadd, vin[(uint64_t)(it.in_row0 + it.row_in_block + row) * T + col], v);
        const uint64_t idx = (uint64_t)(it.out_row0 + row) * T + col;
        if (pt.accumulate) v += out[idx];
        out[idx] = v;
      }
    }
  }
  daccy += __shfl_xor(daccy, 16);
  daccy += __shfl_xor(daccy, 32);
  if (kg == 0 && lr < nrows) {
    double v = scale * daccy;
    if (add_diag) v = fma(dadd, vin[(uint64_t)(it.in_row0 + it.row_in_block + lr) * T], v);
    const uint64_t idx = (uint64_t)(it.out_row0 + lr) * T;
    if (pt.accumulate) v += out[idx];
    out[idx] = v;
  }
#endif
}

// out[i] = sum over `parts` slabs of in[part * stride + i]  (fixed order: deterministic)
template <typename VT>
__global__ void k_sum_parts(const VT* __restrict__ in, VT* __restrict__ out, int64_t count, int parts,
                            uint64_t stride) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) {
    VT s = in[i];
    for (int p = 1; p < parts; ++p) s += in[(uint64_t)p * stride + i];
    out[i] = s;
  }
}

int launch_sum_parts(const void* in, void* out, int64_t count, int parts, uint64_t stride, bool acc64,
                     hipStream_t s) {
  const int grid = (int)std::min<int64_t>((count + 255) / 256, 2048);
  if (acc64)
    hipLaunchKernelGGL((k_sum_parts<double>), dim3(grid), dim3(256), 0, s, (const double*)in, (double*)out, count,
                       parts, stride);
  else
    hipLaunchKernelGGL((k_sum_parts<float>), dim3(grid), dim3(256), 0, s, (const float*)in, (float*)out, count,
                       parts, stride);
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

constexpr int RING1_CH = 32, RING1_ST = 4, RING2_CH = 32, RING2_ST = 3;     // chunk columns and ring depth by column groups
typedef RingCfg<1, RING1_CH, RING1_ST> Ring1;
typedef RingCfg<2, RING2_CH, RING2_ST> Ring2;

const char* strip_kernel_name(const StripTable& tab, int T, bool acc64) {
  const int ng = (T - 1 + 15) / 16;
  if (acc64 && ng == 1) {
    if (tab.sym && T == 17) return "k_strip_ring<1, 32, 4, true, 17>";
    if (tab.sym) return "k_strip_ring<1, 32, 4, true, 0>";
    if (T == 17) return "k_strip_ring<1, 32, 4, false, 17>";
    return "k_strip_ring<1, 32, 4, false, 0>";
  }
  if (acc64 && ng == 2) return T == 33 ? "k_strip_ring<2, 32, 3, false, 33>" : "k_strip_ring<2, 32, 3, false, 0>";
  if (acc64) return ng == 0 ? "k_strip<0, true>" : (ng == 1 ? "k_strip<1, true>" : "k_strip<2, true>");
  return ng == 0 ? "k_strip<0, false>" : (ng == 1 ? "k_strip<1, false>" : "k_strip<2, false>");
}
static_assert(RING1_CH == 32 && RING1_ST == 4 && RING2_CH == 32 && RING2_ST == 3, "strip_kernel_name spells these out");

template <bool ACC64>
static void launch_typed(int ng, dim3 grid, hipStream_t s, const StripArgs& a) {
  dim3 block(256);
  if (ng == 0) hipLaunchKernelGGL((k_strip<0, ACC64>), grid, block, 0, s, a);
  else if (ng == 1) hipLaunchKernelGGL((k_strip<1, ACC64>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((k_strip<2, ACC64>), grid, block, 0, s, a);
}

int launch_strip(const StripTable& tab, const StripPort& p0, const StripPort& p1, int T, bool acc64,
                 hipStream_t s) {
  if (tab.count == 0) return NUGPR_OK;
  if (T < 1 || T > MAX_COLS) { set_error("vector block wider than 33 columns"); return NUGPR_ERR_INVALID; }
  StripArgs a;
  a.port[0] = p0;
  a.port[1] = p1;
  a.items = tab.dev;
  a.T = T;
  a.magicT = T == 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)T + 1ull);
  const int ng = (T - 1 + 15) / 16;
  // the ring kernels use more than the default 64 KiB of dynamic LDS: raise their limit once
  static const hipError_t ring_attr = []() {
    const void* k1[] = {reinterpret_cast<const void*>(&k_strip_ring<1, RING1_CH, RING1_ST, false, 0>),
                        reinterpret_cast<const void*>(&k_strip_ring<1, RING1_CH, RING1_ST, true, 0>),
                        reinterpret_cast<const void*>(&k_strip_ring<1, RING1_CH, RING1_ST, false, 17>),
                        reinterpret_cast<const void*>(&k_strip_ring<1, RING1_CH, RING1_ST, true, 17>)};
    const void* k2[] = {reinterpret_cast<const void*>(&k_strip_ring<2, RING2_CH, RING2_ST, false, 0>),
                        reinterpret_cast<const void*>(&k_strip_ring<2, RING2_CH, RING2_ST, false, 33>)};
    for (const void* f : k1) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, Ring1::LDS_BYTES);
      if (e != hipSuccess) return e;
    }
    for (const void* f : k2) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, Ring2::LDS_BYTES);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }();
  NUGPR_HIP(ring_attr);
  // Tables with strips of symmetric blocks take the instantiation that pairs their tiles, the others the
  // plain loop.  With two column groups (T > 17) the launch is bound by the matrix cores, the pairing
  // saves nothing and its operand read costs 6 %: those launches read every strip whole.  The widths of
  // 16 and 32 probes have instantiations with T as a constant.
  const dim3 grid(tab.count), block(320);
  if (acc64 && ng == 1) {
    if (tab.sym && T == 17) hipLaunchKernelGGL((k_strip_ring<1, RING1_CH, RING1_ST, true, 17>), grid, block, Ring1::LDS_BYTES, s, a);
    else if (tab.sym) hipLaunchKernelGGL((k_strip_ring<1, RING1_CH, RING1_ST, true, 0>), grid, block, Ring1::LDS_BYTES, s, a);
    else if (T == 17) hipLaunchKernelGGL((k_strip_ring<1, RING1_CH, RING1_ST, false, 17>), grid, block, Ring1::LDS_BYTES, s, a);
    else hipLaunchKernelGGL((k_strip_ring<1, RING1_CH, RING1_ST, false, 0>), grid, block, Ring1::LDS_BYTES, s, a);
  } else if (acc64 && ng == 2) {
    if (T == 33) hipLaunchKernelGGL((k_strip_ring<2, RING2_CH, RING2_ST, false, 33>), grid, block, Ring2::LDS_BYTES, s, a);
    else hipLaunchKernelGGL((k_strip_ring<2, RING2_CH, RING2_ST, false, 0>), grid, block, Ring2::LDS_BYTES, s, a);
  }
  else if (acc64) launch_typed<true>(ng, dim3(tab.count), s, a);
  else launch_typed<false>(ng, dim3(tab.count), s, a);
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

}  // namespace nugpr
