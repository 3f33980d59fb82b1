// Strip GEMM: the bandwidth-bound product of a stored fp32 matrix strip (64 rows,
// any number of columns) with a tall-skinny vector block of T <= 33 columns.
//
// Every matrix of the hot path is applied through this one kernel:
//   K_ii D_i, C S (coupling), W_i^T D_i, W_i P_i        -- the block-low-rank product
//                                                          K' D of eq. (odsplit), Section 3.3
//   tril(L_i^-1) R_i, triu(L_i^-T) V_i                   -- the block-Jacobi preconditioner,
//                                                          applied as explicit inverses (Table 2)
//   tril(L_i) Z_i                                        -- probe right-hand sides
//
// Design (gfx950, wave64): a workgroup of 4 waves owns a strip of 64 matrix rows,
// each wave 16 of them, and walks along the rows so every matrix element is read
// from HBM exactly once, with 16-byte loads, for all T columns.  Lane (m, kg) of a
// wave loads float4 A[row m][c + 16 s + 4 kg ..]; the four components feed four
// v_mfma_f32_16x16x4_f32, whose contraction index is the kg of the lane, so the
// column permutation inside a 16-column group is absorbed by reading the matching
// rows of the vector block from LDS (stored as float4 over 4 consecutive rows).
// Columns 1..T-1 (the probes) go through the matrix cores in groups of 16; column 0
// (y) rides on the vector ALUs from the same registers, so T = 17 costs one MFMA
// group, not two.  The vector block chunk is double-buffered in LDS, the matrix
// chunk is prefetched one stage ahead in registers.
#include "nugpr_internal.h"

namespace nugpr {

typedef float v4f __attribute__((ext_vector_type(4)));

template <int NG, int CHUNK>
__global__ __launch_bounds__(256) void k_strip(const StripArgs a) {
  constexpr int NL = CHUNK / 16;                 // float4 loads per lane per chunk
  constexpr int NCOLM = NG > 0 ? 16 * NG : 1;    // columns handled by the matrix cores
  constexpr int NE = (CHUNK * (16 * NG + 1) + 255) / 256;   // staged vector elements per thread
  __shared__ float4 sB[2][(CHUNK / 4) * NCOLM];
  __shared__ __attribute__((aligned(16))) float sY[2][CHUNK];

  const StripItem it = a.items[blockIdx.x];
  const StripPort& pt = a.port[it.port];
  const int T = a.T;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int m = lane & 15, kg = lane >> 4;
  const int nrows = (int)it.nrows;
  const int lda = (int)it.lda;
  const int lr = wave * 16 + m;                               // local row this lane loads
  const int lrc = lr < nrows ? lr : nrows - 1;
  const float* __restrict__ Arow = pt.A + it.a_off + (uint64_t)lrc * (uint64_t)lda;
  const int diag = (int)it.row_in_block + lr;                 // diagonal column of that row
  const int mode = it.mode;
  const int c_begin = (int)it.c_begin, c_end = (int)it.c_end;
  const int nchunks = c_end > c_begin ? (c_end - c_begin + CHUNK - 1) / CHUNK : 0;

  // zero the LDS once: the padding columns of the MFMA operand are never written again
  for (int i = tid; i < 2 * (CHUNK / 4) * NCOLM; i += 256) (&sB[0][0])[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  __syncthreads();

  v4f acc[NG > 0 ? NG : 1];
#pragma unroll
  for (int g = 0; g < (NG > 0 ? NG : 1); ++g) acc[g] = (v4f){0.f, 0.f, 0.f, 0.f};
  float accy = 0.f;

  // staging slots of this thread: flat element e of the chunk's (CHUNK x T) slab
  const int nelem = CHUNK * T;
  int e_q[NE], e_col[NE];
#pragma unroll
  for (int k = 0; k < NE; ++k) {
    int e = tid + 256 * k;
    int q = (T == 1) ? e : (int)__umulhi((uint32_t)e, a.magicT);
    e_q[k] = e < nelem ? q : -1;
    e_col[k] = e - q * T;
  }

  auto load_A = [&](int c, float4 (&reg)[NL]) {
#pragma unroll
    for (int s = 0; s < NL; ++s) {
      int col = c + 16 * s + 4 * kg;
      if (col < lda) reg[s] = *reinterpret_cast<const float4*>(Arow + col);
      else reg[s] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto load_in = [&](int c, float (&reg)[NE]) {
#pragma unroll
    for (int k = 0; k < NE; ++k) {
      float v = 0.f;
      int q = e_q[k];
      if (q >= 0 && c + q < c_end) {
        uint64_t idx = (uint64_t)(it.in_row0 + (uint32_t)(c + q)) * (uint64_t)T + (uint32_t)e_col[k];
        v = pt.in[idx];
        for (int part = 1; part < pt.nin; ++part) v += pt.in[idx + (uint64_t)part * pt.in_part_stride];
      }
      reg[k] = v;
    }
  };
  auto store_in = [&](int buf, const float (&reg)[NE]) {
#pragma unroll
    for (int k = 0; k < NE; ++k) {
      int q = e_q[k];
      if (q >= 0) {
        int col = e_col[k];
        if (col == 0) sY[buf][q] = reg[k];
        else if (NG > 0) reinterpret_cast<float*>(&sB[buf][(q >> 2) * NCOLM + (col - 1)])[q & 3] = reg[k];
      }
    }
  };

  float4 areg[NL], anext[NL];
  float inreg[NE];
  if (nchunks > 0) {
    load_A(c_begin, areg);
    load_in(c_begin, inreg);
    store_in(0, inreg);
  }
  __syncthreads();

  for (int ch = 0; ch < nchunks; ++ch) {
    const int c = c_begin + ch * CHUNK;
    const int buf = ch & 1;
    const bool more = ch + 1 < nchunks;
    if (more) {
      load_A(c + CHUNK, anext);
      load_in(c + CHUNK, inreg);
    }
    // elements outside the item's column range or on the wrong side of the diagonal are dropped
    const bool need_mask = (c + CHUNK > c_end) || (mode == 1 && c + CHUNK > (int)it.row_in_block) ||
                           (mode == 2 && c < (int)it.row_in_block + TILE);
    if (need_mask) {
#pragma unroll
      for (int s = 0; s < NL; ++s) {
        int q0 = c + 16 * s + 4 * kg;
        float* v = reinterpret_cast<float*>(&areg[s]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          int q = q0 + j;
          bool ok = q < c_end;
          if (mode == 1) ok = ok && (q <= diag);
          if (mode == 2) ok = ok && (q >= diag);
          v[j] = ok ? v[j] : 0.f;
        }
      }
    }
#pragma unroll
    for (int s = 0; s < NL; ++s) {
      const float4 av = areg[s];
      if (NG > 0) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const float4 bv = sB[buf][(4 * s + kg) * NCOLM + 16 * g + m];
          acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.x, acc[g], 0, 0, 0);
          acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bv.y, acc[g], 0, 0, 0);
          acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, bv.z, acc[g], 0, 0, 0);
          acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, bv.w, acc[g], 0, 0, 0);
        }
      }
      const float4 yv = *reinterpret_cast<const float4*>(&sY[buf][16 * s + 4 * kg]);
      accy = fmaf(av.x, yv.x, accy);
      accy = fmaf(av.y, yv.y, accy);
      accy = fmaf(av.z, yv.z, accy);
      accy = fmaf(av.w, yv.w, accy);
    }
    if (more) {
      store_in(buf ^ 1, inreg);
#pragma unroll
      for (int s = 0; s < NL; ++s) areg[s] = anext[s];
    }
    __syncthreads();
  }

  // ---- epilogue ----
  float* __restrict__ out = pt.out + (uint64_t)it.out_part * pt.out_part_stride;
  const float dadd = it.diag_add * pt.diag_add;     // residual of the fp32 diagonal, see build_blocks
  const bool add_diag = (dadd != 0.f);
  if (NG > 0) {
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int col = 1 + 16 * g + m;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = wave * 16 + 4 * kg + i;
        if (row < nrows && col < T) {
          float v = acc[g][i];
          if (add_diag)
            v = fmaf(dadd, pt.in[(uint64_t)(it.in_row0 + it.row_in_block + row) * T + col], v);
          const uint64_t idx = (uint64_t)(it.out_row0 + row) * T + col;
          if (pt.accumulate) v += out[idx];
          out[idx] = v;
        }
      }
    }
  }
  accy += __shfl_xor(accy, 16);
  accy += __shfl_xor(accy, 32);
  if (kg == 0 && lr < nrows) {
    float v = accy;
    if (add_diag) v = fmaf(dadd, pt.in[(uint64_t)(it.in_row0 + it.row_in_block + lr) * T], v);
    const uint64_t idx = (uint64_t)(it.out_row0 + lr) * T;
    if (pt.accumulate) v += out[idx];
    out[idx] = v;
  }
}

static int g_chunk = 0;

int launch_strip(const StripTable& tab, const StripPort& p0, const StripPort& p1, int T, hipStream_t s) {
  if (tab.count == 0) return NUGPR_OK;
  if (T < 1 || T > MAX_COLS) { set_error("vector block wider than 33 columns"); return NUGPR_ERR_INVALID; }
  if (g_chunk == 0) {
    const char* e = getenv("NUGPR_STRIP_CHUNK");
    g_chunk = (e && atoi(e) == 64) ? 64 : 128;
  }
  StripArgs a;
  a.port[0] = p0;
  a.port[1] = p1;
  a.items = tab.dev;
  a.T = T;
  a.magicT = T == 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)T + 1ull);
  const int ng = (T - 1 + 15) / 16;
  dim3 grid(tab.count), block(256);
#define LAUNCH(NGV, CH) hipLaunchKernelGGL((k_strip<NGV, CH>), grid, block, 0, s, a)
  if (g_chunk == 64) {
    if (ng == 0) LAUNCH(0, 64); else if (ng == 1) LAUNCH(1, 64); else LAUNCH(2, 64);
  } else {
    if (ng == 0) LAUNCH(0, 128); else if (ng == 1) LAUNCH(1, 128); else LAUNCH(2, 128);
  }
#undef LAUNCH
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

}  // namespace nugpr
