// Host-side planning: argument validation, workspace layout, strip work tables.
#include <algorithm>
#include <cstring>

#include "nugpr_internal.h"

namespace nugpr {

static thread_local std::string g_last_error = "";

void set_error(const std::string& msg) { g_last_error = msg; }

const char* last_error_cstr() { return g_last_error.c_str(); }

int hip_fail(hipError_t e, const char* what) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  (void)hipGetLastError();
  return NUGPR_ERR_HIP;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static size_t take(size_t& cursor, size_t bytes) {
  size_t at = align_up(cursor, 256);
  cursor = at + bytes;
  return at;
}

int plan_layout(const nugpr_problem* pb, uint32_t flags, Layout& L) {
  if (!pb || !pb->cluster_offsets) { set_error("null problem or cluster_offsets"); return NUGPR_ERR_INVALID; }
  if (pb->n <= 0 || pb->n > (int64_t)0x7fff0000) { set_error("n out of range"); return NUGPR_ERR_INVALID; }
  if (pb->d < 1 || pb->d > MAX_D) { set_error("d must be 1..64"); return NUGPR_ERR_INVALID; }
  if (pb->n_clusters < 1 || pb->n_clusters > 65535) { set_error("n_clusters out of range"); return NUGPR_ERR_INVALID; }
  if (pb->rank < 1) { set_error("rank must be >= 1"); return NUGPR_ERR_INVALID; }
  if (pb->n_probes < 0 || pb->n_probes > MAX_COLS - 1) { set_error("n_probes must be 0..32"); return NUGPR_ERR_INVALID; }
  const int64_t* off = pb->cluster_offsets;
  if (off[0] != 0 || off[pb->n_clusters] != pb->n) { set_error("cluster_offsets must start at 0 and end at n"); return NUGPR_ERR_INVALID; }
  L = Layout();
  L.n = pb->n; L.d = pb->d; L.nc = pb->n_clusters; L.r = pb->rank; L.t = pb->n_probes;
  L.T = L.t + 1;
  L.p = (flags & NUGPR_ISOTROPIC) ? 3 : L.d + 2;
  L.max_iter = MAX_ITER_CAP;          // the coefficient logs are sized for the cap
  L.compensate = (flags & NUGPR_COMPENSATE) != 0;
  if ((int64_t)L.nc * L.r > (int64_t)1 << 24) { set_error("n_clusters*rank too large"); return NUGPR_ERR_INVALID; }
  L.ncr = L.nc * L.r;
  L.ldc = (int)align_up(L.ncr, TILE);
  L.ldw = (int)align_up(L.r, TILE);
  L.cl.resize(L.nc);
  uint64_t koff = 0, wtoff = 0, prow = 0;
  for (int i = 0; i < L.nc; ++i) {
    int64_t b = off[i + 1] - off[i];
    if (b < L.r) { set_error("a cluster is smaller than rank (or offsets not ascending)"); return NUGPR_ERR_INVALID; }
    if (b > 64 * 4096) { set_error("cluster too large"); return NUGPR_ERR_INVALID; }
    ClusterInfo& c = L.cl[i];
    c.row0 = (uint32_t)off[i];
    c.b = (uint32_t)b;
    c.ld = (uint32_t)align_up((size_t)b, TILE);
    c.nt = c.ld / TILE;
    c.koff = koff;
    c.wtoff = wtoff;
    c.prow = (uint32_t)prow;
    c.pad_ = 0;
    prow += c.ld;
    koff += (uint64_t)c.ld * c.ld;
    wtoff += (uint64_t)L.r * c.ld;
    L.ntmax = std::max<int>(L.ntmax, (int)c.nt);
    L.n_diag_tiles += (uint64_t)c.nt * (c.nt + 1) / 2;
  }
  L.kd_elems = koff;
  L.rows_pad = prow;
  if (prow > 0xffffffffull) { set_error("padded row count out of range"); return NUGPR_ERR_INVALID; }
  L.wt_elems = wtoff;
  {
    uint64_t ct = (uint64_t)L.ldc / TILE;
    L.n_c_tiles = ct * (ct + 1) / 2;
  }
  // how many column slabs the two reductions over long rows are split into
  {
    int strips_S = L.nc * ((L.r + TILE - 1) / TILE);
    int want = (1024 + strips_S - 1) / strips_S;
    int min_chunks = 1 << 30;
    for (auto& c : L.cl) min_chunks = std::min<int>(min_chunks, (int)c.nt);
    L.nsS = std::max(1, std::min({want, 8, min_chunks}));
    int strips_P = L.ldc / TILE;
    want = (2048 + strips_P - 1) / strips_P;
    L.nsP = std::max(1, std::min({want, 16, L.ldc / TILE}));
  }
  L.n_dot_blocks = (int)std::min<int64_t>(1024, (L.n + 255) / 256);

  size_t cur = 0;
  const size_t f = sizeof(float);
  const size_t vec = (size_t)L.n * L.T * sizeof(double);      // fp64 vector blocks (fp32 mode uses half)
  L.o_cl = take(cur, sizeof(ClusterInfo) * L.nc);
  L.o_Kd = take(cur, L.kd_elems * f);
  L.o_G = take(cur, L.kd_elems * f);
  L.o_C = take(cur, (size_t)L.ldc * L.ldc * f);
  L.o_Kd2 = take(cur, L.kd_elems * f);
  L.o_C2 = take(cur, (size_t)L.ldc * L.ldc * f);
  L.o_Wd = take(cur, (size_t)L.n * L.ldw * f);
  L.o_Wt = take(cur, L.wt_elems * f);
  L.o_reps = take(cur, (size_t)L.ncr * L.d * f);
  {
    const size_t kd = (size_t)((L.d + 3) & ~3);
    L.o_Xs = take(cur, (size_t)L.rows_pad * kd * sizeof(double));
    L.o_Xn = take(cur, (size_t)L.rows_pad * sizeof(double));
    L.o_Rs = take(cur, (size_t)L.ldc * kd * sizeof(double));
    L.o_Rn = take(cur, (size_t)L.ldc * sizeof(double));
  }
  // residual matrix of the compensated coupling; reserved whenever the problem is small enough for the
  // compensation, so that the workspace size does not depend on the flags
  // (larger couplings keep it in the spare coupling matrix, which only the pair assembly uses and the
  // compensation does without)
  if (L.ncr <= COMPENSATE_HOST_MAX) L.o_Clo = take(cur, (size_t)L.ldc * L.ldc * sizeof(float));
  if (L.ncr > COMPENSATE_HOST_MAX) L.o_dav = take(cur, eigmin_workspace_doubles((size_t)L.ldc, (size_t)L.ncr) * sizeof(double));
  L.o_assign = take(cur, (size_t)L.n * sizeof(int32_t));
  L.o_rep_ptr = take(cur, ((size_t)L.ncr + 1) * sizeof(int32_t));
  L.o_rep_pts = take(cur, (size_t)L.n * sizeof(int32_t));
  L.o_B = take(cur, vec);
  L.o_X = take(cur, vec);
  L.o_R = take(cur, vec);
  L.o_Z = take(cur, vec);
  L.o_D = take(cur, vec);
  L.o_Q = take(cur, vec);
  L.o_V = take(cur, vec);
  L.o_U = take(cur, vec);
  L.o_x0 = take(cur, (size_t)L.n * sizeof(double));
  L.o_Z0 = take(cur, vec);
  L.o_P = take(cur, vec);
  L.o_Q0 = take(cur, vec);
  L.o_S0 = take(cur, (size_t)L.ncr * L.T * sizeof(double));
  L.o_Spart = take(cur, (size_t)L.nsS * L.ncr * L.T * sizeof(double));
  L.o_Ppart = take(cur, (size_t)L.nsP * L.ncr * L.T * sizeof(double));
  L.o_dot = take(cur, (size_t)2 * L.n_dot_blocks * MAX_COLS * sizeof(double));
  L.o_state = take(cur, sizeof(PcgState));
  L.o_alog = take(cur, (size_t)L.max_iter * MAX_COLS * sizeof(double));
  L.o_blog = take(cur, (size_t)L.max_iter * MAX_COLS * sizeof(double));
  L.o_logdet = take(cur, (size_t)L.nc * sizeof(double));
  // tile list of the diagonal blocks (mirroring) + row-panel work items of the two assembly launches
  // tile list of the diagonal blocks + the assembly work items (32 bytes each, at most one per tile)
  L.o_tiles = take(cur, (5 * L.n_diag_tiles + 4 * L.n_c_tiles) * sizeof(uint64_t));
  // strip tables: exact item counts
  size_t items = 0;
  for (auto& c : L.cl) {
    items += (size_t)((L.r + TILE - 1) / TILE) * L.nsS;  // Wt * D
    items += c.nt;                                       // K_ii * D
    items += c.nt;                                       // W * P
    items += 3 * (size_t)c.nt;                           // tril(G), triu(G), tril(L)
  }
  items += 2 * (size_t)(L.ldc / TILE) * L.nsP;           // C * S, in the joint table and on its own
  L.items_bytes = items * sizeof(StripItem);
  L.o_items = take(cur, L.items_bytes);
  L.total = align_up(cur, 256);
  return NUGPR_OK;
}

}  // namespace nugpr
