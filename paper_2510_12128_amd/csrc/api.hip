// C ABI of libnugpr: context set-up, the five entry points of the hot path, and the
// host-side parts of one loss evaluation (SLQ log-determinant, central differences, Adam).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <mutex>
#include <new>
#include <vector>

#include "nugpr_internal.h"

using namespace nugpr;

namespace {

// plain 16-byte grid-stride copy: the known-size reference the HBM byte counters are scaled by
__global__ void k_copy16(const float4* __restrict__ src, float4* __restrict__ dst, size_t count) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// ---- scratch memory of the entry point that allocates nothing (nugpr_matvec_static) ----------------
// One file-scope device array per GPU the library is loaded on, held until the process ends.  Host code
// never uses the array's name as an address: its device address is looked up once per device with
// hipGetSymbolAddress (at nugpr_create, with that device current) and kept in g_scratch_ptr.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// address of `scratch` on the CURRENT device (looked up on first use), or an error code
int scratch_address(int* device_out, void** ptr_out) {
  int dev = -1;
  NUGPR_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) { set_error("device index out of range"); return NUGPR_ERR_INVALID; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    NUGPR_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) { set_error("hipGetSymbolAddress returned a null address for the static scratch"); return NUGPR_ERR_HIP; }
    g_scratch_ptr[dev] = ptr;
  }
  if (device_out) *device_out = dev;
  if (ptr_out) *ptr_out = g_scratch_ptr[dev];
  return NUGPR_OK;
}

// ---- strip work tables ------------------------------------------------------
StripItem make_item(uint64_t a_off, uint32_t lda, uint32_t nrows, uint32_t c_begin, uint32_t c_end,
                    uint32_t in_row0, uint32_t out_row0, uint32_t row_in_block, int out_part, int port, int mode,
                    float diag_add) {
  StripItem it{};
  it.a_off = a_off; it.lda = lda; it.nrows = nrows; it.c_begin = c_begin; it.c_end = c_end;
  it.in_row0 = in_row0; it.out_row0 = out_row0; it.row_in_block = row_in_block;
  it.out_part = (uint16_t)out_part; it.port = (uint8_t)port; it.mode = (uint8_t)mode; it.diag_add = diag_add;
  return it;
}

void sort_longest_first(std::vector<StripItem>& v) {
  std::stable_sort(v.begin(), v.end(), [](const StripItem& a, const StripItem& b) {
    const uint32_t la = a.c_end > a.c_begin ? a.c_end - a.c_begin : 0;
    const uint32_t lb = b.c_end > b.c_begin ? b.c_end - b.c_begin : 0;
    return la > lb;
  });
}

// Workgroups are handed to the 8 accelerator dies (XCDs, each with its own L2) round-robin by
// workgroup index.  Items that read the same rows of the vector block (the strips of one cluster,
// the row strips of one column slab of C) are therefore placed 8 apart, so that they run on ONE die
// and the slab is fetched from HBM once instead of once per die.  Inside a die's queue the order
// (longest first) is kept.
constexpr int NUM_XCD = 8;
void arrange_for_dies(std::vector<StripItem>& v) {
  if (v.size() < 2 * NUM_XCD) return;
  std::vector<std::vector<StripItem>> q(NUM_XCD);
  std::vector<uint64_t> keys;
  for (const StripItem& it : v) {
    const uint64_t key = ((uint64_t)it.port << 62) | ((uint64_t)it.in_row0 << 30) | (uint64_t)(it.c_begin & 0x3fffffffu);
    size_t g = 0;
    // groups are few (clusters + column slabs): a linear search over the last ones seen is enough
    for (g = keys.size(); g > 0 && keys[g - 1] != key; --g) {}
    if (g == 0) { keys.push_back(key); g = keys.size(); }
    q[(g - 1) % NUM_XCD].push_back(it);
  }
  std::vector<size_t> pos(NUM_XCD, 0);
  std::vector<StripItem> out;
  out.reserve(v.size());
  while (out.size() < v.size()) {
    const int die = (int)(out.size() % NUM_XCD);
    int src = die;
    if (pos[src] >= q[src].size()) {          // this die's queue is empty: take from the fullest one
      size_t best = 0;
      for (int k = 0; k < NUM_XCD; ++k)
        if (q[k].size() - pos[k] > best) { best = q[k].size() - pos[k]; src = k; }
    }
    out.push_back(q[src][pos[src]++]);
  }
  v.swap(out);
}

// The same for whole groups of items that must run together (the strips of one cluster; the two sets of
// strips that share the tiles of a pair of super-blocks of the coupling matrix): the groups go to the dies
// in turn, in the order given, each die works through its groups in order, and a die whose queue has run
// dry takes from the fullest one.
uint64_t group_work(const std::vector<StripItem>& g) {
  uint64_t w = 0;
  for (const StripItem& it : g) w += it.c_end > it.c_begin ? it.c_end - it.c_begin : 0;
  return w;
}
void heaviest_first(std::vector<std::vector<StripItem>>& groups, size_t from) {
  std::stable_sort(groups.begin() + from, groups.end(),
                   [](const std::vector<StripItem>& a, const std::vector<StripItem>& b) { return group_work(a) > group_work(b); });
}
std::vector<StripItem> deal_groups(std::vector<std::vector<StripItem>>& groups) {
  std::vector<std::vector<StripItem>> q(NUM_XCD);
  size_t total = 0;
  for (size_t g = 0; g < groups.size(); ++g) {
    q[g % NUM_XCD].insert(q[g % NUM_XCD].end(), groups[g].begin(), groups[g].end());
    total += groups[g].size();
  }
  std::vector<size_t> pos(NUM_XCD, 0);
  std::vector<StripItem> out;
  out.reserve(total);
  while (out.size() < total) {
    int src = (int)(out.size() % NUM_XCD);
    if (pos[src] >= q[src].size()) {
      size_t best = 0;
      for (int k = 0; k < NUM_XCD; ++k)
        if (q[k].size() - pos[k] > best) { best = q[k].size() - pos[k]; src = k; }
    }
    out.push_back(q[src][pos[src]++]);
  }
  return out;
}

struct Tables {
  std::vector<StripItem> WtD, KC, Conly, WP, lowG, upG, lowL;
};

void build_tables(const Layout& L, Tables& t) {
  const uint32_t r = (uint32_t)L.r;
  std::vector<std::vector<StripItem>> kc_groups;      // work of the K_diag + C launch, by group (deal_groups)
  for (int i = 0; i < L.nc; ++i) {
    const ClusterInfo& c = L.cl[i];
    kc_groups.emplace_back();
    // S_i = W_i^T D_i: strips over the r rows of W_i^T, columns split into nsS slabs
    const uint32_t chunks = c.nt, cpp = (chunks + L.nsS - 1) / L.nsS;
    for (uint32_t rs = 0; rs * TILE < r; ++rs) {
      const uint32_t nrows = std::min<uint32_t>(TILE, r - rs * TILE);
      for (int k = 0; k < L.nsS; ++k) {
        const uint32_t cb = std::min<uint32_t>(k * cpp, chunks) * TILE;
        const uint32_t ce = std::min<uint32_t>(std::min<uint32_t>((k + 1) * cpp, chunks) * TILE, c.b);
        t.WtD.push_back(make_item(c.wtoff + (uint64_t)rs * TILE * c.ld, c.ld, nrows, cb, std::max(cb, ce), c.row0,
                                  (uint32_t)i * r + rs * TILE, 0, k, 0, 0, 0.f));
      }
    }
    for (uint32_t s = 0; s < c.nt; ++s) {
      const uint32_t nrows = std::min<uint32_t>(TILE, c.b - s * TILE);
      const uint64_t a_off = c.koff + (uint64_t)s * TILE * c.ld;
      const uint32_t row = c.row0 + s * TILE;
      kc_groups.back().push_back(make_item(a_off, c.ld, nrows, 0, c.b, c.row0, row, s * TILE, 0, 0, 0, 1.f));
      kc_groups.back().back().blocked = c.nt >= 2 ? 3 : 1;      // K_ii is symmetric: its strips pair up tile by tile
      t.WP.push_back(make_item((uint64_t)row * L.ldw, (uint32_t)L.ldw, nrows, 0, r, (uint32_t)i * r, row, 0, 0, 0, 0, 0.f));
      t.lowG.push_back(make_item(a_off, c.ld, nrows, 0, s * TILE + nrows, c.row0, row, s * TILE, 0, 0, 1, 0.f));
      t.upG.push_back(make_item(a_off, c.ld, nrows, s * TILE, c.b, c.row0, row, s * TILE, 0, 0, 2, 0.f));
      t.lowL.push_back(make_item(a_off, c.ld, nrows, 0, s * TILE + nrows, c.row0, row, s * TILE, 0, 0, 1, 0.f));
      t.lowG.back().blocked = t.upG.back().blocked = t.lowL.back().blocked = 1;     // L and L^-1 are stored blocked too
    }
  }
  // the clusters first, heaviest first (the assembly writes cluster 0 last, so with equal clusters the product
  // starts on blocks that are still in the memory-side cache), then the groups of the coupling matrix
  heaviest_first(kc_groups, 0);
  const size_t first_c_group = kc_groups.size();
  // P = C S: strips over the n_c r rows of C, columns split into nsP slabs of cpp tiles.  C is symmetric:
  // with the strips grouped like the slabs, the strips of row group I on slab k and the strips of row group
  // k on slab I share their tiles (one set reads them transposed) and form one group of work; see
  // k_strip_ring for the order in which they visit them.
  {
    const uint32_t ncr = (uint32_t)L.ncr, chunks = (uint32_t)L.ldc / TILE, cpp = (chunks + L.nsP - 1) / L.nsP;
    const uint32_t ngroups = (chunks + cpp - 1) / cpp;              // non-empty slabs = row groups
    const bool pairing = chunks >= 2 && cpp <= 1023;
    auto c_item = [&](uint32_t rs, int k) {
      const uint32_t nrows = std::min<uint32_t>(TILE, ncr - rs * TILE);
      const uint32_t cb = std::min<uint32_t>(k * cpp, chunks) * TILE;
      const uint32_t ce = std::min<uint32_t>(std::min<uint32_t>((k + 1) * cpp, chunks) * TILE, ncr);
      StripItem it = make_item((uint64_t)rs * TILE * L.ldc, (uint32_t)L.ldc, nrows, cb, std::max(cb, ce), 0, rs * TILE,
                               rs * TILE, k, 1, 0, 0.f);
      it.blocked = 1;
      // the item whose columns hold the strip's own rows adds the port's scalar diagonal (used when the diagonal
      // of the matrix is carried as an exact scalar: the eigenvalue iteration for lambda_0)
      it.diag_add = (rs / cpp == (uint32_t)k) ? 1.f : 0.f;
      if (pairing && (uint32_t)k < ngroups) {
        const uint32_t I = rs / cpp, na = std::min<uint32_t>(cpp, chunks - I * cpp), jr = rs - I * cpp;
        const uint32_t kind = I == (uint32_t)k ? 0u : (I > (uint32_t)k ? 1u : 2u);
        it.blocked = 3u | (kind << 2) | (na << 4) | (jr << 15);
      }
      return it;
    };
    for (uint32_t I = 0; I < ngroups; ++I)
      for (uint32_t k = I; k < ngroups; ++k) {
        kc_groups.emplace_back();
        for (uint32_t rs = I * cpp; rs < std::min<uint32_t>((I + 1) * cpp, chunks) && rs * TILE < ncr; ++rs)
          kc_groups.back().push_back(c_item(rs, (int)k));
        if (k != I)
          for (uint32_t rs = k * cpp; rs < std::min<uint32_t>((k + 1) * cpp, chunks) && rs * TILE < ncr; ++rs)
            kc_groups.back().push_back(c_item(rs, (int)I));
      }
    // slabs past the last tile are empty; their items only clear their slab of the partial sums
    kc_groups.emplace_back();
    for (int k = (int)ngroups; k < L.nsP; ++k)
      for (uint32_t rs = 0; rs * TILE < ncr; ++rs) kc_groups.back().push_back(c_item(rs, k));
  }
  heaviest_first(kc_groups, first_c_group);
  t.KC = deal_groups(kc_groups);
  sort_longest_first(t.WtD);
  sort_longest_first(t.lowG);
  sort_longest_first(t.upG);
  sort_longest_first(t.lowL);
  for (const StripItem& it : t.KC)
    if (it.port == 1) t.Conly.push_back(it);       // the coupling product on its own (eq. (linear1) route)
  arrange_for_dies(t.lowG);
  arrange_for_dies(t.upG);
  arrange_for_dies(t.lowL);
}

int upload_table(const std::vector<StripItem>& v, StripItem*& cursor, StripTable& tab, hipStream_t s) {
  tab.dev = cursor;
  tab.count = (int)v.size();
  tab.sym = false;
  for (const StripItem& it : v) tab.sym = tab.sym || (it.blocked & 2u) != 0;
  if (!v.empty())
    NUGPR_HIP(hipMemcpyAsync(cursor, v.data(), v.size() * sizeof(StripItem), hipMemcpyHostToDevice, s));
  cursor += v.size();
  return NUGPR_OK;
}

}  // namespace

extern "C" {

const char* nugpr_last_error_string(void) { return last_error_cstr(); }

size_t nugpr_workspace_bytes(const nugpr_problem* problem) {
  Layout L;
  if (plan_layout(problem, 0, L) != NUGPR_OK) return 0;
  return L.total;
}

int32_t nugpr_num_hyper(const nugpr_ctx* ctx) { return ctx ? ctx->L.p : 0; }

int nugpr_create(nugpr_ctx** out, const nugpr_problem* pb, const nugpr_params* prm, void* stream) {
  if (!out) { set_error("ctx out-pointer is null"); return NUGPR_ERR_INVALID; }
  *out = nullptr;
  if (!pb || !prm) { set_error("problem or params is null"); return NUGPR_ERR_INVALID; }
  if (!(prm->tol > 0.0) || !(prm->tol < 1.0)) { set_error("tol must be in (0, 1)"); return NUGPR_ERR_INVALID; }
  if (prm->max_iter < 1 || prm->max_iter > MAX_ITER_CAP) { set_error("max_iter must be 1..4096"); return NUGPR_ERR_INVALID; }
  if (!(prm->fd_step > 0.0) || !(prm->lr >= 0.0)) { set_error("fd_step must be > 0 and lr >= 0"); return NUGPR_ERR_INVALID; }
  if (prm->fd_max_halvings < 0 || prm->fd_max_halvings > 30 || !(prm->fd_threshold >= 0.0)) {
    set_error("fd_max_halvings must be 0..30 and fd_threshold >= 0");
    return NUGPR_ERR_INVALID;
  }
  Layout L;
  int rc = plan_layout(pb, prm->flags, L);
  if (rc) return rc;
  if (L.compensate && L.ncr > COMPENSATE_HOST_MAX && (prm->flags & NUGPR_ACC_FP32)) {
    set_error("NUGPR_COMPENSATE with n_clusters * rank > 512 needs the default (fp64) arithmetic mode");
    return NUGPR_ERR_INVALID;
  }
  if ((prm->flags & NUGPR_PRECOND_COMPENSATED) && (!L.compensate || pb->W)) {
    set_error("NUGPR_PRECOND_COMPENSATED needs NUGPR_COMPENSATE and the default basis (W = null)");
    return NUGPR_ERR_INVALID;
  }
  if (!pb->X || !pb->y || (pb->n_probes > 0 && !pb->probes)) { set_error("X, y or probes is null"); return NUGPR_ERR_INVALID; }
  if (!pb->workspace || (reinterpret_cast<uintptr_t>(pb->workspace) & 255u)) {
    set_error("workspace is null or not 256-byte aligned");
    return NUGPR_ERR_WORKSPACE;
  }
  if (pb->workspace_bytes < L.total) { set_error("workspace smaller than nugpr_workspace_bytes()"); return NUGPR_ERR_WORKSPACE; }
  if ((reinterpret_cast<uintptr_t>(pb->X) & 3u) || (reinterpret_cast<uintptr_t>(pb->y) & 3u)) {
    set_error("X / y misaligned");
    return NUGPR_ERR_INVALID;
  }
  int device = -1;
  if ((rc = scratch_address(&device, nullptr))) return rc;      // also records which GPU this context lives on
  nugpr_ctx* c = new (std::nothrow) nugpr_ctx();
  if (!c) { set_error("out of host memory"); return NUGPR_ERR_INVALID; }
  c->device = device;
  c->L = L;
  c->params = *prm;
  c->acc64 = (prm->flags & NUGPR_ACC_FP32) == 0;
  if (c->params.beta1 == 0.0) c->params.beta1 = 0.9;
  if (c->params.beta2 == 0.0) c->params.beta2 = 0.999;
  if (c->params.eps == 0.0) c->params.eps = 1e-8;
  if (c->params.fd_max_halvings == 0) c->params.fd_max_halvings = 8;
  if (c->params.fd_threshold == 0.0) c->params.fd_threshold = 1e-2;
  c->fd_halvings.assign(L.p, 0);
  c->ws = static_cast<char*>(pb->workspace);
  c->X = pb->X; c->y = pb->y; c->probes = pb->probes;
  char* w = c->ws;
  c->d_cl = reinterpret_cast<ClusterInfo*>(w + L.o_cl);
  c->Kd = reinterpret_cast<float*>(w + L.o_Kd);
  c->G = reinterpret_cast<float*>(w + L.o_G);
  c->C = reinterpret_cast<float*>(w + L.o_C);
  c->Kd2 = reinterpret_cast<float*>(w + L.o_Kd2);
  c->Q0v = w + L.o_Q0;
  c->C2 = reinterpret_cast<float*>(w + L.o_C2);
  c->Clo = !L.compensate ? nullptr : (L.ncr <= COMPENSATE_HOST_MAX ? reinterpret_cast<float*>(w + L.o_Clo) : c->C2);
  c->dav = L.ncr > COMPENSATE_HOST_MAX ? reinterpret_cast<double*>(w + L.o_dav) : nullptr;
  c->Wd = reinterpret_cast<float*>(w + L.o_Wd);
  c->Wt = reinterpret_cast<float*>(w + L.o_Wt);
  c->reps = reinterpret_cast<float*>(w + L.o_reps);
  c->Xs = reinterpret_cast<double*>(w + L.o_Xs);
  c->Xn = reinterpret_cast<double*>(w + L.o_Xn);
  c->Rs = reinterpret_cast<double*>(w + L.o_Rs);
  c->Rn = reinterpret_cast<double*>(w + L.o_Rn);
  c->Bv = w + L.o_B;
  c->Xv = w + L.o_X;
  c->Rv = w + L.o_R;
  c->Zv = w + L.o_Z;
  c->Dv = w + L.o_D;
  c->Qv = w + L.o_Q;
  c->Vv = w + L.o_V;
  c->Uv = w + L.o_U;
  c->x0 = w + L.o_x0;
  c->Z0v = w + L.o_Z0;
  c->S0v = w + L.o_S0;
  c->assign = reinterpret_cast<int32_t*>(w + L.o_assign);
  c->rep_ptr = reinterpret_cast<int32_t*>(w + L.o_rep_ptr);
  c->rep_pts = reinterpret_cast<int32_t*>(w + L.o_rep_pts);
  c->Pv = w + L.o_P;
  c->Spart = w + L.o_Spart;
  c->Ppart = w + L.o_Ppart;
  c->dotpart = reinterpret_cast<double*>(w + L.o_dot);
  c->d_state = reinterpret_cast<PcgState*>(w + L.o_state);
  c->alog = reinterpret_cast<double*>(w + L.o_alog);
  c->blog = reinterpret_cast<double*>(w + L.o_blog);
  c->d_logdet = reinterpret_cast<double*>(w + L.o_logdet);
  c->d_tiles = reinterpret_cast<uint64_t*>(w + L.o_tiles);
  hipStream_t s = as_stream(stream);

  auto fail = [&](int code) { nugpr_destroy(c); return code; };
  // pinned host staging (host memory; the library allocates no device memory)
  c->h_buf_doubles = (size_t)2 * MAX_ITER_CAP * MAX_COLS + (size_t)1024 * MAX_COLS + sizeof(PcgState) + L.nc;
  hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&c->h_flags), sizeof(HostFlags), hipHostMallocDefault);
  if (e != hipSuccess) return fail(hip_fail(e, "hipHostMalloc(flags)"));
  e = hipHostMalloc(reinterpret_cast<void**>(&c->h_buf), c->h_buf_doubles * sizeof(double), hipHostMallocDefault);
  if (e != hipSuccess) return fail(hip_fail(e, "hipHostMalloc(buf)"));
  std::memset(c->h_flags, 0, sizeof(HostFlags));

  e = hipMemsetAsync(c->d_state, 0, sizeof(PcgState), s);         // counters in it start at zero
  if (e != hipSuccess) return fail(hip_fail(e, "clear solver state"));
  e = hipMemcpyAsync(c->d_cl, L.cl.data(), sizeof(ClusterInfo) * L.nc, hipMemcpyHostToDevice, s);
  if (e != hipSuccess) return fail(hip_fail(e, "upload cluster table"));
  Tables t;
  build_tables(L, t);
  const size_t total_items = t.WtD.size() + t.KC.size() + t.Conly.size() + t.WP.size() + t.lowG.size() + t.upG.size() + t.lowL.size();
  if (total_items * sizeof(StripItem) > L.items_bytes) { set_error("internal: strip table overflow"); return fail(NUGPR_ERR_INVALID); }
  StripItem* cur = reinterpret_cast<StripItem*>(w + L.o_items);
  if ((rc = upload_table(t.WtD, cur, c->tab_WtD, s))) return fail(rc);
  if ((rc = upload_table(t.KC, cur, c->tab_KC, s))) return fail(rc);
  c->c_paired = false;
  for (const StripItem& it : t.KC) c->c_paired = c->c_paired || (it.port == 1 && (it.blocked & 2u) != 0);
  if ((rc = upload_table(t.Conly, cur, c->tab_C, s))) return fail(rc);
  if ((rc = upload_table(t.WP, cur, c->tab_WP, s))) return fail(rc);
  if ((rc = upload_table(t.lowG, cur, c->tab_lowG, s))) return fail(rc);
  if ((rc = upload_table(t.upG, cur, c->tab_upG, s))) return fail(rc);
  if ((rc = upload_table(t.lowL, cur, c->tab_lowL, s))) return fail(rc);
  e = hipStreamSynchronize(s);          // host vectors go out of scope below
  if (e != hipSuccess) return fail(hip_fail(e, "sync after table upload"));
  if ((rc = launch_setup(c, pb->reps, pb->W, s))) return fail(rc);
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail(hip_fail(e, "sync after setup"));
  if (!pb->W) {
    // default basis: the points of every representative, in ascending order (counting sort on the host, once)
    std::vector<int32_t> as((size_t)L.n), ptr((size_t)L.ncr + 1, 0), pts((size_t)L.n);
    e = hipMemcpy(as.data(), c->assign, as.size() * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(hip_fail(e, "copy the basis assignment to the host"));
    for (int64_t p = 0; p < L.n; ++p) {
      if (as[p] < 0 || as[p] >= L.ncr) { set_error("internal: basis assignment out of range"); return fail(NUGPR_ERR_INVALID); }
      ptr[as[p] + 1] += 1;
    }
    for (int a = 0; a < L.ncr; ++a) ptr[a + 1] += ptr[a];
    std::vector<int32_t> fill(ptr.begin(), ptr.end() - 1);
    for (int64_t p = 0; p < L.n; ++p) pts[fill[as[p]]++] = (int32_t)p;
    e = hipMemcpy(c->rep_ptr, ptr.data(), ptr.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->rep_pts, pts.data(), pts.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(hip_fail(e, "upload the basis lists"));
    c->onehot = true;
  }
  if (L.compensate && L.ncr <= COMPENSATE_HOST_MAX) {
    // lambda_0 is computed on the host from the representatives themselves, in fp64
    std::vector<float> hr((size_t)L.ncr * L.d);
    e = hipMemcpy(hr.data(), c->reps, hr.size() * sizeof(float), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(hip_fail(e, "copy representatives to the host"));
    c->h_reps.assign(hr.begin(), hr.end());
  }
  *out = c;
  return NUGPR_OK;
}

int nugpr_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || (bytes & 15u) || ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u)) {
    set_error("copy_probe needs 16-byte aligned buffers and a multiple of 16 bytes");
    return NUGPR_ERR_INVALID;
  }
  hipLaunchKernelGGL(k_copy16, dim3(8192), dim3(256), 0, as_stream(stream), static_cast<const float4*>(src),
                     static_cast<float4*>(dst), bytes / 16);
  NUGPR_HIP(hipGetLastError());
  return NUGPR_OK;
}

int nugpr_profile_enable(nugpr_ctx* c, int32_t on) {
  if (!c) { set_error("ctx is null"); return NUGPR_ERR_INVALID; }
  if (on && c->prof_ev.empty()) {
    c->prof_ev.resize(2 * 2048);
    for (size_t i = 0; i < c->prof_ev.size(); ++i) {
      hipError_t e = hipEventCreate(&c->prof_ev[i]);
      if (e != hipSuccess) {
        for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(c->prof_ev[j]);
        c->prof_ev.clear();
        return hip_fail(e, "hipEventCreate");
      }
    }
  }
  c->prof_on = on != 0;
  c->prof_used = 0;
  return NUGPR_OK;
}

int nugpr_profile_read(nugpr_ctx* c, double* total_ms, int32_t* launches, void* stream) {
  if (!c || !total_ms || !launches) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  NUGPR_HIP(hipStreamSynchronize(as_stream(stream)));
  double acc = 0.0;
  for (int i = 0; i < c->prof_used; ++i) {
    float ms = 0.f;
    NUGPR_HIP(hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
    acc += ms;
  }
  *total_ms = acc;
  *launches = c->prof_used;
  c->prof_used = 0;
  return NUGPR_OK;
}

double nugpr_profile_bytes(const nugpr_ctx* c, int32_t ncols) {
  if (!c || ncols < 1) return 0.0;
  const Layout& L = c->L;
  double entries = (double)L.ncr * (double)L.ncr;
  for (const auto& ci : L.cl) entries += (double)ci.b * (double)ci.b;
  const double vs = c->acc64 ? 8.0 : 4.0;
  // reads D and the S slabs, writes Q and the P slabs
  const double vec = vs * ncols * (2.0 * (double)L.n + (double)L.ncr * (L.nsS + L.nsP));
  return 4.0 * entries + vec;
}

int nugpr_profile_kernel_name(const nugpr_ctx* c, int32_t ncols, char* buf, int32_t len) {
  if (!c || !buf || len < 1 || ncols < 1 || ncols > MAX_COLS) { set_error("bad argument"); return NUGPR_ERR_INVALID; }
  const char* name = strip_kernel_name(c->tab_KC, ncols, c->acc64);
  std::strncpy(buf, name, (size_t)len - 1);
  buf[len - 1] = 0;
  return NUGPR_OK;
}

int nugpr_stats_read(nugpr_ctx* c, nugpr_stats* out, int32_t reset) {
  if (!c || !out) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  *out = c->stats;
  if (reset) c->stats = nugpr_stats{};
  return NUGPR_OK;
}

int nugpr_destroy(nugpr_ctx* c) {
  if (!c) return NUGPR_OK;
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  if (c->h_flags) (void)hipHostFree(c->h_flags);
  if (c->h_buf) (void)hipHostFree(c->h_buf);
  delete c;
  return NUGPR_OK;
}

int nugpr_build_blocks(nugpr_ctx* c, const double* theta, void* stream) {
  if (!c) { set_error("ctx is null"); return NUGPR_ERR_INVALID; }
  return launch_build(c, theta, as_stream(stream), !kd_lower_suffices(c));
}

int nugpr_set_nystrom_basis(nugpr_ctx* c, const double* theta, double jitter, void* stream) {
  if (!c) { set_error("ctx is null"); return NUGPR_ERR_INVALID; }
  return launch_nystrom_basis(c, theta, jitter, as_stream(stream));
}

int nugpr_precond_factor(nugpr_ctx* c, double* logdet_M, int32_t* bad_cluster, void* stream) {
  if (!c) { set_error("ctx is null"); return NUGPR_ERR_INVALID; }
  if (!c->built) { set_error("precond_factor needs build_blocks first"); return NUGPR_ERR_STATE; }
  hipStream_t s = as_stream(stream);
  int rc = launch_factor(c, s);
  if (rc) return rc;
  const Layout& L = c->L;
  NUGPR_HIP(hipMemcpyAsync(c->h_buf, c->d_logdet, (size_t)L.nc * sizeof(double), hipMemcpyDeviceToHost, s));
  PcgState* hs = reinterpret_cast<PcgState*>(c->h_buf + L.nc);
  NUGPR_HIP(hipMemcpyAsync(hs, c->d_state, sizeof(PcgState), hipMemcpyDeviceToHost, s));
  NUGPR_HIP(hipStreamSynchronize(s));
  double acc = 0.0;
  for (int i = 0; i < L.nc; ++i) acc += c->h_buf[i];
  c->logdetM = acc;
  if (logdet_M) *logdet_M = acc;
  const bool bad = hs->bad_cluster != std::numeric_limits<int>::max();
  if (bad_cluster) *bad_cluster = bad ? hs->bad_cluster : -1;
  const bool nonfinite = c->assembly_mark != 0 && hs->nonfinite_mark == c->assembly_mark;
  c->factored = !bad && !nonfinite;
  if (nonfinite) return NUGPR_NOT_FINITE;        // NaN / Inf among the coordinates the blocks were assembled from
  return bad ? NUGPR_NOT_PD : NUGPR_OK;
}

static int check_block_args(nugpr_ctx* c, const void* a, const void* b, int ncols) {
  if (!c || !a || !b) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  if (a == b) { set_error("input and output alias"); return NUGPR_ERR_INVALID; }
  if (ncols < 1 || ncols > c->L.T) { set_error("ncols must be 1..n_probes+1"); return NUGPR_ERR_INVALID; }
  return NUGPR_OK;
}

int nugpr_matvec(nugpr_ctx* c, const float* D, float* Q, int32_t ncols, void* stream) {
  int rc = check_block_args(c, D, Q, ncols);
  if (rc) return rc;
  if (!c->built) { set_error("matvec needs build_blocks first"); return NUGPR_ERR_STATE; }
  hipStream_t s = as_stream(stream);
  if (!c->acc64) return run_matvec(c, D, Q, ncols, s);
  // default basis: the projection widens D into the solver's fp64 block while it gathers it, and the expansion
  // writes the fp32 result: three launches (four when the coupling product is summed over column slabs)
  if (c->onehot) return run_matvec(c, c->Dv, c->Qv, ncols, s, nullptr, nullptr, D, Q);
  const int64_t cnt = c->L.n * ncols;
  if ((rc = to_internal(c, D, c->Dv, cnt, s))) return rc;
  if ((rc = run_matvec(c, c->Dv, c->Qv, ncols, s))) return rc;
  return from_internal(c, c->Qv, Q, cnt, s);
}

size_t nugpr_matvec_static_max_bytes(void) { return STATIC_SCRATCH_BYTES; }

int nugpr_matvec_static(nugpr_ctx* c, const float* D, float* Q, int32_t ncols, void* stream) {
  int rc = check_block_args(c, D, Q, ncols);
  if (rc) return rc;
  if (!c->built) { set_error("matvec needs build_blocks first"); return NUGPR_ERR_STATE; }
  const Layout& L = c->L;
  // what nugpr_matvec takes from the context's workspace beyond the stored matrices: the two vector blocks in
  // the solver's own type and the slabs of partial sums of W^T D and C S
  const size_t vs = c->acc64 ? sizeof(double) : sizeof(float);
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  const size_t b_vec = c->acc64 ? up((size_t)L.n * ncols * vs) : 0;
  const size_t b_S = up((size_t)L.nsS * L.ncr * ncols * vs), b_P = up((size_t)L.nsP * L.ncr * ncols * vs);
  const size_t need = 2 * b_vec + b_S + b_P;
  if (need > STATIC_SCRATCH_BYTES) {
    set_error("nugpr_matvec_static: this product needs " + std::to_string(need) + " bytes of scratch, the static "
              "buffer holds " + std::to_string(STATIC_SCRATCH_BYTES) + "; use nugpr_matvec");
    return NUGPR_ERR_WORKSPACE;
  }
  int dev = -1;
  NUGPR_HIP(hipGetDevice(&dev));
  if (dev != c->device) { set_error("the current device is not the one the context was created on"); return NUGPR_ERR_STATE; }
  char* base = static_cast<char*>(g_scratch_ptr[dev]);        // looked up at nugpr_create on this device
  if (!base) { set_error("static scratch address unknown on this device"); return NUGPR_ERR_STATE; }
  // the kernels take their buffers as arguments, as in nugpr_matvec: only the addresses differ.  Nothing in the
  // scratch needs clearing: every slab and block that is read was written by an earlier kernel of this call.
  void *sDv = c->Dv, *sQv = c->Qv, *sS = c->Spart, *sP = c->Ppart;
  c->Dv = base; c->Qv = base + b_vec; c->Spart = base + 2 * b_vec; c->Ppart = base + 2 * b_vec + b_S;
  rc = nugpr_matvec(c, D, Q, ncols, stream);
  c->Dv = sDv; c->Qv = sQv; c->Spart = sS; c->Ppart = sP;
  return rc;
}

int nugpr_split_apply(nugpr_ctx* c, const float* D, float* out, int32_t ncols, void* stream) {
  int rc = check_block_args(c, D, out, ncols);
  if (rc) return rc;
  if (!c->built || !c->factored) { set_error("split_apply needs build_blocks and precond_factor first"); return NUGPR_ERR_STATE; }
  hipStream_t s = as_stream(stream);
  const int64_t cnt = c->L.n * ncols;
  if (!c->acc64) {
    // fp32 blocks are the internal type: stage through R / Q, which the operator does not use
    NUGPR_HIP(hipMemcpyAsync(c->Rv, D, (size_t)cnt * sizeof(float), hipMemcpyDeviceToDevice, s));
    if ((rc = run_split_op(c, c->Rv, c->Qv, ncols, s))) return rc;
    NUGPR_HIP(hipMemcpyAsync(out, c->Qv, (size_t)cnt * sizeof(float), hipMemcpyDeviceToDevice, s));
    return NUGPR_OK;
  }
  if ((rc = to_internal(c, D, c->Rv, cnt, s))) return rc;
  if ((rc = run_split_op(c, c->Rv, c->Qv, ncols, s))) return rc;
  return from_internal(c, c->Qv, out, cnt, s);
}

int nugpr_precond_apply(nugpr_ctx* c, const float* R, float* Z, int32_t ncols, void* stream) {
  int rc = check_block_args(c, R, Z, ncols);
  if (rc) return rc;
  if (!c->factored) { set_error("precond_apply needs precond_factor first"); return NUGPR_ERR_STATE; }
  hipStream_t s = as_stream(stream);
  if (!c->acc64) return run_precond(c, R, Z, ncols, s);
  const int64_t cnt = c->L.n * ncols;
  if ((rc = to_internal(c, R, c->Rv, cnt, s))) return rc;
  if ((rc = run_precond(c, c->Rv, c->Zv, ncols, s))) return rc;
  return from_internal(c, c->Zv, Z, cnt, s);
}

int nugpr_pcg_solve(nugpr_ctx* c, const float* B, float* Xout, int32_t ncols, int32_t* iters, double* alpha,
                    double* beta, void* stream) {
  int rc = check_block_args(c, B, Xout, ncols);
  if (rc) return rc;
  if (!c->built || !c->factored) { set_error("pcg_solve needs build_blocks and precond_factor first"); return NUGPR_ERR_STATE; }
  hipStream_t s = as_stream(stream);
  if (!c->acc64) return run_pcg(c, B, Xout, ncols, iters, alpha, beta, nullptr, s);
  const int64_t cnt = c->L.n * ncols;
  if ((rc = to_internal(c, B, c->Uv, cnt, s))) return rc;
  const int status = run_pcg(c, c->Uv, c->Xv, ncols, iters, alpha, beta, nullptr, s);
  if (status < 0) return status;
  if ((rc = from_internal(c, c->Xv, Xout, cnt, s))) return rc;
  NUGPR_HIP(hipStreamSynchronize(s));
  return status;
}

// statuses after which a loss has no value: negative errors, an indefinite operator, non-finite inputs
static inline bool no_value(int rc) { return rc < 0 || rc == NUGPR_INDEFINITE || rc == NUGPR_NOT_FINITE; }

// The operator of a loss evaluation at theta.  If the stored blocks were assembled with the same
// lengthscales, nothing is assembled: with s = alpha / alpha_0,
//   K_ii(theta) = s K_ii(theta_0) + (sigma^2 - s sigma_0^2) I,   C(theta) = s C(theta_0)
// (eqs. (linear2) and (linear3), stated on the unpreconditioned operator), so the product only
// changes its scale and its diagonal shift.  Both sides of a central difference in alpha or
// sigma^2 then see the SAME rounded entries, and their rounding cancels in the difference.
static int set_operator(nugpr_ctx* c, const double* theta, bool allow_reuse, hipStream_t s) {
  const Layout& L = c->L;
  const int nl = L.p - 2;
  bool same = allow_reuse && c->built && (int)c->theta_built.size() == L.p &&
              !(c->params.flags & NUGPR_NO_SHORTCUTS);
  for (int k = 0; same && k < nl; ++k) same = (theta[k] == c->theta_built[k]);
  if (!same) return launch_build(c, theta, s, !kd_lower_suffices(c));
  for (int i = 0; i < L.p; ++i)
    if (!(theta[i] > 0.0) || !std::isfinite(theta[i])) { set_error("theta entries must be finite and > 0"); return NUGPR_ERR_INVALID; }
  const double a0 = c->theta_built[L.p - 2], s0 = c->theta_built[L.p - 1];
  const double sc = theta[L.p - 2] / a0;
  c->op_scale = sc;
  c->op_shift = sc * (double)c->diag_residual + (theta[L.p - 1] - sc * s0);
  return NUGPR_OK;
}

// The loss with the paper's own log-determinant (Section 3.1): y solved by the left-preconditioned CG
// as one column; Q(A) s_i = z_i by plain batched CG on the split-preconditioned A (eq. (PQ)), then
// z_i^T P(A) s_i = 3 z_i^T (A^2 s_i - s_i), averaged over the probes and completed by log det M (eq. (logdet)).
static int mll_pade(nugpr_ctx* c, nugpr_mll_result* res, hipStream_t s) {
  const Layout& L = c->L;
  const int T = L.T;
  int rc = to_internal(c, c->y, c->x0, L.n, s);               // y as an n x 1 block
  if (rc) return rc;
  PcgExtras ex;
  int mx = 0, mx2 = 0;
  rc = run_pcg(c, c->x0, c->Xv, 1, nullptr, nullptr, nullptr, &mx, s, &ex);
  if (rc < 0) return rc;
  res->max_iters_used = mx;
  res->status = rc;
  if (no_value(rc)) return rc;
  res->quad = ex.bx[0];
  int worst = rc;
  double est = 0.0;
  if (L.t > 0) {
    rc = run_pcg(c, c->Pv, c->Xv, T, nullptr, nullptr, nullptr, &mx2, s, nullptr, PCG_PADE_Q);
    if (rc < 0) return rc;
    res->max_iters_used = std::max(mx, mx2);
    if (no_value(rc)) { res->status = rc; return rc; }
    worst = std::max(worst, rc);
    int rc2;
    if ((rc2 = run_split_op(c, c->Xv, c->Zv, T, s))) return rc2;           // A s
    if ((rc2 = run_split_op(c, c->Zv, c->Qv, T, s))) return rc2;           // A^2 s
    double zaas[MAX_COLS], zs[MAX_COLS];
    if ((rc2 = run_dot2(c, c->Pv, c->Qv, c->Pv, c->Xv, T, zaas, zs, s))) return rc2;
    for (int col = 1; col < T; ++col) est += 3.0 * (zaas[col] - zs[col]);
    est /= L.t;
  }
  res->status = worst;
  res->logdet = c->logdetM + est;
  res->nll = 0.5 * (res->quad + res->logdet + (double)L.n * std::log(2.0 * M_PI));
  return worst;
}

static int mll_impl(nugpr_ctx* c, const double* theta, nugpr_mll_result* res, bool allow_reuse, void* stream) {
  if (!c || !res) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  if (!c->factored) { set_error("mll needs precond_factor first"); return NUGPR_ERR_STATE; }
  hipStream_t s = as_stream(stream);
  const Layout& L = c->L;
  const double nan = std::numeric_limits<double>::quiet_NaN();
  res->nll = res->quad = res->logdet = nan;
  res->logdet_precond = c->logdetM;
  res->max_iters_used = 0;
  res->status = NUGPR_OK;
  if (!theta) { set_error("theta is null"); return NUGPR_ERR_INVALID; }
  int rc = set_operator(c, theta, allow_reuse, s);
  if (rc) return rc;
  if (c->params.flags & NUGPR_LOGDET_PADE) {
    rc = mll_pade(c, res, s);
    if (rc >= 0 && !no_value(rc)) c->stats.loss_evals += 1;
    return rc;
  }
  const int T = L.T, max_iter = c->params.max_iter;
  std::vector<int32_t> iters(T);
  std::vector<double> alpha((size_t)max_iter * T), beta((size_t)max_iter * T);
  int mx = 0;
  PcgExtras ex;
  rc = run_pcg(c, c->Bv, c->Xv, T, iters.data(), alpha.data(), beta.data(), &mx, s, &ex);
  if (rc < 0) return rc;
  res->max_iters_used = mx;
  res->status = rc;
  if (no_value(rc)) return rc;
  res->quad = ex.bx[0];                          // <y, K'^-1 y>: column 0 of B is y
  double est = 0.0;
  for (int col = 1; col < T; ++col) {
    double q = 0.0;
    if (slq_e1_log_e1(alpha.data() + col, beta.data() + col, T, iters[col], &q)) {
      res->status = NUGPR_INDEFINITE;
      return NUGPR_INDEFINITE;
    }
    est += ex.rho0[col] * q;            // rho_0: squared norm of the Lanczos start vector
  }
  res->logdet = c->logdetM + (L.t > 0 ? est / L.t : 0.0);
  res->nll = 0.5 * (res->quad + res->logdet + (double)L.n * std::log(2.0 * M_PI));
  c->stats.loss_evals += 1;
  return rc;
}

int nugpr_mll(nugpr_ctx* c, const double* theta, nugpr_mll_result* res, void* stream) {
  return mll_impl(c, theta, res, false, stream);     // always assembles at theta
}

int nugpr_train_step(nugpr_ctx* c, double* log_theta, double* adam_m, double* adam_v, int64_t* step, double* nll0,
                     double* grad, void* stream) {
  if (!c || !log_theta || !adam_m || !adam_v || !step || !nll0 || !grad) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  const int p = c->L.p;
  const double h = c->params.fd_step;
  std::vector<double> theta(p);
  for (int i = 0; i < p; ++i) {
    if (!std::isfinite(log_theta[i])) { set_error("log_theta is not finite"); return NUGPR_ERR_INVALID; }
    theta[i] = std::exp(log_theta[i]);
  }
  int worst = NUGPR_OK;
  int rc = nugpr_build_blocks(c, theta.data(), stream);
  if (rc) return rc;
  double ldm; int32_t bad;
  rc = nugpr_precond_factor(c, &ldm, &bad, stream);
  if (rc) return rc;
  // The blocks assembled for the factorisation serve the base loss and, through set_operator, the
  // output-scale and noise differences; those come first, before the lengthscale differences
  // overwrite the stored blocks.
  nugpr_mll_result r0;
  rc = mll_impl(c, theta.data(), &r0, true, stream);
  if (no_value(rc)) return rc;
  worst = std::max(worst, rc);
  *nll0 = r0.nll;
  const bool forward = (c->params.flags & NUGPR_FD_FORWARD) != 0;
  // A forward quotient takes both of its losses by the same route, so that what the fp32 factor
  // contributes to each cancels: the split-preconditioned operator of the Pade log-determinant goes
  // through the identity relation on the factored blocks (base loss, alpha, sigma^2) but through the
  // streamed blocks after a lengthscale has changed, and the lengthscale quotients therefore get a base
  // loss of their own, evaluated on the factored blocks by the streamed route.
  nugpr_mll_result r0_general = r0;
  if (forward && (c->params.flags & NUGPR_LOGDET_PADE) && !(c->params.flags & NUGPR_NO_SHORTCUTS)) {
    c->general_route = true;
    rc = mll_impl(c, theta.data(), &r0_general, true, stream);
    c->general_route = false;
    if (no_value(rc)) return rc;
    worst = std::max(worst, rc);
  }
  for (int k = 0; forward && k < p; ++k) {
    // Forward quotient on theta_i, step halved until two consecutive quotients agree (Section 3.1);
    // the gradient with respect to log(theta_i) is theta_i times it.
    const int i = k < 2 ? p - 2 + k : k - 2;          // alpha, sigma^2, then the lengthscales
    const double t0 = theta[i];
    double delta = h * t0, g_prev = 0.0, g = 0.0;
    int halv = 0;
    for (int e = 0; e <= c->params.fd_max_halvings; ++e) {
      if (e > 0) delta *= 0.5;
      nugpr_mll_result r1;
      theta[i] = t0 + delta;
      rc = mll_impl(c, theta.data(), &r1, true, stream);
      theta[i] = t0;
      if (no_value(rc)) return rc;
      worst = std::max(worst, rc);
      g = (r1.nll - (k < 2 ? r0.nll : r0_general.nll)) / delta;
      halv = e;
      if (e > 0 && std::fabs(g - g_prev) <= c->params.fd_threshold * std::fabs(g)) break;
      g_prev = g;
    }
    c->fd_halvings[i] = halv;
    grad[i] = t0 * g;
  }
  // The two assemblies of a lengthscale difference are made in one pass (they share the distance
  // computation); NUGPR_NO_SHORTCUTS and the compensated operator keep one assembly per evaluation.
  const bool pairs = !(c->params.flags & NUGPR_NO_SHORTCUTS) && !c->L.compensate;
  for (int k = 0; !forward && k < p; ++k) {
    const int i = k < 2 ? p - 2 + k : k - 2;          // alpha, sigma^2, then the lengthscales
    nugpr_mll_result rp, rm;
    const double tp = std::exp(log_theta[i] + h), tm = std::exp(log_theta[i] - h);
    const bool pair = pairs && i < p - 2;
    if (pair) {
      rc = launch_build_pair(c, theta.data(), i, h, tp, tm, as_stream(stream), !kd_lower_suffices(c));
      if (rc) return rc;
    }
    theta[i] = tp;
    rc = mll_impl(c, theta.data(), &rp, true, stream);
    if (no_value(rc)) return rc;
    worst = std::max(worst, rc);
    if (pair && (rc = swap_pair(c))) return rc;
    theta[i] = tm;
    rc = mll_impl(c, theta.data(), &rm, true, stream);
    if (no_value(rc)) return rc;
    worst = std::max(worst, rc);
    theta[i] = std::exp(log_theta[i]);
    grad[i] = (rp.nll - rm.nll) / (2.0 * h);
  }
  // Adam (bias corrected), minimising the loss
  const double b1 = c->params.beta1, b2 = c->params.beta2, eps = c->params.eps, lr = c->params.lr;
  *step += 1;
  const double c1 = 1.0 - std::pow(b1, (double)*step), c2 = 1.0 - std::pow(b2, (double)*step);
  for (int i = 0; i < p; ++i) {
    adam_m[i] = b1 * adam_m[i] + (1.0 - b1) * grad[i];
    adam_v[i] = b2 * adam_v[i] + (1.0 - b2) * grad[i] * grad[i];
    const double mh = adam_m[i] / c1, vh = adam_v[i] / c2;
    log_theta[i] -= lr * mh / (std::sqrt(vh) + eps);
  }
  return worst;
}

int nugpr_predict(nugpr_ctx* c, const double* theta, const float* Xtest, int64_t m, double* mean, double* var,
                  int32_t* max_iters_used, void* stream) {
  if (!c || !theta) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  if (m < 0) { set_error("m must be >= 0"); return NUGPR_ERR_INVALID; }
  if (m > 0 && (!Xtest || !mean)) { set_error("Xtest or mean is null"); return NUGPR_ERR_INVALID; }
  if (reinterpret_cast<uintptr_t>(Xtest) & 3u) { set_error("Xtest misaligned"); return NUGPR_ERR_INVALID; }
  if (!c->factored) { set_error("predict needs precond_factor first"); return NUGPR_ERR_STATE; }
  if (max_iters_used) *max_iters_used = 0;
  if (m == 0) return NUGPR_OK;
  hipStream_t s = as_stream(stream);
  int rc = launch_build(c, theta, s);          // validates theta
  if (rc) return rc;
  return run_predict(c, theta, Xtest, m, mean, var, max_iters_used, s);
}

int nugpr_rmse(const double* mean, const double* ytest, int64_t m, double* out) {
  if (!mean || !ytest || !out || m < 1) { set_error("rmse needs m >= 1 and non-null arrays"); return NUGPR_ERR_INVALID; }
  double acc = 0.0;
  for (int64_t j = 0; j < m; ++j) { const double e = mean[j] - ytest[j]; acc += e * e; }
  *out = std::sqrt(acc / (double)m);
  return NUGPR_OK;
}

int nugpr_confidence_band(const double* mean, const double* var, int64_t m, double* lo, double* hi) {
  if (m < 0 || (m > 0 && (!mean || !var || !lo || !hi))) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  for (int64_t j = 0; j < m; ++j) {
    const double sd = std::sqrt(var[j] > 0.0 ? var[j] : 0.0);
    lo[j] = mean[j] - 2.0 * sd;
    hi[j] = mean[j] + 2.0 * sd;
  }
  return NUGPR_OK;
}

int nugpr_compensation_steps(const nugpr_ctx* c, int32_t* out) {
  if (!c || !out) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  if (!c->L.compensate || !c->built) { set_error("no compensated assembly yet"); return NUGPR_ERR_STATE; }
  *out = c->lambda0_steps;
  return NUGPR_OK;
}

int nugpr_compensation_lambda(const nugpr_ctx* c, double* out) {
  if (!c || !out) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  if (!c->L.compensate || !c->built) { set_error("no compensated assembly yet"); return NUGPR_ERR_STATE; }
  *out = c->lambda0;
  return NUGPR_OK;
}

int nugpr_host_smallest_eigenvalue(const double* A, int32_t n, double* out) {
  if (!A || !out || n < 1 || n > 4096) { set_error("smallest_eigenvalue needs a matrix with n = 1..4096"); return NUGPR_ERR_INVALID; }
  std::vector<double> work((size_t)n * n);
  for (int i = 0; i < n; ++i)                      // symmetric copy of the lower triangle
    for (int j = 0; j <= i; ++j) work[(size_t)i * n + j] = work[(size_t)j * n + i] = A[(size_t)i * n + j];
  if (sym_smallest_eigenvalue(work, n, out)) { set_error("eigen-solve did not converge"); return NUGPR_ERR_INVALID; }
  return NUGPR_OK;
}

int nugpr_fd_halvings(const nugpr_ctx* c, int32_t* out) {
  if (!c || !out) { set_error("null argument"); return NUGPR_ERR_INVALID; }
  for (int i = 0; i < c->L.p; ++i) out[i] = c->fd_halvings[i];
  return NUGPR_OK;
}

int nugpr_export(nugpr_ctx* c, int32_t what, int32_t index, float* dst, int64_t ld, void* stream) {
  if (!c) { set_error("ctx is null"); return NUGPR_ERR_INVALID; }
  return launch_export(c, what, index, dst, ld, as_stream(stream));
}

}  // extern "C"
