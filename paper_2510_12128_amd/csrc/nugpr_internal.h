// Internal declarations shared by the HIP translation units of libnugpr.
// gfx950 only; wave64.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "nugpr.h"

namespace nugpr {

constexpr int TILE = 64;        // rows per strip / edge of the square tiles
constexpr int MAX_COLS = 33;    // widest vector block (1 + 32 probes)
constexpr int MAX_D = 64;
constexpr int MAX_ITER_CAP = 4096;
constexpr int COMPENSATE_HOST_MAX = 512;     // lambda_0 of eq. (krep): dense host eigen-solve up to this n_c r, iteration on the device beyond
constexpr double EIGMIN_REL_TOL = 2e-11;     // stopping tolerance of that iteration on lambda_0, relative to alpha
constexpr double EIGMIN_PSD_TOL = 1e-5;      // at its step cap a Ritz value below this (times alpha) is accepted: lambda_min lies in [0, theta]
// doubles of workspace the device iteration needs for a coupling matrix of leading dimension ldc with n rows:
// 24 + 24 basis vectors and their images, residual, new direction, a few scalars, the factors of the 128 x 128 blocks
inline size_t eigmin_workspace_doubles(size_t ldc, size_t n) { return 50 * ldc + 64 + ((n + 127) / 128) * 128 * 128; }

// ---------------------------------------------------------------------------
// per-cluster geometry (device copy lives in the workspace)
// ---------------------------------------------------------------------------
struct ClusterInfo {
  uint64_t koff;    // element offset of this cluster's b x ld block in Kd / Lf / G
  uint64_t wtoff;   // element offset of this cluster's r x ld block in Wt
  uint32_t row0;    // first point of the cluster
  uint32_t b;       // points in the cluster
  uint32_t ld;      // leading dimension of its square blocks: b rounded up to 64
  uint32_t nt;      // number of 64-wide tiles per side: ld / 64
  uint32_t prow;    // first row of the cluster in the padded row numbering (sum of ld of the clusters before it)
  uint32_t pad_;
};

// Work item of the block assembly: tile (tr, tc0) of the lower triangle of one square symmetric
// matrix (a cluster's K_ii or the coupling C), with everything the kernel needs to address it, so
// that no second dependent load follows the descriptor (tc1 = tc0 + 1).
struct BuildItem {
  uint64_t out_off;   // element offset of the matrix in its buffer
  uint32_t prow;      // first row of the matrix in the padded row numbering of the scaled coordinates
  uint32_t total;     // valid rows / columns of the matrix
  uint32_t ld;        // its leading dimension
  uint16_t tr, tc0, tc1, pad_;
  uint32_t pad2_;
};
static_assert(sizeof(BuildItem) == 32, "BuildItem is read as four 8-byte words");

// Storage of the matrices that only the streaming kernels read in bulk (K_diag and the coupling matrix):
// 64-row strips, each cut into blocks of 32 columns stored one after the other (64 x 32 fp32 = 8 KiB).
// Inside a block the order is that of the matrix-core operand fragments: eight fragments of 16 rows x 16
// columns (fragment (w, s) = rows 16 w .., columns 16 s ..), each 1 KiB, row-major inside.  Every memory
// instruction of the kernels that touch these matrices (a wave loading the operand of one 16-column step,
// the assembly storing a 16 x 16 piece of a tile or of its mirror image) then covers ONE contiguous 1 KiB,
// and one pipeline stage of a strip is one contiguous 8 KiB run.  ld is a multiple of 64.
// Element (row, col) of a matrix with leading dimension ld:
constexpr int BLK_COLS = 32;
constexpr int FRAG = 256;                   // floats in a 16 x 16 fragment
__host__ __device__ inline uint64_t blocked_index(uint32_t ld, uint32_t row, uint32_t col) {
  const uint32_t r = row % TILE, c = col % BLK_COLS;
  return (uint64_t)(row / TILE) * TILE * ld + (uint64_t)(col / BLK_COLS) * (TILE * BLK_COLS) +
         (uint64_t)(((r / 16) * 2 + c / 16) * FRAG + (r % 16) * 16 + c % 16);
}

// ---------------------------------------------------------------------------
// strip GEMM work item: out[64 rows] (+)= A[64 rows, c_begin:c_end] * in[c_begin:c_end]
// ---------------------------------------------------------------------------
struct StripItem {
  uint64_t a_off;        // element offset (within the port's matrix) of strip row 0, column 0
  uint32_t lda;
  uint32_t nrows;        // valid rows of the strip, 1..64
  uint32_t c_begin;      // first column, multiple of 64
  uint32_t c_end;        // one past the last valid column
  uint32_t in_row0;      // vector-block row matching column 0
  uint32_t out_row0;     // vector-block row of strip row 0
  uint32_t row_in_block; // index of strip row 0 inside its square block (diagonal position)
  uint16_t out_part;     // which partial-output slab this item writes
  uint8_t port;          // 0 / 1: which (matrix, in, out) triple of the launch
  uint8_t mode;          // 0 full, 1 lower triangle (col <= row), 2 upper triangle (col >= row)
  float diag_add;        // 1 for square diagonal blocks: out += port.diag_add * in[row]; else 0
  uint32_t blocked;      // bit 0: the matrix is stored in blocks of operand fragments (blocked_index), else row-major;
                         // bit 1: full strip of a symmetric square block, upper tiles read as transposed lower ones
};
static_assert(sizeof(StripItem) == 48, "StripItem layout");

struct StripPort {
  const float* A;            // matrix base (always fp32)
  const void* in;            // input vector block(s), fp32 or fp64 by the arithmetic mode
  void* out;                 // output vector block(s), same type
  uint64_t in_part_stride;   // elements between the nin input slabs (summed on load)
  uint64_t out_part_stride;  // elements between output slabs
  int32_t nin;
  int32_t accumulate;        // out += result instead of out = result
  double scale = 1.0;        // the product is multiplied by this before anything is added
  double diag_add = 0.0;     // scalar added on the diagonal of items that ask for it
};

struct StripArgs {
  StripPort port[2];
  const StripItem* items;
  int32_t T;                 // columns of the vector blocks (row stride)
  uint32_t magicT;           // floor(2^32 / T) + 1, for division by T
};

struct StripTable {
  StripItem* dev = nullptr;
  int count = 0;
  bool sym = false;      // some items are strips of symmetric blocks (StripItem::blocked bit 1)
};

// ---------------------------------------------------------------------------
// device-side PCG scalars (all double), one slot per column
// ---------------------------------------------------------------------------
struct PcgState {
  double rho[MAX_COLS];
  double rho0[MAX_COLS];     // <r_0, M^-1 r_0>: squared norm of the Lanczos start vector
  double bnorm2[MAX_COLS];
  double alpha[MAX_COLS];
  double beta[MAX_COLS];
  int32_t active[MAX_COLS];
  int32_t iters[MAX_COLS];
  int32_t converged[MAX_COLS];
  int32_t indef[MAX_COLS];      // column met <d, K'd> <= 0
  int32_t n_active;
  int32_t indefinite;
  int32_t bad_cluster;    // Cholesky: lowest failing cluster index, or INT_MAX
  int32_t tail_count;     // workgroups of the end-of-solve report that are done (returns to 0)
  int32_t check_count;    // workgroups of the stop test that are done (returns to 0)
  int32_t nonfinite_mark; // mark of the last assembly that met NaN / Inf coordinates (nugpr_ctx::assembly_mark)
  // <b, b> and <b, z_0> of the two right-hand-side blocks the context owns ([y | L Z] with z_0 = M^-1 b,
  // and the probe block [0 | Z] with z_0 = b): they depend on the factor only and are taken with it
  double known_bb[2][MAX_COLS];
  double known_rz[2][MAX_COLS];
};

// host-visible mirror (pinned)
struct HostFlags {
  int32_t n_active;
  int32_t indefinite;
  int32_t bad_cluster;
  int32_t pad_;
  // Sequence numbers the device stores AFTER the data they announce (system-scope fence in between):
  // the host polls them in pinned memory instead of paying a stream synchronisation's wake-up latency.
  uint64_t seq;        // the three fields above belong to stop test number `seq`
  uint64_t tail_seq;   // the end-of-solve record in the pinned buffer belongs to report number `tail_seq`
};

struct Layout {
  // geometry
  int64_t n = 0;
  int d = 0, nc = 0, r = 0, t = 0, T = 0, p = 0;
  int ncr = 0, ldc = 0, ldw = 0;
  int ntmax = 0;
  int nsS = 1, nsP = 1;
  bool compensate = false;    // SPD compensation: full coupling matrix minus lambda_0 I, with an fp32 residual matrix
  std::vector<ClusterInfo> cl;
  uint64_t kd_elems = 0, wt_elems = 0;
  uint64_t rows_pad = 0;      // sum of ld over the clusters
  // byte offsets into the workspace
  size_t o_cl = 0, o_Kd = 0, o_G = 0, o_C = 0, o_Wd = 0, o_Wt = 0, o_reps = 0;
  size_t o_Q0 = 0;                   // K' z_0 kept from the base loss
  size_t o_Kd2 = 0, o_C2 = 0;        // spare K_diag and C: second matrix of a pair assembly
  size_t o_B = 0, o_X = 0, o_R = 0, o_Z = 0, o_D = 0, o_Q = 0, o_V = 0, o_U = 0;
  size_t o_Spart = 0, o_Ppart = 0, o_dot = 0, o_state = 0, o_alog = 0, o_blog = 0;
  size_t o_theta = 0, o_logdet = 0, o_tiles = 0, o_items = 0;
  size_t o_Xs = 0, o_Xn = 0, o_Rs = 0, o_Rn = 0;
  size_t o_x0 = 0, o_Z0 = 0, o_P = 0, o_Clo = 0, o_S0 = 0, o_dav = 0;
  size_t o_assign = 0, o_rep_ptr = 0, o_rep_pts = 0;
  size_t items_bytes = 0;
  int n_dot_blocks = 0;
  int max_iter = 0;
  uint64_t n_diag_tiles = 0, n_c_tiles = 0;
  size_t total = 0;
};

}  // namespace nugpr

struct nugpr_ctx {
  nugpr::Layout L;
  nugpr_params params;
  char* ws = nullptr;
  int device = -1;                       // the GPU that was current at nugpr_create
  const float* X = nullptr;
  const float* y = nullptr;
  const float* probes = nullptr;
  // device views into the workspace
  nugpr::ClusterInfo* d_cl = nullptr;
  float *Kd = nullptr, *Lf = nullptr, *G = nullptr, *C = nullptr, *Wd = nullptr, *Wt = nullptr, *reps = nullptr;
  float *Kd2 = nullptr, *C2 = nullptr;     // spare blocks (launch_build_pair / swap_pair)
  // The Cholesky factor L has no storage of its own: the factorisation writes it into the spare K_diag blocks
  // (Lf = Kd2 at that time).  After the factorisation only the inverse factor G is applied; L itself is needed
  // for the right-hand sides B = [y | L Z], formed in the same call, and by nugpr_export.  The next lengthscale
  // pair assembly overwrites it (lf_valid).
  bool lf_valid = false;
  // lengthscale-scaled coordinates in fp64, in MFMA operand order, and their squared norms:
  // of the points (padded row numbering) and of the representatives
  double *Xs = nullptr, *Xn = nullptr, *Rs = nullptr, *Rn = nullptr;
  // vector blocks: fp64 when acc64, else fp32 (sized for fp64 either way)
  void *Bv = nullptr, *Xv = nullptr, *Rv = nullptr, *Zv = nullptr, *Dv = nullptr, *Qv = nullptr, *Vv = nullptr,
       *Uv = nullptr;
  void *Spart = nullptr, *Ppart = nullptr;
  // M^-1 [y | L Z]: the first preconditioned residual of every solve on the context's own right-hand
  // sides; it depends on the factor only, so the factorisation computes it once
  void* Z0v = nullptr;
  void* S0v = nullptr;                   // W^T z_0: the projection the first product of such a solve needs
  bool z0_ready = false;
  // Default (one-hot) basis: W^T D is a sum over each representative's points and W P a gather, so the
  // dense W is not streamed.  assign[p]: row of C / S / P that point p belongs to; rep_ptr / rep_pts: the
  // points of every such row in ascending order (CSR).
  bool onehot = false;
  int32_t *assign = nullptr, *rep_ptr = nullptr, *rep_pts = nullptr;
  void* Pv = nullptr;                    // [0 | Z]: the probes as a vector block (column 0 empty)
  void* x0 = nullptr;                    // K'^-1 y of a prediction call (one column, internal type)
  bool acc64 = true;                     // arithmetic mode of the operator applications
  double *dotpart = nullptr, *alog = nullptr, *blog = nullptr, *d_theta = nullptr, *d_logdet = nullptr;
  nugpr::PcgState* d_state = nullptr;
  uint64_t* d_tiles = nullptr;       // packed (cluster, tile row, tile col) list of the diagonal blocks
  nugpr::BuildItem* d_pan_diag = nullptr;    // work items of the K_ii assembly
  nugpr::BuildItem* d_pan_c = nullptr;       // work items of the coupling assembly
  int n_pan_diag = 0, n_pan_c = 0;
  nugpr::StripTable tab_WtD, tab_KC, tab_C, tab_WP, tab_lowG, tab_upG, tab_lowL;
  // optional event timing of the K_diag / C streaming launch
  bool prof_on = false;
  std::vector<hipEvent_t> prof_ev;       // start/stop pairs
  int prof_used = 0;                     // pairs recorded since the last read
  nugpr::HostFlags* h_flags = nullptr;   // pinned
  uint64_t flag_seq = 0, tail_seq = 0;   // last numbers handed to the device
  int expect_iters[2] = {1, 1};          // iterations the last solve of each system took (when to report early)
  double* h_buf = nullptr;               // pinned scratch for small device->host reads
  size_t h_buf_doubles = 0;
  float diag_residual = 0.f;             // (alpha + sigma^2) - float(alpha + sigma^2) of the stored blocks
  // The stored blocks K_0 were assembled at theta_built.  The operator applied by run_matvec is
  //   op_scale * K_0 + op_shift * I  (shift on the diagonal blocks only; the coupling is scaled),
  // which is the covariance at any theta with the same lengthscales (eqs. (linear2), (linear3)).
  std::vector<double> theta_built;
  std::vector<double> theta_spare;     // theta of the spare blocks after a pair assembly (empty: none)
  double op_scale = 1.0, op_shift = 0.0;
  bool built = false, factored = false;
  // The stored blocks are the very ones the factor was computed from while build_gen == factor_gen:
  // then Y K_diag Y^T = I for the stored K_diag and Y = L^-1 (eq. (linear1)).
  uint64_t build_gen = 0, factor_gen = ~0ull;
  // every assembly pass hands its kernels a fresh non-zero mark; the coordinate-scaling kernel stores it in the
  // device state when it meets a NaN or Inf among the points or representatives (the kernel values of such a
  // point would otherwise quietly come out as zero)
  int32_t assembly_mark = 0;
  // The assembly may leave out the strictly upper tiles of the K_ii (the product's usual launch reads the
  // lower ones only, see k_strip_ring); whoever needs whole strips calls ensure_kd_upper first.
  bool kd_upper_valid = false, spare_upper_valid = false;
  // the same for the coupling matrix, whose strips pair up when c_paired (set with the work tables)
  bool c_upper_valid = false, spare_c_upper_valid = false, c_paired = false;
  // K' z_0 of the factored blocks, kept from the base loss: the output-scale and noise evaluations apply
  // s K_0 + shift I to the same first direction z_0 and get their first product as a combination of Q0v and z_0
  void* Q0v = nullptr;
  uint64_t q0_gen = ~0ull;
  double q0_scale = 1.0, q0_shift = 0.0;
  bool general_route = false;   // take the streamed-K_diag route even where the identity relation holds
  // SPD compensation (eq. (krep)): host copy of the representatives and lambda_0 of the last assembly.
  // Clo holds what fp32 storage of C - lambda_0 I drops: C_exact - lambda_0 I - C_stored, itself in fp32,
  // applied as a second small product so that the compensation term is carried to ~2^-48.
  std::vector<double> h_reps;
  double lambda0 = 0.0;
  int lambda0_steps = 0;                 // steps the device iteration for the last lambda_0 took (0: dense host eigen-solve)
  float* Clo = nullptr;
  double* dav = nullptr;                 // workspace of that iteration (eigmin_workspace_doubles)
  nugpr_stats stats{};                   // work counters (nugpr_stats_read)
  std::vector<int32_t> fd_halvings;      // halvings per hyperparameter in the last forward-difference step
  double logdetM = 0.0;
};

namespace nugpr {

// error plumbing ------------------------------------------------------------
void set_error(const std::string& msg);
const char* last_error_cstr();
int hip_fail(hipError_t e, const char* what);
#define NUGPR_HIP(call)                                         \
  do {                                                          \
    hipError_t e__ = (call);                                    \
    if (e__ != hipSuccess) return ::nugpr::hip_fail(e__, #call); \
  } while (0)

// layout.cpp ----------------------------------------------------------------
int plan_layout(const nugpr_problem* pb, uint32_t flags, Layout& L);

// build_blocks.hip ----------------------------------------------------------
int launch_setup(nugpr_ctx* c, const float* user_reps, const float* user_W, hipStream_t s);
// need_upper = false: the strictly upper tiles of the K_ii are not written (kd_upper_valid records it)
int launch_build(nugpr_ctx* c, const double* theta, hipStream_t s, bool need_upper = true);
// The two assemblies of a central difference in lengthscale `param` (step h on its logarithm) in one pass:
// ell e^{+h} into the blocks in force, ell e^{-h} into the spare ones; swap_pair puts the spare ones in force.
int launch_build_pair(nugpr_ctx* c, const double* theta, int param, double h, double value_plus, double value_minus,
                      hipStream_t s, bool need_upper);
int swap_pair(nugpr_ctx* c);
// true when every product this context launches on its own vector blocks reads lower tiles only
bool kd_lower_suffices(const nugpr_ctx* c);
// fills the strictly upper tiles of the K_ii from the lower ones if the last assembly left them out
int ensure_kd_upper(nugpr_ctx* c, hipStream_t s);
int ensure_c_upper(nugpr_ctx* c, hipStream_t s);
int launch_export(nugpr_ctx* c, int what, int index, float* dst, int64_t ld, hipStream_t s);

// basis.hip ------------------------------------------------------------------
// W_i = k(X_i, R_i) (k(R_i, R_i) + jitter alpha I)^-1 at theta (jitter_rel = 0 selects 1e-4); rank <= 128
int launch_nystrom_basis(nugpr_ctx* c, const double* theta, double jitter_rel, hipStream_t s);

// eigmin.hip -----------------------------------------------------------------
// smallest eigenvalue of the kernel matrix of the representatives at theta: off-diagonal part from (c->C + c->Clo),
// the scalar alpha on the diagonal, diagonal blocks for the preconditioner recomputed from the representatives
int coupling_lambda_min(nugpr_ctx* c, const double* theta, hipStream_t s, double* lambda_out, int* steps_out);
// Chi_ii = float(value), Clo_ii = what that drops
int coupling_set_diag(nugpr_ctx* c, double value, hipStream_t s);

// strip_gemm.hip ------------------------------------------------------------
int launch_strip(const StripTable& tab, const StripPort& p0, const StripPort& p1, int T, bool acc64,
                 hipStream_t s);

// name of the kernel instantiation launch_strip picks for such a table and width (profilers' spelling, no namespace)
const char* strip_kernel_name(const StripTable& tab, int T, bool acc64);

int launch_sum_parts(const void* in, void* out, int64_t count, int parts, uint64_t stride, bool acc64,
                     hipStream_t s);

// factor.hip ----------------------------------------------------------------
int launch_factor(nugpr_ctx* c, hipStream_t s);

// pcg.hip ---------------------------------------------------------------------
// (vector blocks are the context's internal type: fp64 when acc64, else fp32)
// (dq_partial: if not null and the basis is one-hot, the per-workgroup sums of <d, q> per column are left
// there by the product's last kernel, in the layout of the solver's dot products; returns 1 in *dq_done then)
// (D32 / Q32, one-hot basis in fp64 mode only: the block is read from the fp32 array D32, its widened copy
// being left in D by the product's first kernel, and the result is written to the fp32 array Q32 by its last
// one, Q holding the block-diagonal part only: a caller's fp32 blocks then cost no conversion passes)
int run_matvec(nugpr_ctx* c, const void* D, void* Q, int T, hipStream_t s, double* dq_partial = nullptr,
               bool* dq_done = nullptr, const float* D32 = nullptr, float* Q32 = nullptr);
int run_precond(nugpr_ctx* c, const void* R, void* Z, int T, hipStream_t s);
// What a loss evaluation needs besides the solution, fetched with the solve's last synchronisation:
// <b_c, x_c> per column and rho_0 = <r_0, M^-1 r_0>.
// Which system a batched CG run solves.
enum PcgSystem {
  PCG_KPRIME = 0,    // K' x = b, left-preconditioned with the block-Jacobi factor
  PCG_PADE_Q = 1     // Q(A) s = z, A = Y K' Y^T the split-preconditioned operator; no further preconditioner
};
struct PcgExtras {
  double bx[MAX_COLS];
  double rho0[MAX_COLS];
};
int run_pcg(nugpr_ctx* c, const void* B, void* X, int T, int32_t* iters, double* alpha, double* beta,
            int* max_it_used, hipStream_t s, PcgExtras* extras = nullptr, int system = PCG_KPRIME);
// A D = Y K' Y^T D (eq. (RKR)); with the linear relations of eqs. (linear1)-(linear3) when they apply
int run_split_op(nugpr_ctx* c, const void* D, void* out, int T, hipStream_t s);
int run_dot2(nugpr_ctx* c, const void* A0, const void* B0, const void* A1, const void* B1, int T, double* out0,
             double* out1, hipStream_t s);
int store_known_starts(nugpr_ctx* c, hipStream_t s);
int to_internal(nugpr_ctx* c, const float* src, void* dst, int64_t count, hipStream_t s);
int from_internal(nugpr_ctx* c, const void* src, float* dst, int64_t count, hipStream_t s);

// predict.hip ----------------------------------------------------------------
int run_predict(nugpr_ctx* c, const double* theta, const float* Xt, int64_t m, double* mean, double* var,
                int32_t* max_iters_used, hipStream_t s);

// slq.cpp ---------------------------------------------------------------------
// e_1^T log(T) e_1 for the k x k Lanczos matrix built from CG coefficients.
int slq_e1_log_e1(const double* alpha, const double* beta, int stride, int k, double* out);
// Eigenvalues (left in d) of the symmetric tridiagonal matrix with diagonal d (k) and sub-diagonal e (k - 1) by the
// implicit-shift QL iteration, with the first components of the eigenvectors in z; 0 on success.
int tridiag_eigen_first_row(std::vector<double>& d, std::vector<double>& e, std::vector<double>& z);
// Smallest eigenvalue of a dense symmetric n x n matrix (row-major, overwritten); 0 on success.
int sym_smallest_eigenvalue(std::vector<double>& A, int n, double* out);

}  // namespace nugpr
