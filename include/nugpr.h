/*
 * nugpr.h -- C ABI of the MI355X (gfx950) implementation of the nuGPR
 * marginal-log-likelihood hot path (Zhao & Sarin, "nuGPR: GPU-Accelerated
 * Gaussian Process Regression with Iterative Algorithms and Low-Rank
 * Approximations").
 *
 * One evaluation assembles the dense RBF diagonal blocks K_ii of a
 * cluster-structured covariance plus the coupling matrix of the cluster
 * representatives (Section 3.3), runs batched block-Jacobi preconditioned CG
 * (Sections 3.1-3.2) on [y | t probe vectors] with the block-diagonal +
 * low-rank product as inner kernel, recovers Lanczos tridiagonals from the CG
 * coefficients for the stochastic log-determinant of eq. (logdet), and returns
 * the loss of eq. (loss function).  Central differences over the
 * hyperparameters and Adam replace back-propagation (Section 3.1, Algorithm 1).
 *
 * Conventions
 *   - Pointers marked DEVICE are device pointers on the GPU current at
 *     nugpr_create; pointers marked HOST are ordinary host memory.
 *   - The caller owns every buffer, including ONE device workspace of at least
 *     nugpr_workspace_bytes() bytes (256-byte aligned).  The library allocates
 *     no device memory.  It never frees caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     GPU work is enqueued there.  Calls with host outputs return when those
 *     are complete: precond_factor, pcg_solve, predict, export and profile_read
 *     synchronise the stream; mll and train_step wait for the device's own
 *     end-of-solve report in pinned memory (every kernel they enqueued has
 *     finished its work by then; later work on the same stream is ordered
 *     behind it as usual).  build_blocks, matvec, precond_apply, split_apply
 *     and copy_probe only enqueue.
 *   - Return value: 0 = NUGPR_OK; negative = caller / runtime error (nothing
 *     useful was computed); positive = numerical status (outputs are written).
 *     No exception, abort or exit crosses this boundary.
 *   - theta = [ell_1..ell_d, outputscale, noise_variance] on the natural scale
 *     (HOST doubles, all > 0); with NUGPR_ISOTROPIC the layout is
 *     [ell, outputscale, noise_variance], the paper's 3-tuple (Section 2.1).
 *   - Vector blocks (right-hand sides, solutions, search directions) are
 *     row-major n x ncols float arrays (column index fastest), ncols <= 33.
 *   - Points are stored cluster-contiguous: cluster i owns rows
 *     cluster_offsets[i] .. cluster_offsets[i+1]-1 of X, y and every vector block.
 */
#ifndef NUGPR_H
#define NUGPR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nugpr_ctx nugpr_ctx;        /* opaque; host-side bookkeeping only */

enum {
  NUGPR_OK = 0,
  /* caller / runtime errors */
  NUGPR_ERR_INVALID = -1,      /* bad argument (null pointer, sizes, theta <= 0, ...) */
  NUGPR_ERR_WORKSPACE = -2,    /* workspace too small or misaligned */
  NUGPR_ERR_HIP = -3,          /* a HIP runtime call failed; see nugpr_last_error_string */
  NUGPR_ERR_STATE = -4,        /* call order violated (e.g. mll before precond_factor) */
  /* numerical status */
  NUGPR_NOT_PD = 1,            /* a diagonal block failed Cholesky (Section 3.3: not SPD) */
  NUGPR_INDEFINITE = 2,        /* PCG met <d, K'd> <= 0: the approximated K' is not SPD */
  NUGPR_NOT_CONVERGED = 3,     /* max_iter reached before every column met the tolerance */
  NUGPR_NOT_FINITE = 4         /* NaN or Inf in the inputs: among the coordinates (X, representatives), found
                                  when the blocks are assembled and reported by precond_factor and by every
                                  solve on those blocks; or in a right-hand side (e.g. y), found in the first
                                  dot products of the solve, <b, b> and <b, M^-1 b>.  The outputs of the
                                  affected columns are not meaningful and a loss is returned as NaN */
};

enum {
  NUGPR_ISOTROPIC = 1u,        /* one tied lengthscale: theta has 3 entries */
  NUGPR_ACC_FP32 = 2u          /* operator applications on fp32 vector blocks with fp32 matrix-core
                                  accumulation (faster).  Default: fp64 vector blocks and fp64
                                  matrix-core accumulation over the same fp32 stored matrices, which
                                  keeps accumulation rounding out of the finite-difference gradient. */
  ,
  NUGPR_NO_SHORTCUTS = 4u      /* nugpr_train_step assembles the blocks anew for every loss evaluation.
                                  Default: evaluations that differ from the assembled blocks only in the
                                  output scale or the noise reuse them through the linear relations of
                                  Section 3.3 (eqs. (linear2), (linear3)): the operator becomes
                                  s K_0 + shift I with s = alpha / alpha_0 (and their first product is taken
                                  from the base loss's, K' z_0 being linear in s and shift); the two
                                  assemblies of a central difference in a lengthscale are made in one pass
                                  into two sets of blocks. */
  ,
  NUGPR_LOGDET_PADE = 8u       /* log-determinant by the paper's own route (Section 3.1, eqs. (PQ), (logdet)):
                                  Q(A) s_i = z_i by batched CG on A = R^-T K' R^-1 (two applications of A per
                                  iteration), then z_i^T P(A) s_i; y is solved on its own.  While the stored
                                  blocks are the factored ones, A is applied through eqs. (linear1)-(linear3)
                                  without streaming K_diag (unless NUGPR_NO_SHORTCUTS).  Default: stochastic
                                  Lanczos quadrature on the CG coefficients of K' x = L z. */
  ,
  NUGPR_FD_FORWARD = 16u       /* nugpr_train_step takes the paper's own gradient (Section 3.1, the while
                                  loops of Algorithm 1): forward differences on theta_i with the step
                                  fd_step * theta_i halved until two consecutive quotients agree to
                                  fd_threshold (relative) or fd_max_halvings halvings were made; the result
                                  is carried to log(theta) by the chain rule.  Default: central differences. */
  ,
  NUGPR_COMPENSATE = 32u       /* the operator is the compensated K'' = K_diag + W (C - lambda_0 I) W^T of
                                  Section 3.3 (eqs. (krep), (kypp)), positive definite by construction:
                                  C is the full kernel matrix of the representatives (its diagonal blocks
                                  included) and lambda_0 its smallest eigenvalue, computed in fp64 at every
                                  assembly: by a dense symmetric eigen-solve on the host for
                                  n_clusters * rank <= 512 (the paper's regime: n_c <= 20, rank 1), beyond that
                                  by a matrix-free, block-preconditioned eigenvalue iteration on the device
                                  over the assembled matrix, to 2e-11 alpha (default arithmetic mode only).  If
                                  its cap of 150 steps is reached, an estimate below 1e-5 alpha is used as it
                                  stands (lambda_min then lies between 0 and the estimate: a kernel matrix is
                                  positive semi-definite); otherwise the assembly returns NUGPR_ERR_INVALID.
                                  Default: the uncompensated K' of eq. (odsplit). */
  ,
  NUGPR_PRECOND_COMPENSATED = 64u /* with NUGPR_COMPENSATE and the default (one-hot) basis: nugpr_precond_factor
                                  factors the diagonal blocks of K'' itself, K_ii + W_i (C_ii - lambda_0 I) W_i^T
                                  (eq. (kypp); C_ii = kernel matrix of cluster i's own representatives), so that
                                  only the coupling BETWEEN clusters is left to the iteration.  An option beyond
                                  the paper, whose preconditioner is the factor of K_diag for K'' as well
                                  (eq. (precond kypp)): with many points per representative that leaves up to
                                  n_clusters * rank large eigenvalues to CG (133 iterations on the 1 M point
                                  configuration, against a handful with this flag).  The loss is the same
                                  quantity either way (log det M changes with the factor and the estimate of
                                  the remainder with it).  nugpr_precond_factor returns NUGPR_ERR_STATE if the
                                  basis is not the one-hot one (supplied by the caller, or Nystrom weights).
                                  Default: the factor of K_diag. */
};

/* Problem description (Section 2.1 notation; Section 3.3 for representatives). */
typedef struct {
  int64_t n;                       /* training points                                  */
  int32_t d;                       /* input dimension, 1..64                           */
  int32_t n_clusters;              /* n_c                                              */
  int32_t rank;                    /* r representatives per cluster, 1..min cluster size */
  int32_t n_probes;                /* t Hutchinson probe vectors, 0..32                */
  const int64_t* cluster_offsets;  /* HOST, n_clusters+1 ascending, [0]=0, [n_c]=n     */
  const float* X;                  /* DEVICE, n*d row-major                            */
  const float* y;                  /* DEVICE, n                                        */
  const float* reps;               /* DEVICE, n_clusters*rank*d row-major, or NULL =
                                      the first `rank` points of every cluster         */
  const float* W;                  /* DEVICE, n*rank row-major basis (row p belongs to
                                      point p, its cluster's r columns), or NULL =
                                      one-hot nearest representative (plain Euclidean
                                      distance, ties to the lowest index)              */
  const float* probes;             /* DEVICE, n*n_probes row-major, entries +1/-1      */
  void* workspace;                 /* DEVICE, caller-owned, 256-byte aligned           */
  size_t workspace_bytes;
} nugpr_problem;

/* Solver / optimiser parameters. */
typedef struct {
  double tol;          /* PCG stops column c when ||r_c||_2 <= tol * ||b_c||_2         */
  int32_t max_iter;    /* PCG iteration cap, 1..4096                                   */
  double fd_step;      /* h of the central differences on log(theta)                   */
  double lr;           /* Adam learning rate (paper: 0.05)                             */
  double beta1, beta2, eps;  /* Adam moments / epsilon (0 selects 0.9, 0.999, 1e-8)    */
  uint32_t flags;      /* NUGPR_ISOTROPIC | NUGPR_ACC_FP32 | NUGPR_NO_SHORTCUTS |
                          NUGPR_LOGDET_PADE | NUGPR_FD_FORWARD | NUGPR_COMPENSATE |
                          NUGPR_PRECOND_COMPENSATED, or 0 */
  int32_t fd_max_halvings;   /* NUGPR_FD_FORWARD: cap on the halvings per hyperparameter,
                                1..30 (0 selects 8)                                    */
  double fd_threshold; /* NUGPR_FD_FORWARD: stop when |g - g_prev| <= fd_threshold |g|
                          (0 selects 1e-2)                                             */
} nugpr_params;

/* Result of one loss evaluation, eq. (loss function): nll = (quad + logdet + n log 2pi)/2. */
typedef struct {
  double nll;             /* the paper's L (negative log marginal likelihood)          */
  double quad;            /* y^T K'^-1 y                                               */
  double logdet;          /* log det K' estimate, eq. (logdet)                         */
  double logdet_precond;  /* log det of the block-Jacobi preconditioner                */
  int32_t max_iters_used; /* largest per-column PCG iteration count                    */
  int32_t status;         /* NUGPR_OK or a positive numerical status                   */
} nugpr_mll_result;

/* Bytes of device workspace a problem of this shape needs.  Pure host arithmetic;
 * only n, d, n_clusters, rank, n_probes and cluster_offsets are read.  Returns 0 on
 * invalid input. */
size_t nugpr_workspace_bytes(const nugpr_problem* problem);

/* Validates the problem, lays out the workspace and builds the theta-independent
 * pieces on `stream`: representatives (default: first r points per cluster) and the
 * basis W (default: one-hot nearest representative), Section 3.3.  The problem's
 * device buffers must stay alive and unchanged until nugpr_destroy. */
int nugpr_create(nugpr_ctx** ctx, const nugpr_problem* problem, const nugpr_params* params,
                 void* stream);
int nugpr_destroy(nugpr_ctx* ctx);

/* Message of the last negative return on this thread (never NULL). */
const char* nugpr_last_error_string(void);

/* Block assembly at theta (Section 2.1 kernel; K_diag of Section 3.2; K_rep of
 * Section 3.3 generalised to r representatives per cluster):
 *   K_ii[p,q] = alpha exp(-1/2 sum_k ((x_pk - x_qk)/ell_k)^2) + sigma^2 [p = q]
 *   C[(i,a),(j,c)] = alpha exp(-1/2 sum_k ((R_iak - R_jck)/ell_k)^2), i != j (no noise).
 * Overwrites the stored K_diag and C; never touches the preconditioner.  Both are symmetric
 * and the tiles above their diagonals may be left unwritten until an operation needs them
 * (nugpr_export and the products on widths that read whole rows fill them in first). */
int nugpr_build_blocks(nugpr_ctx* ctx, const double* theta /*HOST*/, void* stream);

/* Replaces the basis W by Nystrom weights at theta (Section 3.3 defines the rank-1 block 1 1^T and leaves higher
 * ranks open): W_i = k(X_i, R_i) (k(R_i, R_i) + jitter alpha I)^-1, every point expressed through all r
 * representatives of its cluster by kernel interpolation, in fp64, stored in fp32.  The basis then stays fixed
 * (it does NOT follow later theta, so the loss remains smooth in theta) until the next call; products use the
 * dense-W strips.  jitter = 0 selects 1e-4: the weights of nearby representatives are large and of mixed sign,
 * and whatever they multiply, the fp32 rounding of the stored coupling matrix included, is amplified by their size;
 * 1e-4 keeps them of order 10 at no visible cost in approximation error.  rank <= 128.  The preconditioner must be factored (again)
 * afterwards: nugpr_precond_factor before any solve.  Only enqueues. */
int nugpr_set_nystrom_basis(nugpr_ctx* ctx, const double* theta /*HOST*/, double jitter, void* stream);

/* Block-Jacobi preconditioner, eq. (cholesky factorization): per cluster
 * K_ii = L_i L_i^T (the paper's R_i = L_i^T) from the CURRENT K_diag, the explicit
 * inverses L_i^-1 (the paper applies R^-1 as an explicit inverse, Table 2), and the
 * right-hand sides B = [y | L Z] for the probes Z.  *logdet_M receives
 * log det of the preconditioner; *bad_cluster the first cluster whose block is not
 * positive definite (or -1).  Returns NUGPR_NOT_PD in that case. */
int nugpr_precond_factor(nugpr_ctx* ctx, double* logdet_M /*HOST*/, int32_t* bad_cluster /*HOST*/,
                         void* stream);

/* Q = K' D for ncols columns, K' = blockdiag(K_ii) + W (C - blockdiag(C_ii)) W^T
 * (eq. (odsplit) with the rank-r blocks): the inner kernel of PCG, exposed for the
 * bandwidth metric.  D, Q: DEVICE n x ncols, must not alias. */
int nugpr_matvec(nugpr_ctx* ctx, const float* D, float* Q, int32_t ncols, void* stream);

/* nugpr_matvec for callers that cannot allocate or hand over scratch memory for the call (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, but the blocks the
 * product needs beyond D, Q and the stored matrices (the two vector blocks in the solver's own type, the
 * slabs of partial sums of W^T D and C S) live in a static device buffer inside the library instead of the
 * context's workspace.  That buffer holds nugpr_matvec_static_max_bytes() = 16 MiB per GPU and is kept until
 * the process ends; a product that needs more (about 16 n ncols + 8 (slabs) n_c r ncols bytes in the default
 * mode) is refused with NUGPR_ERR_WORKSPACE.  No hipMalloc / hipFree or allocating routine is called.
 * Every call on a GPU shares that GPU's buffer, which keeps the last call's contents (nothing in it needs to
 * start at zero): calls that overlap on one GPU, on any streams or contexts, race.  The context must have
 * been created on the device that is current.  Does not synchronise. */
int nugpr_matvec_static(nugpr_ctx* ctx, const float* D, float* Q, int32_t ncols, void* stream);
size_t nugpr_matvec_static_max_bytes(void);

/* Z = M^-1 R with M the factored block-Jacobi preconditioner (Section 3.2).
 * R, Z: DEVICE n x ncols, must not alias. */
int nugpr_precond_apply(nugpr_ctx* ctx, const float* R, float* Z, int32_t ncols, void* stream);

/* out = A D with A = R^-T K' R^-1 = L^-1 K' L^-T, the split-preconditioned operator of
 * eq. (RKR) on which the Pade log-determinant works (Section 3.1).  While the stored blocks are
 * the ones the factor was computed from (no nugpr_build_blocks since nugpr_precond_factor), the
 * block-diagonal part is applied as the identity (eq. (linear1)) instead of being streamed,
 * unless NUGPR_NO_SHORTCUTS.  D, out: DEVICE n x ncols row-major fp32, must not alias. */
int nugpr_split_apply(nugpr_ctx* ctx, const float* D, float* out, int32_t ncols, void* stream);

/* Batched PCG (Sections 3.1-3.2): solves K' X = B for ncols columns in lock step
 * from X = 0, preconditioned by the stored factor, until every column meets the
 * tolerance or max_iter.  B, Xout: DEVICE n x ncols.  iters: HOST ncols (iterations
 * each column ran).  alpha, beta: HOST max_iter*ncols row-major CG coefficients
 * (zero past a column's count), or NULL.  Returns NUGPR_OK, NUGPR_INDEFINITE,
 * NUGPR_NOT_CONVERGED or NUGPR_NOT_FINITE (Xout is written in every case). */
int nugpr_pcg_solve(nugpr_ctx* ctx, const float* B, float* Xout, int32_t ncols,
                    int32_t* iters, double* alpha, double* beta, void* stream);

/* One loss evaluation (ComputeLoss of Algorithm 1) at theta with the stored
 * preconditioner, which may have been factored at a different theta (Section 3.2,
 * reuse of R within an epoch): build_blocks(theta), PCG on [y | L Z], quadratic
 * term, SLQ log-determinant, eq. (loss function). */
int nugpr_mll(nugpr_ctx* ctx, const double* theta /*HOST*/, nugpr_mll_result* result /*HOST*/,
              void* stream);

/* One pass of Algorithm 1's loop body on phi = log(theta): assemble and factor at
 * theta_0 = exp(phi), base loss, central differences
 *   g_i = (L(phi + h e_i) - L(phi - h e_i)) / (2h)
 * all with the theta_0 preconditioner and the same probes (the output-scale and noise
 * differences on the theta_0 blocks, see NUGPR_NO_SHORTCUTS), then a bias-corrected
 * Adam update of phi.  With NUGPR_FD_FORWARD the differences are the forward ones with step
 * halving described at that flag.  log_theta, adam_m, adam_v: HOST, p entries, in/out
 * (p = d+2, or 3 with NUGPR_ISOTROPIC); *step in/out; *nll0 and grad (p) out. */
int nugpr_train_step(nugpr_ctx* ctx, double* log_theta, double* adam_m, double* adam_v,
                     int64_t* step, double* nll0, double* grad, void* stream);

/* Posterior prediction (Section 2.1, posterior forward formulae) at theta, with the
 * approximated covariance K' (Section 3.3) in the place of the exact one:
 *   mean_j = <k_j, K'^-1 y>,    var_j = alpha - <k_j, K'^-1 k_j>,
 * k_j the exact kernel between the training points and test point j; alpha is the
 * diagonal of K_** (the latent function's prior variance; add sigma^2 for a noisy
 * observation).  Assembles the blocks at theta and solves with the stored preconditioner:
 * one single-column PCG for y, then, only if var is not NULL, ceil(m / (n_probes+1))
 * batched PCG solves on the cross-covariance columns, which are generated on the device
 * and never stored as a whole.  Xtest: DEVICE m x d row-major fp32, read only, caller
 * keeps ownership.  mean: HOST m doubles.  var: HOST m doubles or NULL (mean only).
 * max_iters_used: HOST, may be NULL.  Synchronises `stream`.  Returns NUGPR_OK,
 * NUGPR_NOT_CONVERGED (some solve hit max_iter; outputs written), NUGPR_INDEFINITE
 * (outputs not complete) or a negative error; m = 0 is a no-op. */
int nugpr_predict(nugpr_ctx* ctx, const double* theta /*HOST*/, const float* Xtest /*DEVICE*/,
                  int64_t m, double* mean /*HOST*/, double* var /*HOST*/, int32_t* max_iters_used,
                  void* stream);

/* Root-mean-square error of a prediction (Section 2.1): sqrt(sum_j (mean_j - ytest_j)^2 / m).
 * All HOST; m >= 1. */
int nugpr_rmse(const double* mean, const double* ytest, int64_t m, double* out);

/* Confidence region of Section 2.1: lo = mean - 2 s, hi = mean + 2 s with
 * s = sqrt(max(var, 0)).  All HOST arrays of m doubles; lo / hi may alias nothing else. */
int nugpr_confidence_band(const double* mean, const double* var, int64_t m, double* lo, double* hi);

/* lambda_0 of eq. (krep) at the last assembly of a NUGPR_COMPENSATE context (HOST double out). */
int nugpr_compensation_lambda(const nugpr_ctx* ctx, double* out /*HOST*/);

/* Steps the device iteration for that lambda_0 took (0: it came from the dense host eigen-solve). */
int nugpr_compensation_steps(const nugpr_ctx* ctx, int32_t* out /*HOST*/);

/* Smallest eigenvalue of a dense symmetric n x n matrix A (HOST, row-major fp64, not modified; only
 * its lower triangle and diagonal are meaningful as a symmetric matrix): the host routine behind
 * lambda_0, Householder tridiagonalisation + QL.  n = 1..4096.  Pure host arithmetic. */
int nugpr_host_smallest_eigenvalue(const double* A /*HOST*/, int32_t n, double* out /*HOST*/);

/* Halvings each hyperparameter's forward difference took in the last nugpr_train_step of a
 * NUGPR_FD_FORWARD context (Section 3.1): out is HOST, p entries; zeros before the first step. */
int nugpr_fd_halvings(const nugpr_ctx* ctx, int32_t* out /*HOST*/);

/* Copies one stored matrix to a dense row-major DEVICE array `dst` with leading
 * dimension `ld` (for verification).  what: 0 = K_ii (b_i x b_i), 1 = L_i lower
 * factor (b_i x b_i, zeros above the diagonal; it shares its storage with the second matrix of a lengthscale
 * pair assembly, so it is available from nugpr_precond_factor until the next nugpr_train_step has assembled
 * such a pair: NUGPR_ERR_STATE afterwards), 2 = L_i^-1 (b_i x b_i), 3 = coupling
 * C with zeroed diagonal blocks, or C - lambda_0 I under NUGPR_COMPENSATE
 * ((n_c r) x (n_c r); index ignored), 4 = W_i (b_i x r),
 * 5 = right-hand sides B (n x (t+1); index ignored), 6 = representatives
 * ((n_c r) x d; index ignored). */
int nugpr_export(nugpr_ctx* ctx, int32_t what, int32_t index, float* dst /*DEVICE*/, int64_t ld,
                 void* stream);

/* Number of hyperparameters p the context expects in theta / log_theta. */
int32_t nugpr_num_hyper(const nugpr_ctx* ctx);

/* Live timing of the dominant kernel (the launch that streams K_diag and C once per
 * product, inside nugpr_matvec and every PCG iteration).  After
 * nugpr_profile_enable(ctx, 1) each such launch is bracketed by HIP events on the stream
 * it runs on (at most 2048 launches are kept; later ones go untimed).
 * nugpr_profile_read synchronises `stream`, returns the summed kernel time in
 * milliseconds and the number of timed launches, and resets the counters.
 * nugpr_profile_bytes returns the bytes one such launch moves at `ncols` columns:
 * the stored matrices it streams (4 * (sum b_i^2 + (n_c r)^2)) plus the vector blocks
 * it reads and writes in the context's arithmetic mode. */
int nugpr_profile_enable(nugpr_ctx* ctx, int32_t on);
int nugpr_profile_read(nugpr_ctx* ctx, double* total_ms /*HOST*/, int32_t* launches /*HOST*/, void* stream);
double nugpr_profile_bytes(const nugpr_ctx* ctx, int32_t ncols);

/* Name of the kernel instantiation behind that launch for vector blocks of `ncols` columns, as profilers print it
 * without the namespace (e.g. "k_strip_ring<1, 32, 4, true, 17>"), copied into buf (HOST, at most len bytes
 * including the terminating zero).  Pure host logic; lets a caller match stored counter readings to the code
 * that is actually running. */
int nugpr_profile_kernel_name(const nugpr_ctx* ctx, int32_t ncols, char* buf /*HOST*/, int32_t len);

/* Work counters of a context since nugpr_create or the last reset (host bookkeeping, no GPU work):
 * what the calls so far did in units of the path's steps (Algorithm 1 / ComputeLoss). */
typedef struct {
  int64_t loss_evals;        /* loss evaluations that returned a value (nugpr_mll, nugpr_train_step)     */
  int64_t pcg_solves;        /* batched PCG solves                                                        */
  int64_t pcg_iterations;    /* iterations summed over the solves (a solve counts its slowest column)     */
  int64_t pcg_iterations_max;/* most iterations any solve took                                            */
  int64_t products;          /* applications of K' that streamed K_diag and C                             */
  int64_t products_reused;   /* applications of K' taken from a kept product through eqs. (linear2), (linear3) */
  int64_t precond_applies;   /* applications of the block-Jacobi preconditioner                           */
  int64_t matrices_assembled;/* sets of blocks (K_diag, C) written by the assembly                        */
  int64_t assembly_passes;   /* assembly passes (a pass over a lengthscale pair writes two sets)          */
  int64_t factorisations;    /* block-Jacobi factorisations                                               */
} nugpr_stats;
int nugpr_stats_read(nugpr_ctx* ctx, nugpr_stats* out /*HOST*/, int32_t reset);

/* A plain device-to-device copy kernel of `bytes` bytes (16-byte loads/stores, both
 * DEVICE pointers 16-byte aligned, bytes a multiple of 16): the known-size dispatch
 * against which hardware HBM byte counters are scaled.  Does not synchronise. */
int nugpr_copy_probe(void* dst /*DEVICE*/, const void* src /*DEVICE*/, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NUGPR_H */
