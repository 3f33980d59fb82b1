"""fp64 CPU oracle for the nuGPR marginal-log-likelihood hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
module; only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do.
It shares no code with the HIP path.  Plain numpy/scipy in float64, written
step by step in the paper's notation so it can be checked against the paper by
eye: no blocking, fusion or reordering beyond what the steps state.

Notation (paper Section 2.1 and 3): n training points in d dimensions, split
into n_c clusters stored contiguously (`offsets`), cluster i holding b_i points;
r representative points per cluster; t Hutchinson probes.
theta = [ell_1..ell_d, alpha, sigma2] (ARD) or [ell, alpha, sigma2] (isotropic,
the paper's 3-tuple (lambda, sigma^2, alpha) in a different order).

What each function follows:
  rbf                 Section 2.1 kernel definition (squared distance, see below)
  diag_blocks         K_diag of Section 3.2 with the noise term of Section 2.1
  default_reps/basis  representative points of Section 3.3 (reading, see below)
  coupling            K_rep of Section 3.3 generalised to r points per cluster
  dense_K/apply_K     the approximated covariance, eq. (odblock)/(odsplit); with a
                      compensation lambda_0 the SPD form of eqs. (krep), (kypp)
  compensation_lambda lambda_0 of eq. (krep); compensation_lambda_iterative: the same number by a
                      block-preconditioned Davidson iteration, for matrices beyond a dense eigen-solve
                      (pinned against the former)
  precond_factor      eq. (cholesky factorization); R_i = L_i^T
  pcg                 batched preconditioned CG, Sections 3.1-3.2
  slq_logdet          eq. (log to trace), (trace estimation), (logdet) with the
                      Lanczos tridiagonal recovered from the CG coefficients
  mll                 eq. (loss function) / ComputeLoss of Algorithm 1
  fd_gradient         eq. (numerical gradient), central form on log theta
  adam_step           Adam update of Algorithm 1
  predict             posterior mean and variance, Section 2.1 "Posterior Forward
                      Formulae", with the approximated covariance in place of K_y
  pade22_log, split_operator, pade_logdet
                      the paper's own log-determinant: eq. (PQ) on the preconditioned
                      operator of eq. (logdet), Q(A) s = z by plain CG
  fd_forward_halving  eq. (numerical gradient) with the step halved until two
                      consecutive quotients agree (Section 3.1, Algorithm 1's while loops)

Readings where the paper is silent or garbled (each is pinned in the tests or
listed as a reading in the design notes):
  * the RBF exponent uses the SQUARED distance (the printed formula drops the
    square);
  * rank-r off-diagonal blocks are K'_ij = W_i C_ij W_j^T with C = k(R, R) the
    kernel matrix of all representatives and W_i a theta-independent b_i x r
    basis (default: one-hot "nearest representative"); at r = 1 this is exactly
    eq. (odblock), at r = b_i with the points as their own representatives it is
    the exact covariance;
  * the uncompensated matrix K' = K_diag + K_offdiag of eq. (odsplit) is the default;
    Problem(compensate=True) switches to the compensated K'' of eq. (kypp), generalised to
    r representatives per cluster as K'' = K_diag + W (C - lambda_0 I) W^T with lambda_0
    the smallest eigenvalue of the full kernel matrix C of all representatives (at r = 1
    this adds k(r_i, r_i) - lambda_0 to every entry of diagonal block i, as printed);
  * the log-determinant uses stochastic Lanczos quadrature on the CG
    coefficients in place of the Pade form, on the preconditioned operator of
    eq. (logdet); probe right-hand sides are b = L z so that left-preconditioned
    CG starts its Lanczos process at z;
  * CG stops per column on the relative recurrence residual
    ||r_c|| <= tol ||b_c||; a stopped column is frozen;
  * forward differences: the initial step is a fraction of the hyperparameter
    (Delta theta_i = rel_step * theta_i) and starts afresh for every gradient; two
    consecutive quotients "agree" when |g - g_prev| <= threshold * |g| (relative: the
    loss scales with n, an absolute threshold would not); after max_halvings
    halvings the last quotient is taken; the gradient is then carried to
    phi = log theta by the chain rule, where Adam acts as everywhere else here;
  * prediction: K_* is the exact kernel between training and test points (the
    paper approximates only the training covariance), K_** its prior variance
    alpha (latent function, no noise term), the solves go through the same
    preconditioned CG as training.

Pins: every function here is pinned by tests/test_oracle_pins.py (dense
Cholesky / slogdet, closed forms, explicit Lanczos, Hadamard-exact traces,
analytic gradients, brute-force loops).  No function is "parity unpinned".
"""
from __future__ import annotations

import numpy as np
from scipy.linalg import cholesky, eigh_tridiagonal, solve_triangular


# --------------------------------------------------------------------------
# hyperparameters
# --------------------------------------------------------------------------
def split_theta(theta, d):
    """theta -> (ell[d], alpha, sigma2).  Length 3 means isotropic (one tied ell)."""
    theta = np.asarray(theta, dtype=np.float64)
    if theta.shape[0] == 3 and d != 1:
        ell = np.full(d, theta[0])
    elif theta.shape[0] == d + 2:
        ell = theta[:d].copy()
    else:
        raise ValueError("theta must have 3 or d+2 entries")
    return ell, float(theta[-2]), float(theta[-1])


# --------------------------------------------------------------------------
# O1: kernel (Section 2.1)
# --------------------------------------------------------------------------
def rbf(XA, XB, ell, alpha):
    """k(x, x') = alpha exp(-1/2 sum_k ((x_k - x'_k)/ell_k)^2), direct differences."""
    XA = np.asarray(XA, dtype=np.float64)
    XB = np.asarray(XB, dtype=np.float64)
    s = np.zeros((XA.shape[0], XB.shape[0]))
    for k in range(XA.shape[1]):
        diff = (XA[:, k][:, None] - XB[:, k][None, :]) / ell[k]
        s += diff * diff
    return alpha * np.exp(-0.5 * s)


# --------------------------------------------------------------------------
# O2: diagonal blocks with noise
# --------------------------------------------------------------------------
def diag_blocks(X, offsets, theta):
    d = X.shape[1]
    ell, alpha, sigma2 = split_theta(theta, d)
    blocks = []
    for i in range(len(offsets) - 1):
        Xi = X[offsets[i]:offsets[i + 1]]
        blocks.append(rbf(Xi, Xi, ell, alpha) + sigma2 * np.eye(Xi.shape[0]))
    return blocks


# --------------------------------------------------------------------------
# O3: representatives and basis (theta independent)
# --------------------------------------------------------------------------
def default_reps(X, offsets, r):
    """First r points of every cluster, in storage order: (n_c*r, d)."""
    return np.concatenate([np.asarray(X[offsets[i]:offsets[i] + r], dtype=np.float64)
                           for i in range(len(offsets) - 1)], axis=0)


def default_basis(X, offsets, reps, r):
    """W_i[p, a] = 1 iff representative a of cluster i is nearest to x_p in the
    plain Euclidean metric (ties to the lowest a).  Returns a list of (b_i, r)."""
    Ws = []
    for i in range(len(offsets) - 1):
        Xi = np.asarray(X[offsets[i]:offsets[i + 1]], dtype=np.float64)
        Ri = reps[i * r:(i + 1) * r]
        d2 = np.zeros((Xi.shape[0], r))
        for k in range(Xi.shape[1]):
            diff = Xi[:, k][:, None] - Ri[:, k][None, :]
            d2 += diff * diff
        a = np.argmin(d2, axis=1)          # first minimum = lowest index on ties
        W = np.zeros((Xi.shape[0], r))
        W[np.arange(Xi.shape[0]), a] = 1.0
        Ws.append(W)
    return Ws


# --------------------------------------------------------------------------
# O4: coupling matrix of the representatives (no noise)
# --------------------------------------------------------------------------
def coupling(reps, theta):
    d = reps.shape[1]
    ell, alpha, _ = split_theta(theta, d)
    return rbf(reps, reps, ell, alpha)


# --------------------------------------------------------------------------
# O5: approximated covariance K' = blockdiag(K_ii) + W (C - blockdiag(C_ii)) W^T
# --------------------------------------------------------------------------
def compensation_lambda(C):
    """lambda_0 of eq. (krep): the smallest eigenvalue of the representatives' kernel matrix."""
    return float(np.linalg.eigvalsh(C)[0])


def compensation_lambda_iterative(C, rel_tol=2e-11, block=128, max_basis=24, keep=3, max_steps=150, psd_tol=1e-5):
    """lambda_0 of eq. (krep) without a dense eigen-solve (the route open to a matrix too large for one):
    generalised Davidson iteration for the smallest eigenvalue.  The low end of the spectrum of a kernel
    matrix of clustered representatives is a dense cluster of small eigenvalues that a plain Krylov process
    resolves only after thousands of steps; those eigenvalues come from within the diagonal blocks, so the
    inverse of a block-diagonal part, T = blockdiag(C_kk + mu I)^-1 with blocks of `block` consecutive indices,
    is the preconditioner.  Steps: Rayleigh-Ritz on an orthonormal basis V (thick restart to `keep` vectors at
    `max_basis`), residual res = C x - theta x, new direction T res orthogonalised against V.  Stop when
    min(|res|, 4 |res|^2 / gap) <= rel_tol * C[0, 0] (gap to the second Ritz value when clearly separate), or
    |theta| <= that tolerance (a kernel matrix is positive semi-definite: lambda_min lies in [0, theta]).
    If max_steps is reached, a theta below psd_tol * C[0, 0] is returned as it stands (same argument: the
    error is at most theta); a larger one raises.  Returns (theta, steps).  Pinned against eigvalsh."""
    n = C.shape[0]
    alpha = abs(C[0, 0])
    tol = rel_tol * alpha
    facs = []
    for k0 in range(0, n, block):
        B = C[k0:k0 + block, k0:k0 + block]
        facs.append(cholesky(B + 1e-10 * alpha * np.eye(B.shape[0]), lower=True))
    idx = np.arange(n, dtype=np.uint64)
    h = (idx * np.uint64(2654435761)) & np.uint64(0xFFFFFFFF)
    h ^= h >> np.uint64(15)
    h = (h * np.uint64(2246822519)) & np.uint64(0xFFFFFFFF)
    h ^= h >> np.uint64(13)
    v = np.where(h & np.uint64(1), 1.0, -1.0) / np.sqrt(n)
    V, AV = [v], [C @ v]
    for step in range(max_steps):
        Vm, AVm = np.array(V).T, np.array(AV).T
        H = Vm.T @ AVm
        ev, Y = np.linalg.eigh(0.5 * (H + H.T))
        if len(V) == max_basis:
            V = [Vm @ Y[:, q] for q in range(keep)]
            AV = [AVm @ Y[:, q] for q in range(keep)]
            Vm, AVm = np.array(V).T, np.array(AV).T
            ev, Y = ev[:keep], np.eye(keep)
        theta, y = ev[0], Y[:, 0]
        res = AVm @ y - theta * (Vm @ y)
        rn = float(np.linalg.norm(res))
        est = rn
        if len(V) > 1 and ev[1] - ev[0] > 10.0 * rn:
            est = min(est, 4.0 * rn * rn / (ev[1] - ev[0]))
        if est <= tol or abs(theta) <= tol:
            return float(theta), step + 1
        t = np.empty(n)
        for k, L in enumerate(facs):
            sl = slice(k * block, min((k + 1) * block, n))
            t[sl] = solve_triangular(L, solve_triangular(L, res[sl], lower=True), lower=True, trans="T")
        for _ in range(2):
            for u in V:
                t -= (u @ t) * u
        nt = float(np.linalg.norm(t))
        if nt <= 1e-300:
            if est <= 1e3 * tol:
                return float(theta), step + 1
            break
        t /= nt
        V.append(t)
        AV.append(C @ t)
    if abs(theta) <= psd_tol * alpha:
        return float(theta), max_steps
    raise ValueError("lambda_0 iteration not converged")


def dense_K(blocks, Ws, C, offsets, r, lam0=None):
    """K' (lam0 None) or the compensated K'' = K_diag + W (C - lam0 I) W^T (eq. (kypp))."""
    n = int(offsets[-1])
    nc = len(blocks)
    K = np.zeros((n, n))
    for i in range(nc):
        si = slice(offsets[i], offsets[i + 1])
        K[si, si] = blocks[i]
        if lam0 is not None:                               # compensation on the diagonal block
            K[si, si] += Ws[i] @ (C[i * r:(i + 1) * r, i * r:(i + 1) * r] - lam0 * np.eye(r)) @ Ws[i].T
        for j in range(nc):
            if j == i:
                continue
            sj = slice(offsets[j], offsets[j + 1])
            K[si, sj] = Ws[i] @ C[i * r:(i + 1) * r, j * r:(j + 1) * r] @ Ws[j].T
    return K


def apply_K(blocks, Ws, C, offsets, r, D, lam0=None):
    """Q = K' D without forming K' (the four sub-steps of the block-low-rank product);
    with lam0 the compensated K'' D: P = (C - lam0 I) S, diagonal blocks of C included."""
    nc = len(blocks)
    T = D.shape[1]
    Q = np.empty_like(D)
    S = np.empty((nc * r, T))
    for j in range(nc):                                   # S_j = W_j^T D_j
        S[j * r:(j + 1) * r] = Ws[j].T @ D[offsets[j]:offsets[j + 1]]
    P = C @ S                                             # P_i = sum_j C_ij S_j ...
    if lam0 is None:
        for i in range(nc):                               # ... minus the j = i term
            P[i * r:(i + 1) * r] -= C[i * r:(i + 1) * r, i * r:(i + 1) * r] @ S[i * r:(i + 1) * r]
    else:
        P -= lam0 * S                                     # ... or all of it, shifted by lambda_0
    for i in range(nc):                                   # Q_i = K_ii D_i + W_i P_i
        si = slice(offsets[i], offsets[i + 1])
        Q[si] = blocks[i] @ D[si] + Ws[i] @ P[i * r:(i + 1) * r]
    return Q


# --------------------------------------------------------------------------
# O6: block-Jacobi preconditioner M = blockdiag(K_ii(theta_0)) = L L^T
# --------------------------------------------------------------------------
def precond_factor(blocks):
    Ls = [cholesky(B, lower=True) for B in blocks]
    logdetM = 2.0 * sum(float(np.sum(np.log(np.diag(L)))) for L in Ls)
    return Ls, logdetM


def precond_apply(Ls, offsets, R):
    Z = np.empty_like(R)
    for i, L in enumerate(Ls):
        si = slice(offsets[i], offsets[i + 1])
        v = solve_triangular(L, R[si], lower=True)
        Z[si] = solve_triangular(L, v, lower=True, trans="T")
    return Z


# --------------------------------------------------------------------------
# O7: right-hand sides B = [ y | L Z ]
# --------------------------------------------------------------------------
def rhs(y, Ls, offsets, probes):
    n = y.shape[0]
    t = probes.shape[1]
    B = np.empty((n, t + 1))
    B[:, 0] = y
    for i, L in enumerate(Ls):
        si = slice(offsets[i], offsets[i + 1])
        B[si, 1:] = L @ np.asarray(probes[si], dtype=np.float64)
    return B


# --------------------------------------------------------------------------
# O8: batched preconditioned CG
# --------------------------------------------------------------------------
def pcg(apply_op, apply_prec, B, tol, max_iter):
    """Solve K' X = B column by column in lock step.

    Returns X, iters[c] (iterations column c ran), alphas, betas
    (max_iter x T arrays; entries past a column's count are zero) and
    converged[c].  Raises ValueError("indefinite") when <d, K'd> <= 0."""
    n, T = B.shape
    X = np.zeros((n, T))
    R = B.copy()
    Zt = apply_prec(R)
    D = Zt.copy()
    rho = np.sum(R * Zt, axis=0)
    bnorm = np.sqrt(np.sum(B * B, axis=0))
    active = np.ones(T, dtype=bool)
    done0 = bnorm == 0.0                       # zero right-hand side: solution 0
    active[done0] = False
    iters = np.zeros(T, dtype=np.int64)
    conv = done0.copy()
    alphas = np.zeros((max_iter, T))
    betas = np.zeros((max_iter, T))
    for j in range(max_iter):
        if not active.any():
            break
        Q = apply_op(D)
        dq = np.sum(D * Q, axis=0)
        if np.any(dq[active] <= 0.0):
            raise ValueError("indefinite")
        alpha = np.where(active, rho / np.where(active, dq, 1.0), 0.0)
        X += D * alpha
        R -= Q * alpha
        alphas[j] = alpha
        iters[active] = j + 1
        rnorm = np.sqrt(np.sum(R * R, axis=0))
        newly = active & (rnorm <= tol * bnorm)
        conv |= newly
        active = active & ~newly
        Zt = apply_prec(R)
        rho_new = np.sum(R * Zt, axis=0)
        beta = np.where(active, rho_new / np.where(active, rho, 1.0), 0.0)
        betas[j] = beta
        D = Zt + D * beta
        D[:, ~active] = 0.0
        rho = np.where(active, rho_new, rho)
    return X, iters, alphas, betas, conv


# --------------------------------------------------------------------------
# O10: Lanczos tridiagonal from CG coefficients, and the SLQ log-determinant
# --------------------------------------------------------------------------
def lanczos_tridiagonal(alpha_c, beta_c, k):
    """Diagonal and off-diagonal of the k x k Lanczos matrix of the
    preconditioned operator, from one column's CG coefficients."""
    diag = np.empty(k)
    off = np.empty(max(k - 1, 0))
    diag[0] = 1.0 / alpha_c[0]
    for j in range(1, k):
        diag[j] = 1.0 / alpha_c[j] + beta_c[j - 1] / alpha_c[j - 1]
        off[j - 1] = np.sqrt(beta_c[j - 1]) / alpha_c[j - 1]
    return diag, off


def slq_quadrature(alpha_c, beta_c, k, norm2):
    """norm2 * e_1^T log(T) e_1: Gauss quadrature for z^T log(A_hat) z, |z|^2 = norm2."""
    diag, off = lanczos_tridiagonal(alpha_c, beta_c, k)
    if k == 1:
        return norm2 * np.log(diag[0])
    lam, Qm = eigh_tridiagonal(diag, off)
    return norm2 * float(np.sum(Qm[0, :] ** 2 * np.log(lam)))


def slq_logdet(alphas, betas, iters, n, logdetM, probe_cols):
    """log det K' ~= log det M + (1/t) sum_c n e_1^T log(T_c) e_1  (eq. (logdet))."""
    est = [slq_quadrature(alphas[:, c], betas[:, c], int(iters[c]), float(n)) for c in probe_cols]
    return logdetM + float(np.mean(est)), np.asarray(est)


# --------------------------------------------------------------------------
# the model state the oracle carries between steps
# --------------------------------------------------------------------------
class Problem:
    """Inputs widened to float64 plus the theta-independent pieces (reps, W)."""

    def __init__(self, X, y, offsets, probes, rank, reps=None, Ws=None, compensate=False):
        self.compensate = bool(compensate)
        self.X = np.asarray(X, dtype=np.float64)
        self.y = np.asarray(y, dtype=np.float64)
        self.offsets = np.asarray(offsets, dtype=np.int64)
        self.probes = np.asarray(probes, dtype=np.float64)
        self.r = int(rank)
        self.n = self.X.shape[0]
        self.d = self.X.shape[1]
        self.nc = self.offsets.shape[0] - 1
        self.reps = default_reps(self.X, self.offsets, self.r) if reps is None \
            else np.asarray(reps, dtype=np.float64)
        self.Ws = default_basis(self.X, self.offsets, self.reps, self.r) if Ws is None \
            else [np.asarray(W, dtype=np.float64) for W in Ws]

    def assemble(self, theta):
        """O2 + O4 at theta: (list of K_ii, C)."""
        return diag_blocks(self.X, self.offsets, theta), coupling(self.reps, theta)

    def operator(self, theta):
        blocks, C = self.assemble(theta)
        lam0 = compensation_lambda(C) if self.compensate else None
        return lambda D: apply_K(blocks, self.Ws, C, self.offsets, self.r, D, lam0)

    def dense(self, theta):
        blocks, C = self.assemble(theta)
        lam0 = compensation_lambda(C) if self.compensate else None
        return dense_K(blocks, self.Ws, C, self.offsets, self.r, lam0)


class Factor:
    """O6/O7 at the factor point theta_0: L, log det M, and B = [y | L Z].

    compensated_blocks = False: the paper's preconditioner, the factor of K_diag (Section 3.2; Algorithm 1 and
    eq. (precond kypp) use it for the compensated matrix as well).
    compensated_blocks = True (an option beyond the paper, for Problem(compensate=True)): the factor of the
    diagonal blocks of the compensated matrix itself.  K'' of eq. (kypp) has the diagonal blocks
    K_ii + W_i (C_ii - lambda_0 I) W_i^T, C_ii the kernel matrix of cluster i's own representatives; only the
    coupling BETWEEN clusters is then left to the iteration."""

    def __init__(self, prob: Problem, theta0, compensated_blocks=False):
        blocks = diag_blocks(prob.X, prob.offsets, theta0)
        if compensated_blocks:
            C = coupling(prob.reps, theta0)
            lam0 = compensation_lambda(C)
            r = prob.r
            blocks = [B + W @ (C[i * r:(i + 1) * r, i * r:(i + 1) * r] - lam0 * np.eye(r)) @ W.T
                      for i, (B, W) in enumerate(zip(blocks, prob.Ws))]
        self.Ls, self.logdetM = precond_factor(blocks)
        self.B = rhs(prob.y, self.Ls, prob.offsets, prob.probes)
        self.offsets = prob.offsets

    def apply(self, R):
        return precond_apply(self.Ls, self.offsets, R)


# --------------------------------------------------------------------------
# O9, O11: the loss (eq. (loss function))
# --------------------------------------------------------------------------
def mll(prob: Problem, fac: Factor, theta, tol, max_iter, logdet="slq"):
    """Negative marginal log likelihood L(theta) with the theta_0 preconditioner.

    logdet = "slq": Lanczos quadrature on the CG coefficients of the probe columns;
    logdet = "pade": the paper's eq. (PQ) route (pade_logdet), y solved on its own.
    Returns dict(nll, quad, logdet, logdet_precond, iters, X, est)."""
    op = prob.operator(theta)
    if logdet == "pade":
        X, iters, _, _, conv = pcg(op, fac.apply, prob.y[:, None].copy(), tol, max_iter)
        quad = float(prob.y @ X[:, 0])
        ld, est, it2 = pade_logdet(prob, fac, theta, tol, max_iter)
        nll = 0.5 * (quad + ld + prob.n * np.log(2.0 * np.pi))
        return dict(nll=nll, quad=quad, logdet=ld, logdet_precond=fac.logdetM,
                    iters=np.concatenate([iters, it2]), X=X, est=est, converged=conv)
    if logdet != "slq":
        raise ValueError(logdet)
    X, iters, alphas, betas, conv = pcg(op, fac.apply, fac.B, tol, max_iter)
    quad = float(prob.y @ X[:, 0])
    t = prob.probes.shape[1]
    logdet, est = slq_logdet(alphas, betas, iters, prob.n, fac.logdetM, range(1, t + 1))
    nll = 0.5 * (quad + logdet + prob.n * np.log(2.0 * np.pi))
    return dict(nll=nll, quad=quad, logdet=logdet, logdet_precond=fac.logdetM,
                iters=iters, X=X, est=est, converged=conv, alphas=alphas, betas=betas)


# --------------------------------------------------------------------------
# The paper's own log-determinant: 2-2 Pade form of the logarithm, eq. (PQ),
# on the preconditioned operator of eq. (logdet)
# --------------------------------------------------------------------------
def pade22_log(x):
    """P(x) / Q(x) of eq. (PQ): (3 x^2 - 3) / (x^2 + 4 x + 1)."""
    return (3.0 * x * x - 3.0) / (x * x + 4.0 * x + 1.0)


def split_operator(apply_op, Ls, offsets):
    """D -> R^-T K' R^-1 D with R = blockdiag(L_i^T), i.e. L^-1 K' L^-T D (eq. (RKR))."""
    def apply(D):
        U = np.empty_like(D)
        for i, L in enumerate(Ls):
            si = slice(offsets[i], offsets[i + 1])
            U[si] = solve_triangular(L, D[si], lower=True, trans="T")       # R^-1 D
        V = apply_op(U)
        out = np.empty_like(D)
        for i, L in enumerate(Ls):
            si = slice(offsets[i], offsets[i + 1])
            out[si] = solve_triangular(L, V[si], lower=True)                # R^-T (.)
        return out
    return apply


def pade_logdet(prob: Problem, fac: Factor, theta, tol, max_iter):
    """log|K'| = 2 sum log|R_i| + (1/t) sum_i z_i^T P(A) Q(A)^-1 z_i, A = R^-T K' R^-1
    (eqs. (logdet), (PQ)): Q(A) s_i = z_i by batched CG without a further
    preconditioner (A is the preconditioned system), then P(A) s_i and the dot with z_i.
    Returns (logdet, per-probe estimates, CG iteration counts)."""
    A = split_operator(prob.operator(theta), fac.Ls, prob.offsets)
    Z = np.asarray(prob.probes, dtype=np.float64)

    def Qop(D):
        AD = A(D)
        return A(AD) + 4.0 * AD + D

    S, iters, _, _, _ = pcg(Qop, lambda R: R.copy(), Z, tol, max_iter)
    PS = 3.0 * (A(A(S)) - S)
    est = np.sum(Z * PS, axis=0)
    return fac.logdetM + float(np.mean(est)), est, iters


# --------------------------------------------------------------------------
# O12: central finite differences on phi = log theta
# --------------------------------------------------------------------------
def fd_gradient(prob: Problem, fac: Factor, log_theta, h, tol, max_iter):
    log_theta = np.asarray(log_theta, dtype=np.float64)
    g = np.empty_like(log_theta)
    for i in range(log_theta.shape[0]):
        e = np.zeros_like(log_theta)
        e[i] = h
        lp = mll(prob, fac, np.exp(log_theta + e), tol, max_iter)["nll"]
        lm = mll(prob, fac, np.exp(log_theta - e), tol, max_iter)["nll"]
        g[i] = (lp - lm) / (2.0 * h)
    return g


# --------------------------------------------------------------------------
# O13: Adam (bias corrected) on phi, minimising L
# --------------------------------------------------------------------------
def adam_step(phi, g, m, v, step, lr=0.05, beta1=0.9, beta2=0.999, eps=1e-8):
    step = step + 1
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    phi = phi - lr * mhat / (np.sqrt(vhat) + eps)
    return phi, m, v, step


def train_step(prob: Problem, log_theta, m, v, step, h, tol, max_iter, lr=0.05,
               beta1=0.9, beta2=0.999, eps=1e-8):
    """One pass of Algorithm 1's loop body: factor at theta_0, base loss,
    gradient by differences with the same factor and probes, Adam update."""
    theta0 = np.exp(log_theta)
    fac = Factor(prob, theta0)
    nll0 = mll(prob, fac, theta0, tol, max_iter)["nll"]
    g = fd_gradient(prob, fac, log_theta, h, tol, max_iter)
    phi, m, v, step = adam_step(np.asarray(log_theta, dtype=np.float64), g, m, v, step,
                                lr, beta1, beta2, eps)
    return phi, m, v, step, nll0, g


# --------------------------------------------------------------------------
# The paper's own gradient: forward differences whose step is halved until two
# consecutive quotients agree (Section 3.1; the while loops of Algorithm 1)
# --------------------------------------------------------------------------
def fd_forward_halving(loss, theta, L0, rel_step, threshold, max_halvings):
    """g_i = (L(theta + Delta e_i) - L0) / Delta on the raw hyperparameters.

    Delta starts at rel_step * theta_i; it is halved and the quotient recomputed until
    |g - g_prev| <= threshold * |g| or max_halvings halvings were made (at least one
    halving always happens: the first quotient has nothing to be compared with).
    Returns (g, halvings[i])."""
    theta = np.asarray(theta, dtype=np.float64)
    g = np.empty_like(theta)
    halvings = np.zeros(theta.shape[0], dtype=np.int64)
    for i in range(theta.shape[0]):
        delta = rel_step * theta[i]
        tp = theta.copy()
        tp[i] = theta[i] + delta
        g_prev = (loss(tp) - L0) / delta
        gi = g_prev
        for k in range(max_halvings):
            delta *= 0.5
            tp[i] = theta[i] + delta
            gi = (loss(tp) - L0) / delta
            halvings[i] = k + 1
            if abs(gi - g_prev) <= threshold * abs(gi):
                break
            g_prev = gi
        g[i] = gi
    return g, halvings


def train_step_forward(prob: Problem, log_theta, m, v, step, rel_step, threshold, max_halvings,
                       tol, max_iter, lr=0.05, beta1=0.9, beta2=0.999, eps=1e-8, logdet="slq"):
    """Algorithm 1's loop body with its own gradient: factor at theta_0, base loss,
    forward differences with halving on theta, chain rule to phi = log theta, Adam."""
    theta0 = np.exp(np.asarray(log_theta, dtype=np.float64))
    fac = Factor(prob, theta0)
    loss = lambda th: mll(prob, fac, th, tol, max_iter, logdet=logdet)["nll"]
    nll0 = loss(theta0)
    g_theta, halvings = fd_forward_halving(loss, theta0, nll0, rel_step, threshold, max_halvings)
    g = theta0 * g_theta
    phi, m, v, step = adam_step(np.asarray(log_theta, dtype=np.float64), g, m, v, step,
                                lr, beta1, beta2, eps)
    return phi, m, v, step, nll0, g, halvings


# --------------------------------------------------------------------------
# posterior prediction (Section 2.1, "Posterior Forward Formulae")
# --------------------------------------------------------------------------
def predict(prob: Problem, fac: Factor, theta, Xtest, tol, max_iter, variance=True):
    """mu = K_*^T K'^-1 y and s^2 = diag(K_** - K_*^T K'^-1 K_*) at the test points.

    K' = the approximated training covariance at theta, K_* = k(X_train, X_test)
    exactly, K_** = k(x, x) = alpha.  Every solve is a preconditioned CG run with
    the factor `fac` (columns: y, then the columns of K_*).
    Returns dict(mean[m], var[m] or None, iters)."""
    Xtest = np.asarray(Xtest, dtype=np.float64)
    ell, alpha, _ = split_theta(theta, prob.d)
    Ks = rbf(prob.X, Xtest, ell, alpha)                      # n x m
    op = prob.operator(theta)
    B = np.concatenate([prob.y[:, None], Ks], axis=1) if variance else prob.y[:, None].copy()
    X, iters, _, _, _ = pcg(op, fac.apply, B, tol, max_iter)
    mean = Ks.T @ X[:, 0]
    var = None
    if variance:
        var = alpha - np.einsum("ij,ij->j", Ks, X[:, 1:])
    return dict(mean=mean, var=var, iters=iters)


def rmse(mean, ytest):
    """Root mean squared error of the predictive mean (the usual definition; the paper's
    printed formula takes the root of the 2-norm)."""
    mean = np.asarray(mean, dtype=np.float64)
    ytest = np.asarray(ytest, dtype=np.float64)
    return float(np.sqrt(np.mean((mean - ytest) ** 2)))
