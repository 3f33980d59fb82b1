"""ctypes binding of libnugpr.so: same entry points as include/nugpr.h, argument
marshalling only.  PyTorch supplies device memory and the stream; every step of the
path runs in the library's HIP kernels.  There is no CPU or PyTorch fallback: if the
library is missing, loading raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

NUGPR_OK = 0
NUGPR_ERR_INVALID = -1
NUGPR_ERR_WORKSPACE = -2
NUGPR_ERR_HIP = -3
NUGPR_ERR_STATE = -4
NUGPR_NOT_PD = 1
NUGPR_INDEFINITE = 2
NUGPR_NOT_CONVERGED = 3
NUGPR_NOT_FINITE = 4
NUGPR_ISOTROPIC = 1
NUGPR_ACC_FP32 = 2
NUGPR_NO_SHORTCUTS = 4
NUGPR_LOGDET_PADE = 8
NUGPR_FD_FORWARD = 16
NUGPR_COMPENSATE = 32
NUGPR_PRECOND_COMPENSATED = 64

EXPORT_K, EXPORT_L, EXPORT_LINV, EXPORT_C, EXPORT_W, EXPORT_B, EXPORT_REPS = range(7)


class NugprError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"nugpr error {code}: {msg}")
        self.code = code


class Problem(C.Structure):
    _fields_ = [("n", C.c_int64), ("d", C.c_int32), ("n_clusters", C.c_int32), ("rank", C.c_int32),
                ("n_probes", C.c_int32), ("cluster_offsets", C.POINTER(C.c_int64)),
                ("X", C.c_void_p), ("y", C.c_void_p), ("reps", C.c_void_p), ("W", C.c_void_p),
                ("probes", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class Params(C.Structure):
    _fields_ = [("tol", C.c_double), ("max_iter", C.c_int32), ("fd_step", C.c_double), ("lr", C.c_double),
                ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double), ("flags", C.c_uint32),
                ("fd_max_halvings", C.c_int32), ("fd_threshold", C.c_double)]


class MllResult(C.Structure):
    _fields_ = [("nll", C.c_double), ("quad", C.c_double), ("logdet", C.c_double),
                ("logdet_precond", C.c_double), ("max_iters_used", C.c_int32), ("status", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [(k, C.c_int64) for k in ("loss_evals", "pcg_solves", "pcg_iterations", "pcg_iterations_max",
                                          "products", "products_reused", "precond_applies",
                                          "matrices_assembled", "assembly_passes", "factorisations")]


_LIB = None


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libnugpr.so")


def load_library():
    """Loads libnugpr.so.  Raises if it has not been built (no fallback exists)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2510_12128_amd.build` "
                           "(or __graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(path)
    dp, ip, vp = C.POINTER(C.c_double), C.POINTER(C.c_int32), C.c_void_p
    lib.nugpr_workspace_bytes.restype = C.c_size_t
    lib.nugpr_workspace_bytes.argtypes = [C.POINTER(Problem)]
    lib.nugpr_create.restype = C.c_int
    lib.nugpr_create.argtypes = [C.POINTER(vp), C.POINTER(Problem), C.POINTER(Params), vp]
    lib.nugpr_destroy.restype = C.c_int
    lib.nugpr_destroy.argtypes = [vp]
    lib.nugpr_last_error_string.restype = C.c_char_p
    lib.nugpr_last_error_string.argtypes = []
    lib.nugpr_build_blocks.restype = C.c_int
    lib.nugpr_build_blocks.argtypes = [vp, dp, vp]
    lib.nugpr_set_nystrom_basis.restype = C.c_int
    lib.nugpr_set_nystrom_basis.argtypes = [vp, dp, C.c_double, vp]
    lib.nugpr_precond_factor.restype = C.c_int
    lib.nugpr_precond_factor.argtypes = [vp, dp, ip, vp]
    lib.nugpr_matvec.restype = C.c_int
    lib.nugpr_matvec.argtypes = [vp, vp, vp, C.c_int32, vp]
    lib.nugpr_matvec_static.restype = C.c_int
    lib.nugpr_matvec_static.argtypes = [vp, vp, vp, C.c_int32, vp]
    lib.nugpr_matvec_static_max_bytes.restype = C.c_size_t
    lib.nugpr_matvec_static_max_bytes.argtypes = []
    lib.nugpr_split_apply.restype = C.c_int
    lib.nugpr_split_apply.argtypes = [vp, vp, vp, C.c_int32, vp]
    lib.nugpr_precond_apply.restype = C.c_int
    lib.nugpr_precond_apply.argtypes = [vp, vp, vp, C.c_int32, vp]
    lib.nugpr_pcg_solve.restype = C.c_int
    lib.nugpr_pcg_solve.argtypes = [vp, vp, vp, C.c_int32, ip, dp, dp, vp]
    lib.nugpr_mll.restype = C.c_int
    lib.nugpr_mll.argtypes = [vp, dp, C.POINTER(MllResult), vp]
    lib.nugpr_train_step.restype = C.c_int
    lib.nugpr_train_step.argtypes = [vp, dp, dp, dp, C.POINTER(C.c_int64), dp, dp, vp]
    lib.nugpr_predict.restype = C.c_int
    lib.nugpr_predict.argtypes = [vp, dp, vp, C.c_int64, dp, dp, ip, vp]
    lib.nugpr_rmse.restype = C.c_int
    lib.nugpr_rmse.argtypes = [dp, dp, C.c_int64, dp]
    lib.nugpr_confidence_band.restype = C.c_int
    lib.nugpr_confidence_band.argtypes = [dp, dp, C.c_int64, dp, dp]
    lib.nugpr_compensation_lambda.restype = C.c_int
    lib.nugpr_compensation_lambda.argtypes = [vp, dp]
    lib.nugpr_compensation_steps.restype = C.c_int
    lib.nugpr_compensation_steps.argtypes = [vp, ip]
    lib.nugpr_host_smallest_eigenvalue.restype = C.c_int
    lib.nugpr_host_smallest_eigenvalue.argtypes = [dp, C.c_int32, dp]
    lib.nugpr_fd_halvings.restype = C.c_int
    lib.nugpr_fd_halvings.argtypes = [vp, ip]
    lib.nugpr_export.restype = C.c_int
    lib.nugpr_export.argtypes = [vp, C.c_int32, C.c_int32, vp, C.c_int64, vp]
    lib.nugpr_num_hyper.restype = C.c_int32
    lib.nugpr_num_hyper.argtypes = [vp]
    lib.nugpr_profile_enable.restype = C.c_int
    lib.nugpr_profile_enable.argtypes = [vp, C.c_int32]
    lib.nugpr_profile_read.restype = C.c_int
    lib.nugpr_profile_read.argtypes = [vp, dp, ip, vp]
    lib.nugpr_profile_bytes.restype = C.c_double
    lib.nugpr_profile_bytes.argtypes = [vp, C.c_int32]
    lib.nugpr_profile_kernel_name.restype = C.c_int
    lib.nugpr_profile_kernel_name.argtypes = [vp, C.c_int32, C.c_char_p, C.c_int32]
    lib.nugpr_stats_read.restype = C.c_int
    lib.nugpr_stats_read.argtypes = [vp, C.POINTER(Stats), C.c_int32]
    lib.nugpr_copy_probe.restype = C.c_int
    lib.nugpr_copy_probe.argtypes = [vp, vp, C.c_size_t, vp]
    _LIB = lib
    return lib


def _dptr(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _check(code):
    if code < 0:
        raise NugprError(code, load_library().nugpr_last_error_string().decode())
    return code


def nugpr_copy_probe(dst, src, stream=None):
    """Plain copy kernel between two equally sized CUDA tensors (counter calibration)."""
    import torch
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    st = C.c_void_p(torch.cuda.current_stream(src.device).cuda_stream if stream is None else stream)
    return _check(lib.nugpr_copy_probe(dst.data_ptr(), src.data_ptr(), nbytes, st))


def nugpr_rmse(mean, ytest):
    a = np.ascontiguousarray(np.asarray(mean, dtype=np.float64))
    b = np.ascontiguousarray(np.asarray(ytest, dtype=np.float64))
    if a.shape != b.shape or a.ndim != 1:
        raise NugprError(NUGPR_ERR_INVALID, "mean and ytest must be vectors of one length")
    out = C.c_double()
    _check(load_library().nugpr_rmse(_dptr(a), _dptr(b), a.shape[0], C.byref(out)))
    return out.value


def nugpr_host_smallest_eigenvalue(A):
    a = np.ascontiguousarray(np.asarray(A, dtype=np.float64))
    if a.ndim != 2 or a.shape[0] != a.shape[1]:
        raise NugprError(NUGPR_ERR_INVALID, "A must be square")
    out = C.c_double()
    _check(load_library().nugpr_host_smallest_eigenvalue(_dptr(a), a.shape[0], C.byref(out)))
    return out.value


def nugpr_confidence_band(mean, var):
    a = np.ascontiguousarray(np.asarray(mean, dtype=np.float64))
    v = np.ascontiguousarray(np.asarray(var, dtype=np.float64))
    if a.shape != v.shape or a.ndim != 1:
        raise NugprError(NUGPR_ERR_INVALID, "mean and var must be vectors of one length")
    lo, hi = np.zeros_like(a), np.zeros_like(a)
    _check(load_library().nugpr_confidence_band(_dptr(a), _dptr(v), a.shape[0], _dptr(lo), _dptr(hi)))
    return lo, hi


class Context:
    """Owns the device buffers (torch tensors) and the nugpr_ctx handle.

    X (n,d), y (n,), probes (n,t): float32 arrays or CUDA tensors; offsets: int64 host
    array; reps / W optional.  Methods mirror the C entry points one to one."""

    def __init__(self, X, y, offsets, probes, rank, tol=1e-6, max_iter=100, fd_step=1e-3, lr=0.05,
                 isotropic=False, reps=None, W=None, device="cuda:0", acc_fp32=False, no_shortcuts=False,
                 logdet_pade=False, fd_forward=False, fd_threshold=0.0, fd_max_halvings=0, compensate=False,
                 precond_compensated=False):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.device = torch.device(device)

        def dev(a):
            if a is None:
                return None
            t = torch.as_tensor(a)
            return t.to(device=self.device, dtype=torch.float32).contiguous()

        self.X, self.y, self.probes = dev(X), dev(y), dev(probes)
        self.reps, self.W = dev(reps), dev(W)
        self.offsets = np.ascontiguousarray(np.asarray(offsets, dtype=np.int64))
        self.n, self.d = int(self.X.shape[0]), int(self.X.shape[1])
        self.t = int(self.probes.shape[1]) if self.probes is not None and self.probes.numel() else 0
        self.T = self.t + 1
        self.rank = int(rank)
        self.nc = int(self.offsets.shape[0] - 1)
        pb = Problem()
        pb.n, pb.d, pb.n_clusters, pb.rank, pb.n_probes = self.n, self.d, self.nc, self.rank, self.t
        pb.cluster_offsets = self.offsets.ctypes.data_as(C.POINTER(C.c_int64))
        pb.X, pb.y = self.X.data_ptr(), self.y.data_ptr()
        pb.reps = self.reps.data_ptr() if self.reps is not None else None
        pb.W = self.W.data_ptr() if self.W is not None else None
        pb.probes = self.probes.data_ptr() if self.t else None
        nbytes = self.lib.nugpr_workspace_bytes(C.byref(pb))
        if nbytes == 0:
            raise NugprError(NUGPR_ERR_INVALID, self.lib.nugpr_last_error_string().decode())
        self.workspace_bytes = int(nbytes)
        self.workspace = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        pb.workspace = (base + 255) // 256 * 256
        pb.workspace_bytes = self.workspace_bytes
        pr = Params(tol=tol, max_iter=max_iter, fd_step=fd_step, lr=lr, beta1=0.0, beta2=0.0, eps=0.0,
                    flags=(NUGPR_ISOTROPIC if isotropic else 0) | (NUGPR_ACC_FP32 if acc_fp32 else 0)
                    | (NUGPR_NO_SHORTCUTS if no_shortcuts else 0) | (NUGPR_LOGDET_PADE if logdet_pade else 0)
                    | (NUGPR_FD_FORWARD if fd_forward else 0) | (NUGPR_COMPENSATE if compensate else 0)
                    | (NUGPR_PRECOND_COMPENSATED if precond_compensated else 0),
                    fd_max_halvings=int(fd_max_halvings), fd_threshold=float(fd_threshold))
        self.params = pr
        self.max_iter = int(max_iter)
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(self.lib.nugpr_create(C.byref(h), C.byref(pb), C.byref(pr), self._stream()))
        self.handle = h
        self.p = int(self.lib.nugpr_num_hyper(self.handle))

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def close(self):
        if getattr(self, "handle", None):
            self.lib.nugpr_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _theta(self, theta):
        th = np.ascontiguousarray(np.asarray(theta, dtype=np.float64))
        if th.shape != (self.p,):
            raise NugprError(NUGPR_ERR_INVALID, f"theta must have {self.p} entries")
        return th

    # ---- entry points -------------------------------------------------------
    def nugpr_build_blocks(self, theta):
        th = self._theta(theta)
        return _check(self.lib.nugpr_build_blocks(self.handle, _dptr(th), self._stream()))

    def nugpr_set_nystrom_basis(self, theta, jitter=0.0):
        th = self._theta(theta)
        return _check(self.lib.nugpr_set_nystrom_basis(self.handle, _dptr(th), float(jitter), self._stream()))

    def nugpr_precond_factor(self):
        ld, bad = C.c_double(), C.c_int32()
        code = _check(self.lib.nugpr_precond_factor(self.handle, C.byref(ld), C.byref(bad), self._stream()))
        return code, ld.value, bad.value

    def _block(self, a):
        t = self.torch.as_tensor(a).to(device=self.device, dtype=self.torch.float32).contiguous()
        if t.dim() == 1:
            t = t[:, None].contiguous()
        return t

    def nugpr_matvec(self, D):
        D = self._block(D)
        Q = self.torch.empty_like(D)
        _check(self.lib.nugpr_matvec(self.handle, D.data_ptr(), Q.data_ptr(), D.shape[1], self._stream()))
        return Q

    def nugpr_matvec_static(self, D):
        D = self._block(D)
        Q = self.torch.empty_like(D)
        _check(self.lib.nugpr_matvec_static(self.handle, D.data_ptr(), Q.data_ptr(), D.shape[1], self._stream()))
        return Q

    def nugpr_split_apply(self, D):
        D = self._block(D)
        out = self.torch.empty_like(D)
        _check(self.lib.nugpr_split_apply(self.handle, D.data_ptr(), out.data_ptr(), D.shape[1], self._stream()))
        return out

    def nugpr_precond_apply(self, R):
        R = self._block(R)
        Z = self.torch.empty_like(R)
        _check(self.lib.nugpr_precond_apply(self.handle, R.data_ptr(), Z.data_ptr(), R.shape[1], self._stream()))
        return Z

    def nugpr_pcg_solve(self, B):
        B = self._block(B)
        ncols = int(B.shape[1])
        X = self.torch.empty_like(B)
        iters = np.zeros(ncols, dtype=np.int32)
        alpha = np.zeros((self.max_iter, ncols), dtype=np.float64)
        beta = np.zeros((self.max_iter, ncols), dtype=np.float64)
        code = _check(self.lib.nugpr_pcg_solve(self.handle, B.data_ptr(), X.data_ptr(), ncols,
                                               iters.ctypes.data_as(C.POINTER(C.c_int32)), _dptr(alpha), _dptr(beta),
                                               self._stream()))
        return code, X, iters, alpha, beta

    def nugpr_mll(self, theta):
        th = self._theta(theta)
        r = MllResult()
        code = _check(self.lib.nugpr_mll(self.handle, _dptr(th), C.byref(r), self._stream()))
        return dict(code=code, nll=r.nll, quad=r.quad, logdet=r.logdet, logdet_precond=r.logdet_precond,
                    max_iters_used=r.max_iters_used, status=r.status)

    def nugpr_train_step(self, log_theta, adam_m, adam_v, step):
        phi = np.ascontiguousarray(np.asarray(log_theta, dtype=np.float64)).copy()
        m = np.ascontiguousarray(np.asarray(adam_m, dtype=np.float64)).copy()
        v = np.ascontiguousarray(np.asarray(adam_v, dtype=np.float64)).copy()
        if phi.shape != (self.p,) or m.shape != (self.p,) or v.shape != (self.p,):
            raise NugprError(NUGPR_ERR_INVALID, f"log_theta / adam_m / adam_v must have {self.p} entries")
        st = C.c_int64(int(step))
        nll0 = C.c_double()
        g = np.zeros(self.p, dtype=np.float64)
        code = _check(self.lib.nugpr_train_step(self.handle, _dptr(phi), _dptr(m), _dptr(v), C.byref(st),
                                                C.byref(nll0), _dptr(g), self._stream()))
        return dict(code=code, log_theta=phi, adam_m=m, adam_v=v, step=st.value, nll0=nll0.value, grad=g)

    def nugpr_predict(self, theta, Xtest, variance=True):
        th = self._theta(theta)
        Xt = self.torch.as_tensor(Xtest).to(device=self.device, dtype=self.torch.float32).contiguous()
        if Xt.dim() != 2 or Xt.shape[1] != self.d:
            raise NugprError(NUGPR_ERR_INVALID, f"Xtest must be (m, {self.d})")
        m = int(Xt.shape[0])
        mean = np.zeros(m, dtype=np.float64)
        var = np.zeros(m, dtype=np.float64) if variance else None
        mx = C.c_int32()
        code = _check(self.lib.nugpr_predict(self.handle, _dptr(th), Xt.data_ptr() if m else None, m, _dptr(mean),
                                             _dptr(var) if variance else None, C.byref(mx), self._stream()))
        return dict(code=code, mean=mean, var=var, max_iters_used=mx.value)

    def nugpr_compensation_lambda(self):
        out = C.c_double()
        _check(self.lib.nugpr_compensation_lambda(self.handle, C.byref(out)))
        return out.value

    def nugpr_compensation_steps(self):
        out = C.c_int32()
        _check(self.lib.nugpr_compensation_steps(self.handle, C.byref(out)))
        return out.value

    def nugpr_fd_halvings(self):
        out = np.zeros(self.p, dtype=np.int32)
        _check(self.lib.nugpr_fd_halvings(self.handle, out.ctypes.data_as(C.POINTER(C.c_int32))))
        return out

    def nugpr_matvec_into(self, D, Q):
        """nugpr_matvec on caller-held device tensors (no allocation; used for timing)."""
        return _check(self.lib.nugpr_matvec(self.handle, D.data_ptr(), Q.data_ptr(), D.shape[1], self._stream()))

    def nugpr_matvec_static_into(self, D, Q):
        """nugpr_matvec_static on caller-held device tensors: nothing is allocated on either side of the ABI."""
        return _check(self.lib.nugpr_matvec_static(self.handle, D.data_ptr(), Q.data_ptr(), D.shape[1],
                                                   self._stream()))

    def nugpr_precond_apply_into(self, R, Z):
        return _check(self.lib.nugpr_precond_apply(self.handle, R.data_ptr(), Z.data_ptr(), R.shape[1],
                                                   self._stream()))

    def nugpr_profile_enable(self, on=True):
        return _check(self.lib.nugpr_profile_enable(self.handle, 1 if on else 0))

    def nugpr_profile_read(self):
        ms, cnt = C.c_double(), C.c_int32()
        _check(self.lib.nugpr_profile_read(self.handle, C.byref(ms), C.byref(cnt), self._stream()))
        return ms.value, cnt.value

    def nugpr_profile_bytes(self, ncols):
        return float(self.lib.nugpr_profile_bytes(self.handle, int(ncols)))

    def nugpr_profile_kernel_name(self, ncols):
        buf = C.create_string_buffer(128)
        _check(self.lib.nugpr_profile_kernel_name(self.handle, int(ncols), buf, 128))
        return buf.value.decode()

    def nugpr_stats_read(self, reset=False):
        st = Stats()
        _check(self.lib.nugpr_stats_read(self.handle, C.byref(st), 1 if reset else 0))
        return {k: int(getattr(st, k)) for k, _ in Stats._fields_}

    def nugpr_export(self, what, index=0):
        if what in (EXPORT_K, EXPORT_L, EXPORT_LINV):
            b = int(self.offsets[index + 1] - self.offsets[index])
            shape = (b, b)
        elif what == EXPORT_C:
            shape = (self.nc * self.rank,) * 2
        elif what == EXPORT_W:
            shape = (int(self.offsets[index + 1] - self.offsets[index]), self.rank)
        elif what == EXPORT_B:
            shape = (self.n, self.T)
        elif what == EXPORT_REPS:
            shape = (self.nc * self.rank, self.d)
        else:
            raise NugprError(NUGPR_ERR_INVALID, "unknown export selector")
        out = self.torch.empty(shape, dtype=self.torch.float32, device=self.device)
        _check(self.lib.nugpr_export(self.handle, what, index, out.data_ptr(), shape[1], self._stream()))
        return out
