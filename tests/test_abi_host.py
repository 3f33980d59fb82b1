"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, sizes workspaces and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2510_12128_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.lib_path()):
        from paper_2510_12128_amd import build
        build.build()
    return B.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "nugpr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nugpr_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    for must in ["nugpr_build_blocks", "nugpr_precond_factor", "nugpr_pcg_solve", "nugpr_mll",
                 "nugpr_train_step", "nugpr_matvec", "nugpr_create", "nugpr_destroy", "nugpr_predict",
                 "nugpr_rmse", "nugpr_confidence_band"]:
        assert must in names
    for n in names:
        assert hasattr(lib, n), n


def problem(offsets, d=3, rank=4, t=8):
    off = np.asarray(offsets, dtype=np.int64)
    pb = B.Problem()
    pb.n, pb.d, pb.n_clusters, pb.rank, pb.n_probes = int(off[-1]), d, len(off) - 1, rank, t
    pb.cluster_offsets = off.ctypes.data_as(C.POINTER(C.c_int64))
    return pb, off


def test_workspace_bytes_scales_with_block_storage(lib):
    pb, keep = problem([0, 512, 1024, 1536, 2048], rank=32, t=8)
    small = lib.nugpr_workspace_bytes(C.byref(pb))
    # three square fp32 copies of the diagonal blocks dominate (K, L, L^-1)
    assert small > 3 * 4 * 512 * 512 * 4
    assert small < 6 * 4 * 512 * 512 * 4
    pb2, keep2 = problem([0, 1000, 2100], rank=32, t=8)          # ragged sizes pad to 64
    assert lib.nugpr_workspace_bytes(C.byref(pb2)) > 3 * 4 * (1024 * 1024 + 1152 * 1152)


@pytest.mark.parametrize("offsets,d,rank,t", [
    ([0, 10, 5], 3, 2, 4),          # not ascending
    ([1, 10, 20], 3, 2, 4),         # does not start at 0
    ([0, 10, 20], 0, 2, 4),         # d out of range
    ([0, 10, 20], 65, 2, 4),
    ([0, 10, 20], 3, 11, 4),        # rank larger than a cluster
    ([0, 10, 20], 3, 0, 4),
    ([0, 10, 20], 3, 2, 33),        # too many probes
])
def test_invalid_problems_are_rejected(lib, offsets, d, rank, t):
    pb, keep = problem(offsets, d, rank, t)
    assert lib.nugpr_workspace_bytes(C.byref(pb)) == 0
    assert len(lib.nugpr_last_error_string()) > 0


def test_create_rejects_bad_params_and_null_buffers_without_gpu(lib):
    pb, keep = problem([0, 10, 20], 3, 2, 4)
    h = C.c_void_p()
    pr = B.Params(tol=0.0, max_iter=10, fd_step=1e-3, lr=0.05, beta1=0, beta2=0, eps=0, flags=0)
    assert lib.nugpr_create(C.byref(h), C.byref(pb), C.byref(pr), None) == B.NUGPR_ERR_INVALID
    pr.tol = 1e-6
    pr.max_iter = 0
    assert lib.nugpr_create(C.byref(h), C.byref(pb), C.byref(pr), None) == B.NUGPR_ERR_INVALID
    pr.max_iter = 10
    assert lib.nugpr_create(C.byref(h), C.byref(pb), C.byref(pr), None) == B.NUGPR_ERR_INVALID   # X is null
    assert not h.value
    assert lib.nugpr_destroy(None) == 0
    assert lib.nugpr_build_blocks(None, None, None) == B.NUGPR_ERR_INVALID


def test_host_side_prediction_scores(lib):
    # Section 2.1: RMSE and the two-sigma band, by hand on three numbers
    assert abs(B.nugpr_rmse([1.0, 2.0, 4.0], [1.0, 0.0, 0.0]) - (20.0 / 3.0) ** 0.5) < 1e-15
    lo, hi = B.nugpr_confidence_band([0.0, 1.0, -2.0], [4.0, 0.25, -1e-9])
    np.testing.assert_allclose(lo, [-4.0, 0.0, -2.0], atol=1e-15)
    np.testing.assert_allclose(hi, [4.0, 2.0, -2.0], atol=1e-15)
    with pytest.raises(B.NugprError):
        B.nugpr_rmse([], [])


def test_host_smallest_eigenvalue_against_lapack(lib):
    # the host routine behind lambda_0 of eq. (krep): Householder + QL, checked against numpy's eigvalsh
    rng = np.random.default_rng(5)
    for n in (1, 2, 3, 17, 130):
        A = rng.standard_normal((n, n))
        A = A + A.T
        want = np.linalg.eigvalsh(A)[0]
        assert abs(B.nugpr_host_smallest_eigenvalue(A) - want) <= 1e-12 * max(1.0, np.abs(A).sum(axis=1).max()), n
    # kernel matrices: nearly singular, clustered small eigenvalues
    R = rng.normal(size=(64, 3))
    d2 = ((R[:, None, :] - R[None, :, :]) ** 2).sum(axis=2)
    for ell in (0.3, 1.0, 3.0):
        K = 1.3 * np.exp(-0.5 * d2 / ell ** 2)
        assert abs(B.nugpr_host_smallest_eigenvalue(K) - np.linalg.eigvalsh(K)[0]) < 1e-12
    # closed form, a diagonal matrix, and only the lower triangle is read
    assert abs(B.nugpr_host_smallest_eigenvalue([[2.0, 99.0], [-0.5, 2.0]]) - 1.5) < 1e-14
    assert abs(B.nugpr_host_smallest_eigenvalue(np.diag([3.0, -1.0, 2.0])) + 1.0) < 1e-14
    with pytest.raises(B.NugprError):
        B.nugpr_host_smallest_eigenvalue(np.zeros((0, 0)))


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setattr(B, "lib_path", lambda: str(tmp_path / "libnugpr.so"))
    with pytest.raises(RuntimeError):
        B.load_library()
