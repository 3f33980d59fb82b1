"""The entry point that allocates nothing, nugpr_matvec_static, against nugpr_matvec (whose parity with the
oracle the other GPU tests hold): same kernels, scratch in the library's static device buffer instead of the
context's workspace.  Two calls in a row share that buffer, the second on a smaller input, so stale contents
of the first must not reach the second's result."""
import numpy as np
import pytest

from oracle import nugpr_oracle as O
from paper_2510_12128_amd import inputs as I
from paper_2510_12128_amd import binding as B

pytestmark = pytest.mark.gpu


def relmax(a, b):
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


def test_static_scratch_matvec_matches_the_workspace_one_on_two_calls_in_a_row(lib):
    import gc
    import torch
    big = I.make_small(n_clusters=17, sizes=[130 + (7 * i) % 23 for i in range(17)], d=3, rank=128, t=16, seed=9,
                       ell=1.5, spacing=7.0, sigma_blob=0.5, tol=1e-6, max_iter=100)
    small = I.make_small(n_clusters=4, sizes=[200, 70, 129, 64], d=3, rank=8, t=8, seed=3, ell=1.5, spacing=4.5,
                         sigma_blob=0.3, tol=1e-6, max_iter=100)
    ctxs = []
    for w in (big, small):
        ctx = lib.Context(w.X, w.y, w.offsets, w.probes, w.rank, tol=w.tol, max_iter=w.max_iter)
        ctx.nugpr_build_blocks(w.theta)
        ctxs.append(ctx)
    rng = np.random.default_rng(5)
    dev = ctxs[0].device
    # first call: the larger problem at its full width; second call: the smaller problem, fewer columns
    plan = [(ctxs[0], big, big.n_probes + 1), (ctxs[1], small, 5), (ctxs[1], small, 1), (ctxs[0], big, 2)]
    for ctx, w, ncols in plan:
        D = torch.as_tensor(rng.standard_normal((w.n, ncols)).astype(np.float32), device=dev)
        Qs = torch.full((w.n, ncols), float("nan"), dtype=torch.float32, device=dev)
        Qw = torch.empty_like(Qs)
        gc.collect()                       # tensors of earlier tests that are still waiting for the collector
        before = torch.cuda.memory_allocated(dev)
        assert ctx.nugpr_matvec_static_into(D, Qs) == 0
        assert torch.cuda.memory_allocated(dev) == before
        assert ctx.nugpr_matvec_into(D, Qw) == 0
        torch.cuda.synchronize(dev)
        got, ref = Qs.cpu().numpy().astype(np.float64), Qw.cpu().numpy().astype(np.float64)
        # the same kernels in the same order on the same data: identical results
        assert np.array_equal(got, ref), (w.name, ncols, relmax(got, ref))
        # and, through the oracle's operator, the bar of the product tests
        prob = O.Problem(w.X, w.y, w.offsets, w.probes, w.rank)
        exp = prob.operator(w.theta)(D.cpu().numpy().astype(np.float64))
        assert relmax(got, exp) < 1e-5, (w.name, ncols)
    for ctx in ctxs:
        ctx.close()


def test_static_scratch_matvec_refuses_products_beyond_its_buffer(lib):
    import torch
    cap = B.load_library().nugpr_matvec_static_max_bytes()
    assert cap == 16 << 20
    w = I.make_config("C3", scale=0.5)                  # n = 65536, 17 columns: the two fp64 blocks alone are 17.8 MB
    assert 2 * w.n * (w.n_probes + 1) * 8 > cap
    ctx = lib.Context(w.X, w.y, w.offsets, w.probes, w.rank, tol=w.tol, max_iter=w.max_iter)
    ctx.nugpr_build_blocks(w.theta)
    D = torch.zeros((w.n, w.n_probes + 1), dtype=torch.float32, device=ctx.device)
    Q = torch.empty_like(D)
    with pytest.raises(B.NugprError) as e:
        ctx.nugpr_matvec_static_into(D, Q)
    assert e.value.code == B.NUGPR_ERR_WORKSPACE
    assert "16777216" in str(e.value)
    # one column of the same problem fits (2 x 0.5 MB + slabs) and runs
    D1 = torch.ones((w.n, 1), dtype=torch.float32, device=ctx.device)
    Q1, Q2 = torch.empty_like(D1), torch.empty_like(D1)
    assert ctx.nugpr_matvec_static_into(D1, Q1) == 0
    assert ctx.nugpr_matvec_into(D1, Q2) == 0
    torch.cuda.synchronize(ctx.device)
    assert torch.equal(Q1, Q2)
    ctx.close()
