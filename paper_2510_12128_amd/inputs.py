"""Seeded synthetic inputs for the nuGPR marginal-log-likelihood hot path.

This module holds NO arithmetic of the method (no kernels, no solves): it only
draws clustered point clouds, targets and Rademacher probe vectors.  Both the
HIP path and the CPU oracle are fed the arrays produced here; neither imports
the other.

The point clouds stand in for the paper's clustered data sets (Section 4.1:
synthetic clusters around chosen centres; real data clustered by k-means or by
label): isotropic Gaussian blobs, one blob per cluster, stored
cluster-contiguous with a cluster-offset array.  Drawing order for a data seed
is fixed: [cluster proportions] -> centres -> points cluster by cluster ->
[linear weights w] -> target noise.  Probes come from their own seed and are
+1/-1 (Section 3.1, Hutchinson vectors).  Everything is cast to float32 once and
handed to both sides.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass
class Workload:
    name: str
    X: np.ndarray                # (n, d) float32, cluster-contiguous
    y: np.ndarray                # (n,)   float32
    offsets: np.ndarray          # (n_clusters + 1,) int64
    probes: np.ndarray           # (n, t) float32, entries +1/-1
    rank: int                    # representatives per cluster
    theta: np.ndarray            # float64: [ell_1..ell_d, outputscale, noise] or [ell, outputscale, noise]
    isotropic: bool
    tol: float
    max_iter: int
    fd_step: float = 1e-3
    lr: float = 0.05
    meta: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return int(self.X.shape[0])

    @property
    def d(self) -> int:
        return int(self.X.shape[1])

    @property
    def n_clusters(self) -> int:
        return int(self.offsets.shape[0] - 1)

    @property
    def n_probes(self) -> int:
        return int(self.probes.shape[1])


def dirichlet_sizes(rng: np.random.Generator, n: int, n_clusters: int, alpha: float,
                    min_size: int) -> np.ndarray:
    """Cluster sizes from Dirichlet(alpha) proportions, floored, the leftover
    points handed one each to the largest fractional parts, so the sizes sum to n."""
    p = rng.dirichlet(np.full(n_clusters, alpha))
    raw = p * n
    sizes = np.floor(raw).astype(np.int64)
    left = int(n - sizes.sum())
    order = np.argsort(-(raw - sizes), kind="stable")
    sizes[order[:left]] += 1
    if sizes.min() < min_size:
        raise ValueError("a cluster came out smaller than the rank")
    return sizes


def rademacher(seed: int, n: int, t: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (2.0 * rng.integers(0, 2, size=(n, t)) - 1.0).astype(np.float32)


def grid_centres(n_clusters: int, d: int, spacing: float) -> np.ndarray:
    """Centres on the vertices of a d-dimensional grid of side `spacing`, enumerated
    in mixed-radix order (the paper's synthetic sets put cluster centres on hypercube
    vertices, Section 4.1)."""
    side = int(np.ceil(n_clusters ** (1.0 / d)))
    idx = np.arange(n_clusters)
    cols = []
    for _ in range(d):
        cols.append(idx % side)
        idx = idx // side
    return spacing * np.stack(cols, axis=1).astype(np.float64)


def blobs(sizes, d: int, centre_halfwidth: float, sigma_blob: float, target: str,
          noise_std: float, seed: int = 0, centre_shrink: float = 1.0,
          rng: Optional[np.random.Generator] = None, spacing: Optional[float] = None):
    """Gaussian blobs, one per cluster; returns X (float32), y (float32), offsets, centres."""
    sizes = np.asarray(sizes, dtype=np.int64)
    if rng is None:
        rng = np.random.default_rng(seed)
    n_clusters = sizes.shape[0]
    n = int(sizes.sum())
    if spacing is not None:
        centres = grid_centres(n_clusters, d, spacing)
    else:
        centres = rng.uniform(-centre_halfwidth, centre_halfwidth, size=(n_clusters, d)) / centre_shrink
    X = np.empty((n, d), dtype=np.float64)
    offsets = np.zeros(n_clusters + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(sizes)
    for i in range(n_clusters):
        X[offsets[i]:offsets[i + 1]] = centres[i] + sigma_blob * rng.standard_normal((int(sizes[i]), d))
    if target == "sin_of_sum":
        f = np.sin(X.sum(axis=1))
    elif target == "sum_of_sin":
        f = np.sin(X).sum(axis=1)
    elif target == "linear_plus_sin":
        w = rng.standard_normal(d) / np.sqrt(d)
        f = X @ w + 0.5 * np.sin(X[:, 0] * X[:, 1])
    else:
        raise ValueError(target)
    yv = f + noise_std * rng.standard_normal(n)
    return X.astype(np.float32), yv.astype(np.float32), offsets, centres


_CONFIGS = {
    # name: n_clusters, b, d, halfwidth, sigma_blob, target, noise_std, rank, t, noise_var, iso, tol
    "C1": dict(n_clusters=4, b=512, d=3, hw=5.0, sb=0.5, target="sin_of_sum", ns=0.1,
               rank=32, t=8, noise=0.1, iso=True, tol=1e-6),
    "C2": dict(n_clusters=32, b=1024, d=8, hw=10.0, sb=1.0, target="sum_of_sin", ns=0.05,
               rank=64, t=16, noise=0.05, iso=False, tol=1e-6),
    "C3": dict(n_clusters=64, b=2048, d=8, hw=10.0, sb=1.0, target="sum_of_sin", ns=0.05,
               rank=64, t=16, noise=0.05, iso=False, tol=1e-5),
    "C4": dict(n_clusters=128, b=2048, d=20, hw=10.0, sb=1.5, target="linear_plus_sin", ns=0.1,
               rank=128, t=16, noise=0.1, iso=False, tol=1e-6),
    "C5": dict(n_clusters=256, b=4096, d=8, hw=10.0, sb=1.0, target="sum_of_sin", ns=0.05,
               rank=32, t=32, noise=0.05, iso=False, tol=1e-5, dirichlet=5.0),
}


# Stress presets (correctness only, never timed): a tied lengthscale wide enough that
# within-cluster kernel values are O(0.3) and the off-diagonal low-rank path carries
# weight, so PCG needs several iterations, while K' stays positive definite.
STRESS = {
    "C1": dict(ell=1.5),
    "C2": dict(ell=2.83),
    "C3": dict(ell=2.83),
    "C4": dict(ell=5.37),
    "C5": dict(ell=2.83),
}


def make_config(name: str, variant: str = "default", scale: float = 1.0,
                ell: Optional[float] = None, centre_shrink: float = 1.0,
                data_seed: int = 0, probe_seed: int = 1) -> Workload:
    """One of the five benchmark configurations (C1..C5).

    variant "default": lengthscale 1 as the configuration states.
    variant "wide":    the STRESS preset lengthscale (see above).
    `ell` overrides the (tied) lengthscale; `centre_shrink` divides the blob centres
    (clusters move closer; the approximated covariance may then lose
    positive-definiteness, which is what the error-path tests use).
    scale < 1 shrinks the cluster count (same per-cluster shape), for parity runs
    the CPU oracle finishes in seconds.
    """
    c = dict(_CONFIGS[name])
    n_clusters = max(2, int(round(c["n_clusters"] * scale)))
    rng = np.random.default_rng(data_seed)
    if "dirichlet" in c:
        n = n_clusters * c["b"]
        sizes = dirichlet_sizes(rng, n, n_clusters, c["dirichlet"], c["rank"])
    else:
        sizes = np.full(n_clusters, c["b"], dtype=np.int64)
    X, y, offsets, centres = blobs(sizes, c["d"], c["hw"], c["sb"], c["target"], c["ns"],
                                   centre_shrink=centre_shrink, rng=rng)
    if variant not in ("default", "wide"):
        raise ValueError(variant)
    if ell is None:
        ell = 1.0 if variant == "default" else STRESS[name]["ell"]
    if c["iso"]:
        theta = np.array([ell, 1.0, c["noise"]], dtype=np.float64)
    else:
        theta = np.concatenate([np.full(c["d"], ell), [1.0, c["noise"]]]).astype(np.float64)
    probes = rademacher(probe_seed, X.shape[0], c["t"])
    tag = f"{name}-{variant}" + ("" if scale == 1.0 else f"-x{scale:g}")
    return Workload(name=tag, X=X, y=y, offsets=offsets, probes=probes, rank=c["rank"], theta=theta,
                    isotropic=c["iso"], tol=c["tol"], max_iter=100,
                    meta=dict(centres=centres, config=name, variant=variant, scale=scale,
                              ell=ell, centre_shrink=centre_shrink))


def make_small(n_clusters: int = 3, sizes=None, d: int = 2, rank: int = 2, t: int = 4,
               ell: float = 1.5, outputscale: float = 1.3, noise: float = 0.2,
               sigma_blob: float = 0.6, halfwidth: float = 3.0, isotropic: bool = False,
               seed: int = 0, probe_seed: int = 1, tol: float = 1e-10,
               max_iter: int = 200, target: str = "sin_of_sum",
               spacing: Optional[float] = None) -> Workload:
    """Tiny free-form workload for pins, edge cases and ragged-size parity tests.
    `spacing` puts the centres on a grid (well-separated clusters with a controlled
    coupling strength) instead of drawing them uniformly."""
    if sizes is None:
        sizes = [8] * n_clusters
    X, y, offsets, centres = blobs(sizes, d, halfwidth, sigma_blob, target, 0.1, seed=seed,
                                   spacing=spacing)
    if isotropic:
        theta = np.array([ell, outputscale, noise], dtype=np.float64)
    else:
        rng = np.random.default_rng(seed + 1000)
        theta = np.concatenate([ell * rng.uniform(0.7, 1.4, size=d), [outputscale, noise]])
    probes = rademacher(probe_seed, X.shape[0], t)
    return Workload(name=f"small-{len(sizes)}x{d}-s{seed}", X=X, y=y, offsets=offsets, probes=probes,
                    rank=rank, theta=np.asarray(theta, dtype=np.float64), isotropic=isotropic,
                    tol=tol, max_iter=max_iter, meta=dict(centres=centres))


def test_points(w: Workload, m: int, seed: int = 0, margin: float = 0.1) -> np.ndarray:
    """m seeded test inputs (float32) for a workload: half are training points displaced by a
    fraction of their cluster's spread (inputs that fall inside the clusters, as a held-out
    split of the same data would), half are uniform over the bounding box of the training set
    widened by `margin` of its extent per side (the uniformly spread test inputs of the
    synthetic experiments, some of them far from every cluster)."""
    rng = np.random.default_rng(seed + 77001)
    X = np.asarray(w.X, dtype=np.float64)
    m_in = m // 2
    idx = rng.integers(0, X.shape[0], size=m_in)
    spread = X.std(axis=0) / max(w.n_clusters, 1) ** (1.0 / max(X.shape[1], 1))
    inside = X[idx] + 0.25 * spread * rng.standard_normal((m_in, X.shape[1]))
    lo, hi = X.min(axis=0), X.max(axis=0)
    ext = hi - lo
    outside = rng.uniform(lo - margin * ext, hi + margin * ext, size=(m - m_in, X.shape[1]))
    out = np.concatenate([inside, outside], axis=0)
    return out[rng.permutation(m)].astype(np.float32)


test_points.__test__ = False     # not a pytest case


def hadamard_probes(n: int) -> np.ndarray:
    """Sylvester-Hadamard matrix of order n (a power of two), entries +1/-1,
    H H^T = n I: with these n probes the Hutchinson trace estimate is exact."""
    if n & (n - 1):
        raise ValueError("n must be a power of two")
    H = np.ones((1, 1), dtype=np.float32)
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    return H.astype(np.float32)
