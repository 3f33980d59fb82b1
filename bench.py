#!/usr/bin/env python3
"""Benchmark of the nuGPR marginal-log-likelihood hot path on one MI355X.

A "step" is one pass of the whole hot path: nugpr_train_step = block assembly and
block-Jacobi factorisation at theta_0, then 1 + 2p loss evaluations (assembly, batched PCG
with the block-low-rank product and the preconditioner apply, SLQ log-determinant) for the
central-difference gradient, and the Adam update.  The metric is loss evaluations per
second over the timed steps (factorisation included); the roofline entry is the dominant
kernel, the launch that streams K_diag and the coupling matrix C once per product, timed
live with HIP events inside the same timed region.

Prints ONE JSON line.  Inputs are synthetic (seeded Gaussian blobs of the configured shape),
resident in HBM before the timed region starts.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per launch of the dominant kernel from the two rocprofv3 --pmc runs summarised in
# profiles/k_strip_C4_*_hbm_traffic.md (FETCH_SIZE + WRITE_SIZE, scaled by the copy probe).
# Counter runs are separate from this program, so the figure is quoted, not measured live.
MEASURED_TRAFFIC_BYTES = {("C4", "fp64"): 2.329e9}


def cpu_baseline(w, n_sample_clusters):
    """The fp64 oracle, as it stands, on the first clusters of the same workload:
    one loss evaluation (assembly + PCG + SLQ; the factor is built outside the timing,
    as on the GPU it is shared by the 1 + 2p evaluations of a step)."""
    import numpy as np
    from oracle import nugpr_oracle as O
    k = min(n_sample_clusters, w.n_clusters)
    hi = int(w.offsets[k])
    prob = O.Problem(w.X[:hi], w.y[:hi], w.offsets[:k + 1], w.probes[:hi], w.rank)
    fac = O.Factor(prob, w.theta)
    t0 = time.perf_counter()
    out = O.mll(prob, fac, w.theta, w.tol, w.max_iter)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    frac = k / w.n_clusters
    return dict(value=frac / dt, unit="evals/s", cores=int(cores), kind="oracle",
                sample=(f"one loss evaluation (assembly + PCG + SLQ, fp64 numpy/scipy) on the first {k} of "
                        f"{w.n_clusters} clusters (n={hi}) took {dt:.2f} s; rate scaled by {k}/{w.n_clusters} "
                        f"to the full workload; oracle nll on the sample {out['nll']:.6e}"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C4")
    ap.add_argument("--acc", choices=["fp64", "fp32"], default="fp64",
                    help="arithmetic of the operator applications over the fp32 stored matrices")
    ap.add_argument("--cpu-clusters", type=int, default=8, help="clusters in the CPU-oracle sample (0 = skip)")
    ap.add_argument("--kv-reps", type=int, default=20)
    ap.add_argument("--copy-probe-gib", type=float, default=0.0,
                    help="also run a plain copy kernel of this many GiB three times (reference dispatch for "
                         "scaling hardware HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, one device); --gpus N with N > 1 is not "
              "supported and no multi-GPU figure exists", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    from paper_2510_12128_amd import Context, inputs

    dev = torch.device("cuda:0")
    if args.copy_probe_gib > 0:
        from paper_2510_12128_amd.binding import nugpr_copy_probe
        nb = int(args.copy_probe_gib * (1 << 30)) // 16 * 16
        src = torch.ones(nb // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            nugpr_copy_probe(dst, src)
        torch.cuda.synchronize(dev)
        del src, dst
    w = inputs.make_config(args.config)
    ctx = Context(w.X, w.y, w.offsets, w.probes, w.rank, tol=w.tol, max_iter=w.max_iter, fd_step=w.fd_step,
                  lr=w.lr, isotropic=w.isotropic, device=dev, acc_fp32=(args.acc == "fp32"))
    p, T = ctx.p, ctx.T
    phi = np.log(w.theta)
    m, v, step = np.zeros(p), np.zeros(p), 0

    def sync():
        torch.cuda.synchronize(dev)

    for _ in range(args.warmup):
        out = ctx.nugpr_train_step(phi, m, v, step)
        phi, m, v, step = out["log_theta"], out["adam_m"], out["adam_v"], out["step"]
    ctx.nugpr_profile_enable(True)
    sync()
    t0 = time.perf_counter()
    codes, step_ms, step_iters = [], [], []
    for _ in range(args.steps):
        ts = time.perf_counter()
        out = ctx.nugpr_train_step(phi, m, v, step)      # returns after the step's last synchronisation
        step_ms.append((time.perf_counter() - ts) * 1e3)
        phi, m, v, step = out["log_theta"], out["adam_m"], out["adam_v"], out["step"]
        codes.append(out["code"])
    sync()
    t1 = time.perf_counter()
    dom_ms, dom_launches = ctx.nugpr_profile_read()
    ctx.nugpr_profile_enable(False)
    total_s = t1 - t0
    evals = args.steps * (1 + 2 * p)
    evals_per_s = evals / total_s

    # ---- the pieces, timed alone with events on the stream the library launches on ----
    def time_ms(fn, reps):
        fn()
        sync()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        sync()
        return e0.elapsed_time(e1) / reps

    theta = np.exp(phi)
    ctx.nugpr_build_blocks(theta)
    rng = torch.Generator(device=dev)
    rng.manual_seed(0)
    D = torch.randn((ctx.n, T), device=dev, dtype=torch.float32, generator=rng)
    Q = torch.empty_like(D)
    kv_ms = time_ms(lambda: ctx.nugpr_matvec_into(D, Q), args.kv_reps)
    pre_ms = time_ms(lambda: ctx.nugpr_precond_apply_into(D, Q), args.kv_reps)
    build_ms = time_ms(lambda: ctx.nugpr_build_blocks(theta), 5)
    sync()
    tf0 = time.perf_counter()
    ctx.nugpr_precond_factor()
    sync()
    factor_ms = (time.perf_counter() - tf0) * 1e3
    mll_t0 = time.perf_counter()
    res = ctx.nugpr_mll(theta)
    sync()
    mll_ms = (time.perf_counter() - mll_t0) * 1e3

    n, r, nc = ctx.n, ctx.rank, ctx.nc
    sizes = np.diff(w.offsets).astype(np.float64)
    dom_bytes = ctx.nugpr_profile_bytes(T)
    # one product K'.D with the default one-hot basis: the dominant launch (K_diag and C streamed once, D and
    # the S slabs read, Q and the P slabs written) + the projection S = W^T D (D read again, 8 bytes of index
    # per point) + the expansion Q += W P (Q read and written).  W itself is not streamed.
    vs = 8.0 if args.acc == "fp64" else 4.0
    kv_alg_bytes = dom_bytes + vs * 3.0 * n * T + 8.0 * n
    dom_avg_ms = dom_ms / max(dom_launches, 1)
    achieved = dom_bytes / (dom_avg_ms * 1e-3) / 1e9 if dom_launches else 0.0

    line = {
        "metric": "MLL evals/sec (block-LR K.V GB/s in kv_gbps / roofline), fp32 storage, t=%d, n=%d" % (ctx.t, n),
        "value": evals_per_s,
        "unit": "evals/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": total_s * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 storage, %s accumulate" % ("f64" if args.acc == "fp64" else "f32"),
        "data": "synthetic",
        "config": {"workload": "%s: n=%d, d=%d, %d clusters, r=%d, t=%d, tol=%g; one step = nugpr_train_step "
                               "(factor + %d loss evaluations + Adam)" % (args.config, n, ctx.d, nc, r, ctx.t,
                                                                          w.tol, 1 + 2 * p),
                   "acc": args.acc, "status_codes": codes, "step_ms": [round(x, 2) for x in step_ms]},
        "kv_gbps": kv_alg_bytes / (kv_ms * 1e-3) / 1e9,
        "kv_ms": kv_ms,
        "kv_algorithmic_bytes": kv_alg_bytes,
        "kv_frac_of_hbm_peak": kv_alg_bytes / (kv_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "precond_apply_ms": pre_ms,
        "build_blocks_ms": build_ms,
        "precond_factor_ms": factor_ms,
        "mll_ms": mll_ms,
        "mll_iters": res["max_iters_used"],
        "roofline": {"bound": "hbm", "kernel": "strip kernel (K_diag.D and C.S in one launch)",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((args.config, args.acc)),
                     "bytes_per_launch": dom_bytes, "avg_ms": dom_avg_ms, "launches_timed": dom_launches},
    }
    if args.cpu_clusters > 0:
        line["cpu_baseline"] = cpu_baseline(w, args.cpu_clusters)
    ctx.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
