#!/usr/bin/env python3
"""Benchmark of the nuGPR marginal-log-likelihood hot path on one MI355X.

A "step" is one pass of the whole hot path: nugpr_train_step = block assembly and
block-Jacobi factorisation at theta_0, then 1 + 2p loss evaluations (assembly, batched PCG
with the block-low-rank product and the preconditioner apply, SLQ log-determinant) for the
central-difference gradient, and the Adam update.

Protocol.  Every timed step starts from the SAME theta_0 (the configuration's hyperparameters):
Adam's update is computed, as part of the step, but not fed back, so the workload is stationary and
`value` does not depend on how many steps are timed.  PCG iterations per solve are printed next to it.
A second, labelled figure (`trajectory`) runs the same number of steps with Adam's update fed back,
as a training run would; it is context, not `value`.

`roofline` describes the dominant kernel, the launch that streams K_diag and the coupling matrix C once
per product, timed live with HIP events inside the timed steps on the stream the library launches on.
It is reported against BOTH ceilings it can meet: fp64 matrix arithmetic (2 T flops per stored entry) and
HBM.  The HBM side is given three ways, each labelled: the bytes that physically cross HBM (hardware
counters, read from the committed profile summary if and only if that summary names the kernel that is
running), the bytes of the lower tiles the launch streams (what the code requests from memory), and the
dense-equivalent figure with full squares.  `bound` names the ceiling the kernel sits closer to.

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
FP64_MATRIX_PEAK_TFLOPS = 78.6


def measured_traffic(config, acc, kernel):
    """HBM bytes per launch of the dominant kernel from the committed counter summary
    (profiles/k_strip_<config>_<acc>_hbm_traffic.md: FETCH_SIZE + WRITE_SIZE of two rocprofv3 --pmc runs,
    scaled by the copy probe).  The summary carries one machine-readable line naming the kernel
    instantiation and the commit it was measured at; the figure is used only if that kernel is the one
    this run launches."""
    path = os.path.join(ROOT, "profiles", "k_strip_%s_%s_hbm_traffic.md" % (config, acc))
    if not os.path.exists(path):
        return None, "no counter summary for this workload under profiles/"
    rec = None
    for ln in open(path):
        ln = ln.strip()
        if ln.startswith('{"nugpr_profile"'):
            rec = json.loads(ln)
            break
    if rec is None:
        return None, "the counter summary has no machine-readable record"
    if rec.get("kernel") != kernel:
        return None, "the counter summary is for %s, this run launches %s" % (rec.get("kernel"), kernel)
    return rec, "profiles/%s (measured at commit %s)" % (os.path.basename(path), rec.get("commit"))


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
                        f"to the full workload (extrapolated, not measured at full size); oracle nll on the "
                        f"sample {out['nll']:.6e}"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C4")
    ap.add_argument("--acc", choices=["fp64", "fp32"], default="fp64",
                    help="arithmetic of the operator applications over the fp32 stored matrices")
    ap.add_argument("--cpu-clusters", type=int, default=-1,
                    help="clusters in the CPU-oracle sample (0 = skip; default: as many leading clusters as "
                         "hold 2e8 covariance entries, about 10 - 20 s of host time)")
    ap.add_argument("--kv-reps", type=int, default=20)
    ap.add_argument("--no-trajectory", action="store_true", help="skip the second (Adam fed back) run")
    ap.add_argument("--compensate", action="store_true",
                    help="solve with the compensated operator K'' of eqs. (krep), (kypp) (needed where the "
                         "uncompensated K' is not positive definite: configuration 5)")
    ap.add_argument("--precond-compensated", action="store_true",
                    help="with --compensate: precondition with the factor of the diagonal blocks of K'' itself "
                         "(NUGPR_PRECOND_COMPENSATED) instead of the paper's factor of K_diag")
    ap.add_argument("--max-iter", type=int, default=0, help="PCG iteration limit (0 = the configuration's own)")
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
    max_iter = args.max_iter if args.max_iter > 0 else w.max_iter
    ctx = Context(w.X, w.y, w.offsets, w.probes, w.rank, tol=w.tol, max_iter=max_iter, fd_step=w.fd_step,
                  lr=w.lr, isotropic=w.isotropic, device=dev, acc_fp32=(args.acc == "fp32"),
                  compensate=args.compensate, precond_compensated=args.precond_compensated)
    p, T = ctx.p, ctx.T
    phi0 = np.log(w.theta)
    zeros = np.zeros(p)

    def sync():
        torch.cuda.synchronize(dev)

    def per_step(stats, steps):
        s = max(steps, 1)
        return {"loss_evals": stats["loss_evals"] / s,
                "pcg_iters_per_solve": stats["pcg_iterations"] / max(stats["pcg_solves"], 1),
                "pcg_iters_max": stats["pcg_iterations_max"],
                "products": stats["products"] / s, "products_reused": stats["products_reused"] / s,
                "precond_applies": stats["precond_applies"] / s,
                "assembly_passes": stats["assembly_passes"] / s,
                "matrices_assembled": stats["matrices_assembled"] / s,
                "factorisations": stats["factorisations"] / s}

    # ---- the timed region: `steps` train steps, every one from theta_0 ----
    for _ in range(args.warmup):
        ctx.nugpr_train_step(phi0, zeros, zeros, 0)
    ctx.nugpr_profile_enable(True)
    ctx.nugpr_stats_read(reset=True)
    sync()
    t0 = time.perf_counter()
    codes, step_ms = [], []
    for _ in range(args.steps):
        ts = time.perf_counter()
        out = ctx.nugpr_train_step(phi0, zeros, zeros, 0)      # returns after the step's last synchronisation
        step_ms.append((time.perf_counter() - ts) * 1e3)
        codes.append(out["code"])
    sync()
    t1 = time.perf_counter()
    dom_ms, dom_launches = ctx.nugpr_profile_read()
    ctx.nugpr_profile_enable(False)
    stats = ctx.nugpr_stats_read(reset=True)
    total_s = t1 - t0
    evals = stats["loss_evals"]             # = steps * (1 + 2 p) when every step ends with status 0
    evals_per_s = evals / total_s

    # ---- second figure: the same number of steps with Adam's update fed back (a training run) ----
    trajectory = None
    if not args.no_trajectory:
        phi, m, v, step = phi0.copy(), np.zeros(p), np.zeros(p), 0
        sync()
        tt0 = time.perf_counter()
        tr_ms, tr_codes = [], []
        for _ in range(args.steps):
            ts = time.perf_counter()
            out = ctx.nugpr_train_step(phi, m, v, step)
            tr_ms.append((time.perf_counter() - ts) * 1e3)
            phi, m, v, step = out["log_theta"], out["adam_m"], out["adam_v"], out["step"]
            tr_codes.append(out["code"])
            if out["code"] not in (0, 3):
                break
        sync()
        tt1 = time.perf_counter()
        tstats = ctx.nugpr_stats_read(reset=True)
        done = len(tr_ms)
        trajectory = {"what": "the same steps with Adam's update fed back (theta moves; later solves need more "
                              "PCG iterations); context only, not `value`",
                      "evals_per_s": tstats["loss_evals"] / (tt1 - tt0), "ms_per_step": (tt1 - tt0) * 1e3 / done,
                      "step_ms": [round(x, 2) for x in tr_ms], "status_codes": tr_codes,
                      "per_step": per_step(tstats, done)}

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

    theta = w.theta
    ctx.nugpr_build_blocks(theta)
    rng = torch.Generator(device=dev)
    rng.manual_seed(0)
    D = torch.randn((ctx.n, T), device=dev, dtype=torch.float32, generator=rng)
    Q = torch.empty_like(D)
    kv_ms = time_ms(lambda: ctx.nugpr_matvec_into(D, Q), args.kv_reps)
    build_ms = time_ms(lambda: ctx.nugpr_build_blocks(theta), 5)
    sync()
    tf0 = time.perf_counter()
    ctx.nugpr_precond_factor()
    sync()
    factor_ms = (time.perf_counter() - tf0) * 1e3
    pre_ms = time_ms(lambda: ctx.nugpr_precond_apply_into(D, Q), args.kv_reps)
    mll_t0 = time.perf_counter()
    res = ctx.nugpr_mll(theta)
    sync()
    mll_ms = (time.perf_counter() - mll_t0) * 1e3

    n, r, nc = ctx.n, ctx.rank, ctx.nc
    sizes = np.diff(w.offsets).astype(np.float64)
    ncr = float(nc * r)
    vs = 8.0 if args.acc == "fp64" else 4.0
    kernel = ctx.nugpr_profile_kernel_name(T)
    lower_only = "true" in kernel.split(",")[3] if kernel.startswith("k_strip_ring") else False
    # --- bytes of one launch of the dominant kernel, three accountings ---
    entries_full = float(np.sum(sizes ** 2) + ncr ** 2)                      # stored entries, whole squares
    tiles = np.ceil(sizes / 64.0)
    ct = np.ceil(ncr / 64.0)
    entries_lower = float(np.sum(tiles * (tiles + 1) / 2) + ct * (ct + 1) / 2) * 4096.0   # lower 64 x 64 tiles
    vec_bytes = ctx.nugpr_profile_bytes(T) - 4.0 * entries_full             # D, S slabs in; Q, P slabs out
    bytes_full = 4.0 * entries_full + vec_bytes                               # dense-equivalent (every entry once)
    bytes_lower = 4.0 * entries_lower + vec_bytes                             # what the launch streams when it pairs tiles
    flops = 2.0 * T * entries_full                                            # every entry meets every column
    dom_avg_ms = dom_ms / max(dom_launches, 1)
    sec = dom_avg_ms * 1e-3
    rec, traffic_note = measured_traffic(args.config, args.acc, kernel)
    traffic = (rec["fetch_bytes_per_launch"] + rec["write_bytes_per_launch"]) if rec else None
    tflops = flops / sec / 1e12 if dom_launches else 0.0
    frac_mfma = tflops / FP64_MATRIX_PEAK_TFLOPS if args.acc == "fp64" else None
    requested = bytes_lower if lower_only else bytes_full
    frac_hbm_physical = (traffic / sec / 1e9 / HBM_PEAK_GBPS) if (traffic and dom_launches) else None
    frac_hbm_requested = requested / sec / 1e9 / HBM_PEAK_GBPS if dom_launches else 0.0
    hbm_side = {"physical_bytes": traffic, "physical_gbps": traffic / sec / 1e9 if traffic else None,
                "physical_frac": frac_hbm_physical, "physical_source": traffic_note,
                "streamed_bytes": requested, "streamed_gbps": requested / sec / 1e9,
                "streamed_frac": frac_hbm_requested,
                "streamed_what": ("lower 64x64 tiles of K_diag and C + vector blocks" if lower_only else
                                  "whole squares of K_diag and C + vector blocks"),
                "dense_equivalent_bytes": bytes_full, "dense_equivalent_gbps": bytes_full / sec / 1e9,
                "dense_equivalent_frac": bytes_full / sec / 1e9 / HBM_PEAK_GBPS,
                "peak_gbps": HBM_PEAK_GBPS}
    hbm_best = frac_hbm_physical if frac_hbm_physical is not None else frac_hbm_requested
    if frac_mfma is not None and frac_mfma >= hbm_best:
        roof = {"bound": "mfma", "achieved": tflops, "peak": FP64_MATRIX_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": frac_mfma, "dtype": "f64"}
    else:
        gb = (traffic if traffic else requested) / sec / 1e9
        roof = {"bound": "hbm", "achieved": gb, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": hbm_best}
    roof.update({"traffic": traffic, "kernel": kernel + " (K_diag.D and C.S in one launch)",
                 "flops_per_launch": flops, "avg_ms": dom_avg_ms, "launches_timed": dom_launches,
                 "mfma_f64_frac": frac_mfma, "hbm": hbm_side})

    # one product K'.D through the C ABI (fp32 blocks in and out) with the default one-hot basis: the dominant
    # launch + the projection S = W^T D (fp32 D read, 8 bytes of index per point, fp64 copy written) + the
    # expansion Q = Q_diag + W P (fp64 block read, fp32 Q written).  W itself is not streamed.
    kv_extra = (4.0 + vs) * n * T + 8.0 * n + (vs + 4.0) * n * T
    kv_bytes_full = bytes_full + kv_extra
    kv_bytes_streamed = requested + kv_extra
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
                   "protocol": "every timed step starts from theta_0 (Adam's update is computed, not fed back)",
                   "acc": args.acc, "operator": ("K'' (compensated, eq. (kypp))" + (", preconditioned by the factor of its own diagonal blocks"
                                                                   if args.precond_compensated else "")) if args.compensate else
                   "K' (eq. (odsplit))", "max_iter": max_iter, "status_codes": codes, "step_ms": [round(x, 2) for x in step_ms],
                   "per_step": per_step(stats, args.steps)},
        "pcg_iters_per_solve": stats["pcg_iterations"] / max(stats["pcg_solves"], 1),
        "kv_ms": kv_ms,
        "kv_what": "nugpr_matvec through the C ABI, fp32 blocks in and out, %d columns, median-free mean of %d "
                   "back-to-back calls" % (T, args.kv_reps),
        "kv_gbps": kv_bytes_full / (kv_ms * 1e-3) / 1e9,
        "kv_algorithmic_bytes": kv_bytes_full,
        "kv_frac_of_hbm_peak": kv_bytes_full / (kv_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "kv_accounting": "full squares of K_diag and C streamed once + vector blocks (dense-equivalent; the "
                         "launch itself streams the lower tiles only, see kv_streamed_*)",
        "kv_streamed_bytes": kv_bytes_streamed,
        "kv_streamed_frac_of_hbm_peak": kv_bytes_streamed / (kv_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "precond_apply_ms": pre_ms,
        "build_blocks_ms": build_ms,
        "precond_factor_ms": factor_ms,
        "mll_ms": mll_ms,
        "mll_iters": res["max_iters_used"],
        "roofline": roof,
    }
    if trajectory is not None:
        line["trajectory"] = trajectory
    if args.cpu_clusters != 0:
        k = args.cpu_clusters
        if k < 0:               # bounded sample: leading clusters holding at most 2e8 entries of K_diag
            k = max(1, int(np.searchsorted(np.cumsum(sizes ** 2), 2.05e8, side="right")))
        line["cpu_baseline"] = cpu_baseline(w, k)
    ctx.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
