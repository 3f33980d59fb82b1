#!/usr/bin/env python3
"""Writes tests/golden/oracle_fullsize.json: values of the fp64 CPU oracle at the full benchmark
sizes, which take minutes to hours on host cores and are therefore stored instead of recomputed in
every GPU test run.

Calls ONLY oracle/ and the seeded input generators; nothing from the HIP path.
Quantities follow eq. (loss function), eq. (logdet) and eq. (numerical gradient) of the
paper in the central-difference form on log(theta) (h = 1e-3), all evaluations sharing
the preconditioner factored at theta_0 and the same probes.

    python tests/golden/make_golden.py [C3 C4 C3-adam20 C3c-adam20 C3p-adam20 ...] [--workers N] [--steps K]

  C3, C4       base loss + central-difference gradient components (several lengthscales, the output
               scale, the noise) at the configured hyperparameters
  C3c-adam20   the same 20 steps with the compensated operator K'' of eqs. (krep), (kypp), which stays
               positive definite when the lengthscales grow (the uncompensated K' of C3-adam20 does not:
               that record ends with the step at which the oracle finds it indefinite)
  C3p-adam20   the same with K'' preconditioned by the factor of its own diagonal blocks (the oracle's
               Factor(compensated_blocks=True)): the same losses up to the stochastic log-determinant estimate, far
               fewer PCG iterations, so all 20 steps are affordable
  C3-adam20    configuration 3's own workload: 20 passes of Algorithm 1's loop body (factor at theta_0,
               base loss, central differences with that factor and the same probes, Adam with
               gamma = 0.05 on log theta); per step the base loss, the whole gradient and the
               updated log theta are stored.  Each step is Factor -> mll -> (mll+ - mll-)/2h -> adam_step,
               the composition the oracle's train_step makes; the 2p difference evaluations of a step
               are independent and are handed to worker processes (forked after the factorisation, so
               the factor is shared), which changes no arithmetic.
"""
import json
import multiprocessing as mp
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import nugpr_oracle as O            # noqa: E402
from paper_2510_12128_amd import inputs as I    # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_fullsize.json")

# which gradient components are stored for the single-point entries: the first three lengthscales,
# the output scale, the noise
def stored_components(p):
    return sorted({0, 1, 2, p - 2, p - 1} & set(range(p)))


_STATE = {}


def _loss_at(phi):
    """Worker body: one oracle loss evaluation at exp(phi) with the factor the parent built."""
    s = _STATE
    try:
        return float(O.mll(s["prob"], s["fac"], np.exp(np.asarray(phi)), s["tol"], s["max_iter"])["nll"])
    except ValueError as e:               # the oracle's verdict "indefinite"
        return str(e)


def losses(phis, workers):
    if workers <= 1:
        return [_loss_at(p) for p in phis]
    with mp.get_context("fork").Pool(workers) as pool:
        return pool.map(_loss_at, [list(map(float, p)) for p in phis], chunksize=1)


def run_point(name, workers):
    w = I.make_config(name)
    t0 = time.time()
    prob = O.Problem(w.X, w.y, w.offsets, w.probes, w.rank)
    fac = O.Factor(prob, w.theta)
    _STATE.update(prob=prob, fac=fac, tol=w.tol, max_iter=w.max_iter)
    base = O.mll(prob, fac, w.theta, w.tol, w.max_iter)
    print(name, "base", base["nll"], "iters", base["iters"].max(), "t %.0f s" % (time.time() - t0), flush=True)
    phi = np.log(w.theta)
    p = phi.shape[0]
    comps = stored_components(p)
    pts = []
    for i in comps:
        e = np.zeros(p)
        e[i] = w.fd_step
        pts += [phi + e, phi - e]
    vals = losses(pts, workers)
    grad = {}
    for k, i in enumerate(comps):
        grad[str(i)] = (vals[2 * k] - vals[2 * k + 1]) / (2 * w.fd_step)
        print(name, "grad", i, grad[str(i)], "t %.0f s" % (time.time() - t0), flush=True)
    return dict(config=name, n=w.n, theta=list(map(float, w.theta)), tol=w.tol, max_iter=w.max_iter,
                fd_step=w.fd_step, nll=base["nll"], quad=base["quad"], logdet=base["logdet"],
                logdet_precond=base["logdet_precond"], max_iters=int(base["iters"].max()), grad=grad)


def run_adam(name, steps, workers, save, compensate=False, own_blocks=False):
    w = I.make_config(name)
    prob = O.Problem(w.X, w.y, w.offsets, w.probes, w.rank, compensate=compensate)
    phi = np.log(w.theta)
    p = phi.shape[0]
    m, v, step = np.zeros(p), np.zeros(p), 0
    rec = dict(config=name, n=w.n, theta0=list(map(float, w.theta)), tol=w.tol, max_iter=w.max_iter,
               fd_step=w.fd_step, lr=w.lr, compensate=bool(compensate), precond_compensated=bool(own_blocks),
               steps_requested=steps, steps=[])
    t0 = time.time()
    for it in range(steps):
        fac = O.Factor(prob, np.exp(phi), compensated_blocks=own_blocks)
        _STATE.update(prob=prob, fac=fac, tol=w.tol, max_iter=w.max_iter)
        pts = [phi]
        for i in range(p):
            e = np.zeros(p)
            e[i] = w.fd_step
            pts += [phi + e, phi - e]
        vals = losses(pts, workers)
        if any(isinstance(x, str) for x in vals):
            rec["stopped"] = dict(step=it, reason=[x for x in vals if isinstance(x, str)][0])
            print(name, "step", it, "stopped:", rec["stopped"], flush=True)
            save(rec)
            break
        nll0 = vals[0]
        g = np.array([(vals[1 + 2 * i] - vals[2 + 2 * i]) / (2 * w.fd_step) for i in range(p)])
        phi, m, v, step = O.adam_step(phi, g, m, v, step, lr=w.lr)
        rec["steps"].append(dict(nll0=nll0, grad=list(map(float, g)), log_theta=list(map(float, phi))))
        print(name, "step", it, "nll0", nll0, "|g|", float(np.linalg.norm(g)), "t %.0f s" % (time.time() - t0),
              flush=True)
        save(rec)
    return rec


if __name__ == "__main__":
    args = sys.argv[1:]
    workers, nsteps = 1, 20
    if "--workers" in args:
        k = args.index("--workers")
        workers = int(args[k + 1])
        del args[k:k + 2]
    if "--steps" in args:                  # fewer than the 20 steps of the workload (recorded as steps_requested)
        k = args.index("--steps")
        nsteps = int(args[k + 1])
        del args[k:k + 2]
    names = args or ["C3", "C4"]
    data = json.load(open(OUT)) if os.path.exists(OUT) else {}

    def write():
        with open(OUT, "w") as f:
            json.dump(data, f, indent=1, sort_keys=True)
            f.write("\n")

    for nm in names:
        if nm.endswith("-adam20"):
            def save(rec, key=nm):
                data[key] = rec
                write()
            base = nm[:-len("-adam20")]
            own = base.endswith("p")                # "C3p-adam20": K'' and the factor of its own diagonal blocks
            comp = own or base.endswith("c")        # "C3c-adam20": the compensated operator of eqs. (krep), (kypp)
            run_adam(base[:-1] if comp else base, nsteps, workers, save, compensate=comp, own_blocks=own)
        else:
            data[nm] = run_point(nm, workers)
            write()
