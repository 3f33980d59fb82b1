#!/usr/bin/env python3
"""Writes tests/golden/oracle_fullsize.json: loss values and a few central-difference
gradient components of the fp64 CPU oracle at the full benchmark sizes (configurations 3
and 4), which take minutes to tens of minutes on host cores and are therefore stored
instead of recomputed in every GPU test run.

Calls ONLY oracle/ and the seeded input generators; nothing from the HIP path.
Quantities follow eq. (loss function), eq. (logdet) and eq. (numerical gradient) of the
paper in the central-difference form on log(theta) (h = 1e-3), all evaluations sharing
the preconditioner factored at theta_0 and the same probes.

    python tests/golden/make_golden.py [C3 C4 ...]
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import nugpr_oracle as O            # noqa: E402
from paper_2510_12128_amd import inputs as I    # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_fullsize.json")


def run(name):
    w = I.make_config(name)
    t0 = time.time()
    prob = O.Problem(w.X, w.y, w.offsets, w.probes, w.rank)
    fac = O.Factor(prob, w.theta)
    base = O.mll(prob, fac, w.theta, w.tol, w.max_iter)
    print(name, "base", base["nll"], "iters", base["iters"].max(), "t %.0f s" % (time.time() - t0), flush=True)
    phi = np.log(w.theta)
    p = phi.shape[0]
    comps = {}
    for i in (0, p - 2, p - 1):
        e = np.zeros(p)
        e[i] = w.fd_step
        lp = O.mll(prob, fac, np.exp(phi + e), w.tol, w.max_iter)["nll"]
        lm = O.mll(prob, fac, np.exp(phi - e), w.tol, w.max_iter)["nll"]
        comps[str(i)] = (lp - lm) / (2 * w.fd_step)
        print(name, "grad", i, comps[str(i)], "t %.0f s" % (time.time() - t0), flush=True)
    return dict(config=name, n=w.n, theta=list(map(float, w.theta)), tol=w.tol, max_iter=w.max_iter,
                fd_step=w.fd_step, nll=base["nll"], quad=base["quad"], logdet=base["logdet"],
                logdet_precond=base["logdet_precond"], max_iters=int(base["iters"].max()), grad=comps)


if __name__ == "__main__":
    names = sys.argv[1:] or ["C3", "C4"]
    data = json.load(open(OUT)) if os.path.exists(OUT) else {}
    for nm in names:
        data[nm] = run(nm)
        with open(OUT, "w") as f:
            json.dump(data, f, indent=1, sort_keys=True)
            f.write("\n")
