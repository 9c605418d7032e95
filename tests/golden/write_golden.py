#!/usr/bin/env python3
"""Writes the oracle's objective/residual/step-size trajectories of the full-size workloads.

Calls only `oracle/` and the seeded input generators in `workloads/` (through tests/helpers.py);
nothing here touches the HIP library. The paper prints no worked numeric example of an update,
so these files are the stored expectations for the full-size trajectory tests:

    python tests/golden/write_golden.py C1 C2 C4

One text file per workload, `<name>_trajectory.txt`: a header with the recipe, then one line per
iteration k = 0..iters (k = 0 is the perturbed start) with
    k risk lin_pen act_pen dual_lin dual_quad F L_rho residual | tau_2..tau_L | theta_1..theta_L
Floating-point numbers are printed with 17 significant digits (round-trip exact for fp64).
"""
from __future__ import annotations

import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import pdadmm_oracle as O                      # noqa: E402
from tests.helpers import oracle_inputs, oracle_state     # noqa: E402
from workloads import get_workload                         # noqa: E402

KEYS = ("risk", "lin_pen", "act_pen", "dual_lin", "dual_quad", "F", "L_rho")


def line(k, st):
    ob = O.objective(st)
    res = O.residual(st)[0]
    nums = [ob[key] for key in KEYS] + [res]
    return (f"{k} " + " ".join(f"{v:.17g}" for v in nums) + " | " +
            " ".join(f"{t:.17g}" for t in st.tau[1:]) + " | " + " ".join(f"{t:.17g}" for t in st.theta))


def write(name: str) -> str:
    w = get_workload(name)
    t0 = time.time()
    inp = oracle_inputs(w)
    st = oracle_state(w, inp)          # forward-consistent start, perturbed, fp32-representable
    path = os.path.join(HERE, f"{name}_trajectory.txt")
    with open(path, "w") as f:
        f.write(f"# oracle trajectory of workload {name}: N={w.n_nodes} dims={w.dims[0]},{w.dims[1]}x{w.n_layers - 1},{w.dims[-1]} "
                f"rho={w.rho} nu={w.nu} quant={w.quant} iters={w.iters}; start = tests.helpers.oracle_state(w)\n")
        f.write("# k " + " ".join(KEYS) + " residual | tau_2..tau_L | theta_1..theta_L\n")
        f.write(line(0, st) + "\n")
        for k in range(1, w.iters + 1):
            O.iterate(st, 1)
            f.write(line(k, st) + "\n")
            f.flush()
            print(f"{name}: iteration {k}/{w.iters} done, {time.time() - t0:.0f} s", flush=True)
    return path


if __name__ == "__main__":
    for nm in sys.argv[1:] or ["C1", "C2"]:
        print(write(nm))
