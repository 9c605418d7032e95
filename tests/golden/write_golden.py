#!/usr/bin/env python3
"""Writes the oracle's objective/residual/step-size trajectories of the full-size workloads.

Calls only `oracle/` and the seeded input generators in `workloads/` (through tests/helpers.py);
nothing here touches the HIP library. The paper prints no worked numeric example of an update,
so these files are the stored expectations for the full-size trajectory tests:

    python tests/golden/write_golden.py C1 C2 C4
    python tests/golden/write_golden.py C3 C5 C5:plain      (hours on 8 cores; run in the background)

One text file per workload, `<name>_trajectory.txt`: a header with the recipe, then one line per
iteration k = 0..iters (k = 0 is the perturbed start) with
    k risk lin_pen act_pen dual_lin dual_quad F L_rho residual | tau_2..tau_L | theta_1..theta_L
Floating-point numbers are printed with 17 significant digits (round-trip exact for fp64).

C3 and C5 do not fit the host memory in fp64: they run in the oracle's memory-lean mode (variables
stored as fp32 between updates, every update computed in fp64), and, because one oracle iteration of
theirs takes a quarter of an hour on one core, with the updates of different layers of one phase running
side by side in forked child processes (`--workers N`; within a phase of Algorithm 1 the layers are
independent, every update is still the oracle's own function call, and a child hands back what its update
replaced). Processes, not threads: numpy's BLAS returns wrong products when large matrix products are
issued from several threads of one process at the same time. `<name>:plain` runs a -Q workload with
the plain backtracking schedule (every p-update starts at the previous tau divided by eta) instead of
the probe back-off and writes `<name>_plain_trajectory.txt`.
"""
from __future__ import annotations

import os
import sys
import time
import multiprocessing as mp
from multiprocessing.connection import wait as wait_for

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


LEAN = ("C3", "C5", "C5pq")     # state too large for fp64 storage on the host


PER_LAYER = ("W", "b", "z", "p", "q", "u", "tau", "theta", "p_trials", "w_trials", "p_wait", "p_skip")
_FORK = mp.get_context("fork")


def _run_update(conn, st, fn, i):
    """Child process: one update of one layer on the state as it was at the fork (shared copy-on-write); sends
    back every per-layer entry of position i that the update rebound (arrays) or may have changed (scalars)."""
    try:
        before = {f: getattr(st, f)[i] for f in PER_LAYER if i < len(getattr(st, f))}
        fn(st, i)
        out = {}
        for f, old in before.items():
            new = getattr(st, f)[i]
            if not hasattr(new, "shape") or new is not old:
                out[f] = new
        conn.send(out)
    except BaseException as e:          # the parent re-raises
        conn.send(e)
    finally:
        conn.close()


def run_phase(st, fn, layers, workers: int) -> None:
    """fn(st, i) for every i in `layers`, at most `workers` at a time, each in a forked child; the results are
    written into `st` as they arrive. The updates of one phase read and write disjoint variables (Algorithm 1)."""
    todo, running = list(layers), {}
    while todo or running:
        while todo and len(running) < workers:
            i = todo.pop(0)
            recv, send = _FORK.Pipe(duplex=False)
            proc = _FORK.Process(target=_run_update, args=(send, st, fn, i))
            proc.start()
            send.close()
            running[recv] = (proc, i)
        for recv in wait_for(list(running)):
            proc, i = running.pop(recv)
            got = recv.recv()
            recv.close()
            proc.join()
            if isinstance(got, BaseException):
                raise got
            for f, val in got.items():
                getattr(st, f)[i] = val


def iterate_layers_side_by_side(st, workers: int) -> None:
    """One iteration of Algorithm 1, phase after phase as O.iterate does it, with the per-layer updates of a
    phase spread over `workers` child processes."""
    L = st.L
    run_phase(st, O.update_p, range(1, L), workers)
    run_phase(st, O.update_W, range(L), workers)
    run_phase(st, O.update_b, range(L), workers)
    run_phase(st, O.update_z_hidden, range(L - 1), workers)
    O.update_z_last(st)
    run_phase(st, O.update_q, range(L - 1), workers)
    run_phase(st, O.update_u, range(L - 1), workers)


def write(spec: str, workers: int = 1, max_iters: int = 0) -> str:
    name, _, mode = spec.partition(":")
    if mode not in ("", "plain"):
        raise SystemExit(f"unknown mode {mode!r}")
    w = get_workload(name)
    lean = name in LEAN
    t0 = time.time()
    inp = oracle_inputs(w)
    kw = dict(store32=True) if lean else {}
    if mode == "plain":
        if w.quant is None:
            raise SystemExit("the plain schedule is the only one pdADMM-G has")
        kw["probe_backoff"] = False
    st = oracle_state(w, inp, **kw)    # forward-consistent start, perturbed, fp32-representable
    del inp
    print(f"{spec}: start state ready, {time.time() - t0:.0f} s", flush=True)
    path = os.path.join(HERE, f"{name}{'_plain' if mode else ''}_trajectory.txt")
    with open(path, "w") as f:
        f.write(f"# oracle trajectory of workload {name}: N={w.n_nodes} dims={w.dims[0]},{w.dims[1]}x{w.n_layers - 1},{w.dims[-1]} "
                f"rho={w.rho} nu={w.nu} quant={w.quant} iters={w.iters}; start = tests.helpers.oracle_state(w"
                f"{', store32=True' if lean else ''}{', probe_backoff=False' if mode else ''})"
                f"{'; variables stored as fp32 between updates, updates in fp64' if lean else ''}\n")
        f.write("# k " + " ".join(KEYS) + " residual | tau_2..tau_L | theta_1..theta_L\n")
        f.write(line(0, st) + "\n")
        f.flush()
        for k in range(1, (min(max_iters, w.iters) if max_iters else w.iters) + 1):
            if workers > 1:
                iterate_layers_side_by_side(st, workers)
            else:
                O.iterate(st, 1)
            f.write(line(k, st) + "\n")
            f.flush()
            print(f"{spec}: iteration {k}/{w.iters} done, {time.time() - t0:.0f} s", flush=True)
    return path


if __name__ == "__main__":
    args = sys.argv[1:]
    n_workers = 1
    if "--workers" in args:
        k = args.index("--workers")
        n_workers = int(args[k + 1])
        del args[k:k + 2]
    n_iters = 0                      # --iters K: stop after K iterations (an incomplete file says so by its length)
    if "--iters" in args:
        k = args.index("--iters")
        n_iters = int(args[k + 1])
        del args[k:k + 2]
    for nm in args or ["C1", "C2"]:
        print(write(nm, n_workers, n_iters))
