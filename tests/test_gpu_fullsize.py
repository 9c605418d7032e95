"""Full-size parity: the HIP path at the sizes and in the launch configuration bench.py times.

Two kinds of checks:
  * trajectories of C1, C2, C4 (all layers, 10/20 iterations) against the oracle's stored trajectories
    in tests/golden/ (written by tests/golden/write_golden.py, which calls only the oracle), plus an
    element-by-element comparison of every variable with the live oracle after the first iteration
    (C1, C2);
  * C3, C4, C5 (too large for the fp64 oracle to hold whole): one iteration with seeded generic values
    placed around sampled layers (first, middle, last); the oracle computes those layers' updates
    one by one from the same host arrays (layers are independent within an iteration, Algorithm 1),
    and every variable of the layer is compared element by element.
Tolerances are the ones fixed for this build: rel-L2 <= 1e-4 per variable after one iteration,
objective/residual within 1e-3; step sizes and trial counts exact; -Q indices at most one level off
at isolated elements.
"""
import os
import time

import numpy as np
import pytest

from oracle import pdadmm_oracle as O
from tests.helpers import F32, F64, grid_of, oracle_inputs, oracle_state, rel_l2
from workloads import (get_workload, layer_window, make_features, make_graph, make_labels, make_weights,
                       stream_rng)

pytestmark = pytest.mark.gpu

TOL_STATE = 1e-4
TOL_TRAJ = 1e-3
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
KEYS = ("risk", "lin_pen", "act_pen", "dual_lin", "dual_quad", "F", "L_rho")


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2105_09837_amd as P
    from tests import gpu_helpers as H
    assert torch.cuda.is_available()
    P.load_library()
    return torch, P, H


@pytest.fixture
def say(capsys):
    """Progress lines that reach the terminal even under output capture (long tests must not look hung)."""
    t0 = time.time()

    def _say(msg):
        with capsys.disabled():
            print(f"\n    [{time.time() - t0:6.1f} s] {msg}", end="", flush=True)
    return _say


def read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, f"{name}_trajectory.txt")) as f:
        for ln in f:
            if ln.startswith("#"):
                continue
            head, taus, thetas = ln.split("|")
            h = head.split()
            rows.append(dict(k=int(h[0]), **{key: float(v) for key, v in zip(KEYS + ("residual",), h[1:])},
                             tau=[float(x) for x in taus.split()], theta=[float(x) for x in thetas.split()]))
    return rows


# ------------------------------------------------------------------------------ trajectories
def _golden_file(name):
    return os.path.join(GOLDEN, f"{name}_trajectory.txt")


LEAN = ("C3", "C5")      # written by the oracle's memory-lean mode (fp32 storage, fp64 updates): see write_golden.py


@pytest.mark.parametrize("name,live_first", [("C1", True), ("C2", True), ("C4", False), ("C3", False), ("C5", False),
                                             ("C5_plain", False)])
def test_full_size_trajectory_against_stored_oracle_run(env, say, name, live_first):
    """All layers, every iteration of the stored oracle run: objective terms and residual within 1e-3, step
    sizes exactly. C3 and C5 start from the memory-lean oracle state the stored run started from.
    C5 (-Q; `C5_plain`: plain backtracking schedule): the projection onto Delta is discontinuous, and where
    a projected value sits within rounding of a midpoint the fp32 products of the HIP path and the fp64
    products of the oracle land on neighbouring members (about 20 of 1e8 elements per layer and iteration,
    each validated in test_full_size_sampled_layer_one_iteration; the small free-running case shows by
    re-running the oracle from the GPU's own state that nothing else separates the runs). Such flips cannot
    be followed by the oracle at this size, so for C5 the 1e-3 bound and the exact step sizes are required
    up to the first iteration at which a step size differs, which must not come before the second half of the
    run; after it the two runs are two valid runs of the algorithm and only finiteness is asserted."""
    torch, P, H = env
    workload = name.split("_")[0]
    plain = name.endswith("_plain")
    if not os.path.exists(_golden_file(name)):
        pytest.skip(f"tests/golden/{name}_trajectory.txt has not been written (hours of oracle time): "
                    f"python tests/golden/write_golden.py {workload}{':plain' if plain else ''}")
    w = get_workload(workload)
    gold = read_golden(name)
    n_iters = len(gold) - 1
    if n_iters < 1:
        pytest.skip(f"tests/golden/{name}_trajectory.txt holds no iteration yet (it is being written)")
    assert n_iters == w.iters or workload in LEAN, "stored trajectory is incomplete"
    lean = workload in LEAN
    say(f"{name}: inputs and oracle start state ({'fp32-stored, ' if lean else ''}{n_iters} stored iterations)")
    inp = oracle_inputs(w)
    if lean:
        st = oracle_state(w, inp, store32=True, probe_backoff=not plain)
    else:
        st = H.round_state_to_fp32(oracle_state(w, inp))
        # the stored run started from these very values
        o0 = O.objective(st)
        assert abs(o0["L_rho"] - gold[0]["L_rho"]) <= 1e-9 * abs(gold[0]["L_rho"])
    ctx = H.gpu_context(w, inp, st)
    del inp
    if lean:      # (the literal oracle objective takes minutes here: the GPU's own, accurate to fp32 rounding)
        o0 = P.pdadmm_objective(ctx)
        assert abs(o0["L_rho"] - gold[0]["L_rho"]) <= 1e-5 * abs(gold[0]["L_rho"]), (o0["L_rho"], gold[0]["L_rho"])
        assert abs(P.pdadmm_residual(ctx)[0] - gold[0]["residual"]) <= 1e-5 * gold[0]["residual"]
    st_start = st.copy() if live_first else None
    if not live_first:
        del st
    L = w.n_layers
    worst = 0.0
    diverged_at = None
    for k in range(1, n_iters + 1):
        P.pdadmm_iterate(ctx, 1)
        og = P.pdadmm_objective(ctx)
        rg = P.pdadmm_residual(ctx)[0]
        g = gold[k]
        tau, theta, _, _ = H.step_sizes(ctx)
        same_steps = [float(t) for t in tau[1:L]] == g["tau"] and [float(t) for t in theta[:L]] == g["theta"]
        errs = {key: abs(og[key] - g[key]) / max(abs(g[key]), 1e-12) for key in ("risk", "lin_pen", "act_pen", "dual_quad", "F", "L_rho")}
        errs["dual_lin"] = abs(og["dual_lin"] - g["dual_lin"]) / max(abs(g["dual_lin"]), abs(g["dual_quad"]), 1e-12)
        errs["residual"] = abs(rg - g["residual"]) / g["residual"]
        if w.quant is not None:
            say(f"{name} it {k}: worst error {max(errs.values()):.1e}, step sizes {'equal' if same_steps else 'DIFFER'}")
        if diverged_at is None and w.quant is not None and not same_steps:
            diverged_at = k
            say(f"{name}: a step size differs from iteration {k} on: two valid runs of the algorithm from here")
            for l in range(2, L + 1):
                if float(tau[l - 1]) != g["tau"][l - 2]:
                    say(f"{name}:   tau_{l}: HIP path {float(tau[l - 1])}, stored run {g['tau'][l - 2]}")
            for l in range(1, L + 1):
                if float(theta[l - 1]) != g["theta"][l - 1]:
                    say(f"{name}:   theta_{l}: HIP path {float(theta[l - 1])}, stored run {g['theta'][l - 1]}")
        if diverged_at is None:
            assert same_steps, (k, "tau/theta", list(tau), g["tau"], list(theta), g["theta"])
            for key, e in errs.items():
                worst = max(worst, e)
                assert e <= TOL_TRAJ, (k, key, e)
        else:
            assert np.isfinite(og["L_rho"]) and np.isfinite(rg)
        if k == 1 and live_first:
            say(f"{name}: oracle iteration 1 (live), element-by-element comparison")
            O.iterate(st, 1)
            ok, w_state, rep = H.compare_state(ctx, st, TOL_STATE, what=f"{name} it 1", before=st_start)
            assert ok, rep
            say(f"{name}: worst rel-L2 after one iteration {w_state:.2e}")
    assert diverged_at is None or diverged_at > n_iters // 2, f"step sizes differ from iteration {diverged_at} on"
    s = P.pdadmm_stats(ctx, drift=True)
    say(f"{name}: {n_iters} iterations, worst objective/residual error {worst:.2e}"
        + (f" (up to iteration {diverged_at - 1})" if diverged_at else "") + f", carried-residual drift {s['r_drift']:.2e}")
    assert s["r_drift"] < 1e-4
    P.pdadmm_destroy(ctx)


# ------------------------------------------------------------------------------ sampled layers at full size
class _Problem:
    """One full-size context per workload, built with the HIP library only (like bench.py)."""

    def __init__(self, torch, P, w):
        dev = torch.device("cuda:0")
        rp, ci = make_graph(w.graph, w.n_nodes, w.graph_param, stream_rng(w, 0))
        self.rp, self.ci = rp, ci
        a_rp, a_ci, a_v = P.pdadmm_normalize_adj(rp, ci)
        self.X = make_features(w)
        Xa = P.pdadmm_augment(torch.from_numpy(a_rp).to(dev), torch.from_numpy(a_ci).to(dev),
                              torch.from_numpy(a_v).to(dev), torch.from_numpy(self.X).to(dev), w.hops)
        Ws, bs = make_weights(w)
        self.y = make_labels(w)
        q = w.quant
        cfg = P.Config(n_nodes=w.n_nodes, dims=list(w.dims), rho=w.rho, nu=w.nu, quantize=(2 if w.quant_q else 1) if q else 0,
                       q_lo=q[0] if q else -1.0, q_hi=q[1] if q else 1.0, q_levels=q[2] if q else 256)
        self.ctx = P.pdadmm_init(cfg, Xa, torch.from_numpy(self.y).to(dev), [torch.from_numpy(a).to(dev) for a in Ws],
                                 [torch.from_numpy(a).to(dev) for a in bs])
        self.w = w


_problems = {}


def _problem(torch, P, name):
    if name not in _problems:
        for k in list(_problems):          # one full-size context at a time
            P.pdadmm_destroy(_problems.pop(k).ctx)
        torch.cuda.empty_cache()
        _problems[name] = _Problem(torch, P, get_workload(name))
    return _problems[name]


def _window_state(w, layer, win, X_aug, y):
    """Oracle State holding only what the updates of layer `layer` (and the p-update of the layer above)
    read: slot order [below (q, u only)] [layer] [above]. Returns (state, index of the layer)."""
    L = w.n_layers
    has_prev, has_next = layer >= 2, layer < L
    i = 1 if has_prev else 0
    n = i + 1 + (1 if has_next else 0)
    none = [None] * n
    st = O.State(W=list(none), b=list(none), z=list(none), p=list(none), q=[None] * (n - 1), u=[None] * (n - 1),
                 y=y, mask=None, rho=float(w.rho), nu=float(w.nu), grid=grid_of(w), tau=[1.0] * n, theta=[1.0] * n,
                 p_trials=[0] * n, w_trials=[0] * n, p_wait=[0] * n, p_skip=[0] * n)
    d64 = lambda a: np.asarray(a, dtype=F64)
    st.W[i], st.b[i], st.z[i] = d64(win["W"]), d64(win["b"]), d64(win["z"])
    st.p[i] = d64(win["p"]) if has_prev else d64(X_aug)
    if has_prev:
        st.q[i - 1], st.u[i - 1] = d64(win["q_prev"]), d64(win["u_prev"])
    if has_next:
        st.q[i], st.u[i] = d64(win["q"]), d64(win["u"])
        st.W[i + 1], st.b[i + 1], st.z[i + 1], st.p[i + 1] = (d64(win[k]) for k in ("W_next", "b_next", "z_next", "p_next"))
    return st, i


# every distinct layer shape of the three large workloads (C5's inner layers all have the shape of layer 2).
# Third entry, -Q only: the probe state {wait, left} the p-updates start from. From (0, 0) the update starts at
# tau/eta, which is what the plain schedule does in every update (one iteration of the two schedules from that
# state is the same sequence of trials; they differ in the bookkeeping afterwards, which the small cases check in
# both modes); from (2, 1) the back-off schedule skips the probe and starts at tau itself.
WINDOWS = [("C4", 1, None), ("C4", 26, None), ("C4", 50, None), ("C3", 1, None), ("C3", 5, None), ("C3", 10, None),
           ("C5", 2, (0, 0)), ("C5", 16, (2, 1)),
           ("C5x16", 9, (0, 0))]        # Delta of 65536 levels: p_l resident as 16-bit indices


@pytest.mark.parametrize("name,layer,probe", WINDOWS)
def test_full_size_sampled_layer_one_iteration(env, say, name, layer, probe):
    torch, P, H = env
    w = get_workload(name)
    L = w.n_layers
    say(f"{name} layer {layer}/{L}: N={w.n_nodes} {w.dims[layer - 1]}->{w.dims[layer]}: context")
    prob = _problem(torch, P, name)
    ctx = prob.ctx
    g = grid_of(w)
    quant = (lambda a: O.quantize(a, g)[1]) if g is not None else None
    win = layer_window(w, layer, quantizer=quant)
    V = P.VAR
    # the same host arrays go to the GPU ...
    P.pdadmm_set_var(ctx, V.W, layer, win["W"]); P.pdadmm_set_var(ctx, V.B, layer, win["b"])
    P.pdadmm_set_var(ctx, V.Z, layer, win["z"]); P.pdadmm_set_var(ctx, V.THETA, layer, 1.0)
    if layer >= 2:
        P.pdadmm_set_var(ctx, V.P, layer, win["p"]); P.pdadmm_set_var(ctx, V.TAU, layer, 1.0)
        if g is not None:
            P.pdadmm_set_var(ctx, V.PROBE, layer, probe)
        P.pdadmm_set_var(ctx, V.Q, layer - 1, win["q_prev"]); P.pdadmm_set_var(ctx, V.U, layer - 1, win["u_prev"])
    if layer < L:
        P.pdadmm_set_var(ctx, V.Q, layer, win["q"]); P.pdadmm_set_var(ctx, V.U, layer, win["u"])
        P.pdadmm_set_var(ctx, V.W, layer + 1, win["W_next"]); P.pdadmm_set_var(ctx, V.B, layer + 1, win["b_next"])
        P.pdadmm_set_var(ctx, V.Z, layer + 1, win["z_next"]); P.pdadmm_set_var(ctx, V.P, layer + 1, win["p_next"])
        P.pdadmm_set_var(ctx, V.TAU, layer + 1, 1.0)
        if g is not None:
            P.pdadmm_set_var(ctx, V.PROBE, layer + 1, probe)
    # ... and to the oracle
    X_aug = None
    if layer == 1:
        say("oracle augmentation (p_1 = X_aug)")
        arp, aci, av = O.normalize_adj(prob.rp, prob.ci)
        X_aug = O.augment(arp, aci, av, prob.X, w.hops)
        assert np.array_equal(P.pdadmm_get_var(ctx, V.P, 1).view(np.uint32), X_aug.view(np.uint32))
    st, i = _window_state(w, layer, win, X_aug, prob.y)
    if g is not None:
        st.p_wait, st.p_skip = [probe[0]] * len(st.W), [probe[1]] * len(st.W)
    del win
    say("GPU iteration")
    P.pdadmm_iterate(ctx, 1)
    P.pdadmm_sync(ctx)
    tau, theta, pt, wt = H.step_sizes(ctx)
    def check(what, kind, lay, ref, skip=None):
        got = P.pdadmm_get_var(ctx, kind, lay)
        e = rel_l2(got, ref) if skip is None or not skip.any() else rel_l2(got[~skip], ref[~skip])
        say(f"  {what}: rel-L2 {e:.2e}")
        assert e <= TOL_STATE, (what, e)

    def check_p(slot, lay):
        say(f"oracle p-update of layer {lay}")
        import copy
        before = copy.copy(st)                      # the update replaces st.p[slot], nothing is changed in place
        before.p, before.tau = list(st.p), list(st.tau)
        O.update_p(st, slot)
        assert float(tau[lay - 1]) == st.tau[slot] and int(pt[lay - 1]) == st.p_trials[slot], \
            (tau[lay - 1], st.tau[slot], pt[lay - 1], st.p_trials[slot])
        if g is not None:
            assert P.pdadmm_get_var(ctx, V.PROBE, lay) == (st.p_wait[slot], st.p_skip[slot])
            # indices: equal, or one level apart where the projected value sits at a midpoint of Delta (validated
            # element by element); there the oracle state takes the GPU's member for the rest of the iteration
            bad, total, worst_mid = H.quant_flips(P, ctx, before, st, what=f"{name} p_{lay}", layers=[slot],
                                                  layer_of=lambda s_: lay)
            say(f"  -Q indices of p_{lay}: {bad} of {total} differ, all one level off at a midpoint of Delta "
                f"(worst distance / slack {worst_mid:.2f}); trials {st.p_trials[slot]}, tau {st.tau[slot]}")
            assert bad <= H.flip_allowance(st, total)
        check(f"p_{lay}", V.P, lay, st.p[slot])

    if layer >= 2:
        check_p(i, layer)
    if layer < L:
        check_p(i + 1, layer + 1)
    say(f"oracle W-, b-update of layer {layer}")
    O.update_W(st, i)
    assert float(theta[layer - 1]) == st.theta[i] and int(wt[layer - 1]) == st.w_trials[i]
    check(f"W_{layer}", V.W, layer, st.W[i])
    O.update_b(st, i)
    check(f"b_{layer}", V.B, layer, st.b[i])
    say(f"oracle z-update of layer {layer}")
    if layer < L:
        z_old, q_old = st.z[i].copy(), st.q[i]
        O.update_z_hidden(st, i)
        # elements where the two candidates of the closed form tie (both are minimisers) are left out
        skip, n_tie = H.z_branch_flips(P.pdadmm_get_var(ctx, V.Z, layer), st.z[i],
                                       lambda rows: st.p[i][rows] @ st.W[i].T + st.b[i], q_old, z_old,
                                       what=f"{name} z_{layer}")
        say(f"  z_{layer}: {n_tie} tie elements of {st.z[i].size} left out")
        check(f"z_{layer}", V.Z, layer, st.z[i], skip)
        O.update_q(st, i)
        check(f"q_{layer}", V.Q, layer, st.q[i], skip)
        O.update_u(st, i)
        check(f"u_{layer}", V.U, layer, st.u[i], skip)
        # Lemma (q optimality): u = nu (q - f(z)) on the GPU's own values
        u = P.pdadmm_get_var(ctx, V.U, layer).astype(F64)
        qv = P.pdadmm_get_var(ctx, V.Q, layer).astype(F64)
        zv = P.pdadmm_get_var(ctx, V.Z, layer).astype(F64)
        assert np.max(np.abs(u - w.nu * (qv - np.maximum(zv, 0)))) <= 1e-5 * w.nu * max(1.0, np.max(np.abs(qv)))
    else:
        O.update_z_last(st)
        check(f"z_{layer}", V.Z, layer, st.z[i])
    if (name, layer, probe) == WINDOWS[-1]:
        for k in list(_problems):
            P.pdadmm_destroy(_problems.pop(k).ctx)
        torch.cuda.empty_cache()
