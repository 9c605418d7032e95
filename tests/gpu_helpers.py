"""Helpers for the GPU parity tests: same seeded inputs on both sides, comparison utilities."""
from __future__ import annotations

import numpy as np

import paper_2105_09837_amd as P
from oracle import pdadmm_oracle as O
from tests.helpers import F32, F64, grid_of, rel_l2


def config_of(w, **kw) -> P.Config:
    q = w.quant
    base = dict(n_nodes=w.n_nodes, dims=list(w.dims), rho=w.rho, nu=w.nu, quantize=(2 if w.quant_q else 1) if q else 0,
                q_lo=q[0] if q else -1.0, q_hi=q[1] if q else 1.0, q_levels=q[2] if q else 256,
                leaky_slope=w.slope)
    base.update(kw)
    return P.Config(**base)


def gpu_context(w, inp, st=None, **kw):
    """Context initialised from the oracle-side inputs; if an oracle state is given, its variables are
    copied in so that both sides start from bit-identical fp32 values."""
    import torch
    dev = torch.device("cuda:0")
    cfg = config_of(w, **kw)
    Xa = torch.from_numpy(inp["X_aug"]).to(dev)
    y = torch.from_numpy(inp["y"]).to(dev)
    W0 = [torch.from_numpy(np.ascontiguousarray(a, dtype=F32)).to(dev) for a in inp["W"]]
    b0 = [torch.from_numpy(np.ascontiguousarray(a, dtype=F32)).to(dev) for a in inp["b"]]
    mask = None
    if st is not None and st.mask is not None:
        mask = torch.from_numpy(st.mask.astype(np.uint8)).to(dev)
    ctx = P.pdadmm_init(cfg, Xa, y, W0, b0, train_mask=mask)
    if st is not None:
        push_state(ctx, st)
    return ctx


def push_state(ctx, st):
    L = st.L
    for i in range(L):
        l = i + 1
        P.pdadmm_set_var(ctx, P.VAR.W, l, st.W[i].astype(F32))
        P.pdadmm_set_var(ctx, P.VAR.B, l, st.b[i].astype(F32))
        P.pdadmm_set_var(ctx, P.VAR.Z, l, st.z[i].astype(F32))
        if i >= 1:
            P.pdadmm_set_var(ctx, P.VAR.P, l, st.p[i].astype(F32))
            P.pdadmm_set_var(ctx, P.VAR.TAU, l, st.tau[i])
            if st.grid is not None:
                P.pdadmm_set_var(ctx, P.VAR.PROBE, l, (st.p_wait[i], st.p_skip[i]))
        if i < L - 1:
            P.pdadmm_set_var(ctx, P.VAR.Q, l, st.q[i].astype(F32))
            P.pdadmm_set_var(ctx, P.VAR.U, l, st.u[i].astype(F32))
        P.pdadmm_set_var(ctx, P.VAR.THETA, l, st.theta[i])


def round_state_to_fp32(st):
    """Make every oracle array fp32-representable (the common starting bits of both sides)."""
    for i in range(st.L):
        st.W[i] = st.W[i].astype(F32).astype(F64)
        st.b[i] = st.b[i].astype(F32).astype(F64)
        st.z[i] = st.z[i].astype(F32).astype(F64)
        if i >= 1:
            st.p[i] = st.p[i].astype(F32).astype(F64)
        if i < st.L - 1:
            st.q[i] = st.q[i].astype(F32).astype(F64)
            st.u[i] = st.u[i].astype(F32).astype(F64)
    return st


def z_branch_flips(gz, z_ref, a_rows, q_old, z_old, what="", far=1e-3, h_tol=1e-4, slope=0.0):
    """Hidden-layer z-update: where the two ReLU candidates of the closed form have (almost) the same
    subproblem value, rounding decides which one is taken and both are correct minimisers. Returns the
    mask of elements where the GPU took the other candidate than the oracle, after checking that each
    such element is such a near-tie (the GPU's value is a minimiser to rounding) and that they are rare.
    a_rows(rows) must return W p + b (new values) for the given node indices. `far` is the relative
    distance from which an element counts as differing, `h_tol` the relative slack of the subproblem value
    (both are widened for -Q, where a one-level flip in p shifts W p + b of a whole row slightly)."""
    rms = float(np.sqrt(np.mean(np.square(z_ref))))
    cand = np.abs(gz - z_ref) > far * (np.abs(z_ref) + rms)
    n = int(cand.sum())
    if n == 0:
        return cand, 0
    assert n <= max(4, 5e-6 * z_ref.size), f"{what}: {n} of {z_ref.size} z elements far from the oracle"
    rows, cols = np.nonzero(cand)
    a = a_rows(rows)[np.arange(rows.size), cols]
    qo, zo = q_old[rows, cols], z_old[rows, cols]
    h_gpu = O.z_subproblem_value(gz[rows, cols].astype(F64), a, qo, zo, slope)
    h_ref = O.z_subproblem_value(z_ref[rows, cols], a, qo, zo, slope)
    assert np.all(h_gpu <= h_ref + h_tol * np.abs(h_ref) + 1e-30), \
        f"{what}: a differing z element is not a tie of the two candidates: {h_gpu} vs {h_ref}"
    return cand, n


def compare_state(ctx, st, tol, what="", before=None):
    """Element-wise comparison of every variable; returns the worst relative L2 error and a report.
    With `before` (the oracle state one iteration earlier) the hidden-layer z, q, u comparisons leave out
    the rare elements where the z-update hit a tie of its two candidates (see z_branch_flips)."""
    L = st.L
    worst, lines = 0.0, []

    def chk(name, got, ref, skip=None):
        nonlocal worst
        if skip is not None and skip.any():
            got, ref = got[~skip], ref[~skip]
        e = rel_l2(got, ref)
        worst = max(worst, e)
        lines.append(f"{what} {name}: rel_l2={e:.3e}")
        return e

    for i in range(L):
        l = i + 1
        chk(f"W{l}", P.pdadmm_get_var(ctx, P.VAR.W, l), st.W[i])
        chk(f"b{l}", P.pdadmm_get_var(ctx, P.VAR.B, l), st.b[i])
        gz = P.pdadmm_get_var(ctx, P.VAR.Z, l)
        skip = None
        if before is not None and i < L - 1:
            skip, n = z_branch_flips(gz, st.z[i], lambda rows: st.p[i][rows] @ st.W[i].T + st.b[i],
                                     before.q[i], before.z[i], what=f"{what} z{l}", slope=st.slope)
            if n:
                lines.append(f"{what} z{l}: {n} tie elements left out")
        chk(f"z{l}", gz, st.z[i], skip)
        if i >= 1:
            chk(f"p{l}", P.pdadmm_get_var(ctx, P.VAR.P, l), st.p[i])
        if i < L - 1:
            chk(f"q{l}", P.pdadmm_get_var(ctx, P.VAR.Q, l), st.q[i], skip)
            chk(f"u{l}", P.pdadmm_get_var(ctx, P.VAR.U, l), st.u[i], skip)
    ok = worst <= tol
    return ok, worst, "\n".join(lines)


def step_sizes(ctx):
    s = P.pdadmm_stats(ctx)
    return s["tau"], s["theta"], s["p_trials"], s["w_trials"]


def oracle_phase(st, phase):
    L = st.L
    if phase == P.PHASE.P:
        for i in range(1, L):
            O.update_p(st, i)
    elif phase == P.PHASE.W:
        for i in range(L):
            O.update_W(st, i)
    else:
        for i in range(L):
            O.update_b(st, i)
        for i in range(L - 1):
            O.update_z_hidden(st, i)
        O.update_z_last(st)
        for i in range(L - 1):
            O.update_q(st, i)
        for i in range(L - 1):
            O.update_u(st, i)
