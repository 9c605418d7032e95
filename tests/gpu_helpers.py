"""Helpers for the GPU parity tests: same seeded inputs on both sides, comparison utilities."""
from __future__ import annotations

import numpy as np

import paper_2105_09837_amd as P
from oracle import pdadmm_oracle as O
from tests.helpers import F32, F64, grid_of, rel_l2


def config_of(w, **kw) -> P.Config:
    q = w.quant
    base = dict(n_nodes=w.n_nodes, dims=list(w.dims), rho=w.rho, nu=w.nu, quantize=1 if q else 0,
                q_lo=q[0] if q else -1.0, q_hi=q[1] if q else 1.0, q_levels=q[2] if q else 256)
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


def compare_state(ctx, st, tol, what=""):
    """Element-wise comparison of every variable; returns the worst relative L2 error and a report."""
    L = st.L
    worst, lines = 0.0, []

    def chk(name, got, ref):
        nonlocal worst
        e = rel_l2(got, ref)
        worst = max(worst, e)
        lines.append(f"{what} {name}: rel_l2={e:.3e}")
        return e

    for i in range(L):
        l = i + 1
        chk(f"W{l}", P.pdadmm_get_var(ctx, P.VAR.W, l), st.W[i])
        chk(f"b{l}", P.pdadmm_get_var(ctx, P.VAR.B, l), st.b[i])
        chk(f"z{l}", P.pdadmm_get_var(ctx, P.VAR.Z, l), st.z[i])
        if i >= 1:
            chk(f"p{l}", P.pdadmm_get_var(ctx, P.VAR.P, l), st.p[i])
        if i < L - 1:
            chk(f"q{l}", P.pdadmm_get_var(ctx, P.VAR.Q, l), st.q[i])
            # u is a small difference of O(1) quantities: measure it against the scale of rho*q
            got_u = P.pdadmm_get_var(ctx, P.VAR.U, l)
            chk(f"u{l}", got_u, st.u[i])
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


def pull_state(ctx, like):
    """Oracle State holding the GPU's current variables (fp32 values widened to fp64)."""
    st = like.copy()
    tau, theta, _, _ = step_sizes(ctx)
    for i in range(st.L):
        l = i + 1
        st.W[i] = P.pdadmm_get_var(ctx, P.VAR.W, l).astype(F64)
        st.b[i] = P.pdadmm_get_var(ctx, P.VAR.B, l).astype(F64)
        st.z[i] = P.pdadmm_get_var(ctx, P.VAR.Z, l).astype(F64)
        if i >= 1:
            st.p[i] = P.pdadmm_get_var(ctx, P.VAR.P, l).astype(F64)
            st.tau[i] = float(tau[i])
        if i < st.L - 1:
            st.q[i] = P.pdadmm_get_var(ctx, P.VAR.Q, l).astype(F64)
            st.u[i] = P.pdadmm_get_var(ctx, P.VAR.U, l).astype(F64)
        st.theta[i] = float(theta[i])
    return st
