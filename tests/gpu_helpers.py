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
                leaky_slope=w.slope, risk_kind=P.RISK[w.risk])
    base.update(kw)
    return P.Config(**base)


def gpu_context(w, inp, st=None, stream=None, aux_stream=None, **kw):
    """Context initialised from the oracle-side inputs; if an oracle state is given, its variables are
    copied in so that both sides start from bit-identical fp32 values. `stream`, `aux_stream`: torch
    streams for the iteration and for its independent parts (default: the default stream alone)."""
    import torch
    dev = torch.device("cuda:0")
    if st is not None:      # the conventions the oracle state runs under
        kw.setdefault("bt_probe_backoff", int(st.probe_backoff))
        kw.setdefault("risk_kind", P.RISK[st.risk_kind])
    cfg = config_of(w, **kw)
    Xa = torch.from_numpy(inp["X_aug"]).to(dev)
    y = torch.from_numpy(inp["y"]).to(dev)
    W0 = [torch.from_numpy(np.ascontiguousarray(a, dtype=F32)).to(dev) for a in inp["W"]]
    b0 = [torch.from_numpy(np.ascontiguousarray(a, dtype=F32)).to(dev) for a in inp["b"]]
    mask = None
    if st is not None and st.mask is not None:
        mask = torch.from_numpy(st.mask.astype(np.uint8)).to(dev)
    torch.cuda.synchronize()
    ctx = P.pdadmm_init(cfg, Xa, y, W0, b0, train_mask=mask, stream=stream, aux_stream=aux_stream)
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


EPS32 = float(np.finfo(np.float32).eps)


def flip_allowance(st, total, base=2e-5, floor=2):
    """How many of `total` projected elements may land on the other side of a midpoint of Delta: the share of
    values that lie within fp32 rounding of a midpoint grows in proportion to the number of midpoints per unit
    length, i.e. with the number of levels; `base` is the share allowed at 256 levels (every differing index is
    checked on its own by quant_flips / q_flips, this only bounds how many there may be)."""
    return max(floor, base * total * max(1.0, (st.grid.levels - 1) / 255.0))


def quant_flips(P_, ctx, before, st, what="", layers=None, layer_of=None, adopt=True):
    """-Q: indices of every p_l (l >= 2) against the oracle's. They must be equal except where the value
    that is projected, v = p - grad/tau (Appendix B), lies within rounding of the midpoint between two
    neighbouring members of Delta: there fp32 products (the HIP path) and fp64 products (the oracle) may
    fall on different sides. Every differing index is checked for exactly that: one level apart, and the
    oracle's v within `slack` of the midpoint, where slack bounds the rounding error of v as the HIP path
    forms it: 4 eps32 times the sum of the magnitudes that enter v (the sums of absolute values behind the
    dot products W p and W^T r included, so the bound already grows with their length; at full size the worst
    case seen is 0.1 of this slack).
    `before` is the oracle state the update started from, `st` the state after it; `layers` the positions
    in these states to check (default: all but the first), `layer_of` maps a position to the paper's layer
    number in the context (default: position + 1).
    At such an element both members are correct results of the update (each is the nearest member of the
    value its side computed). With adopt=True the oracle state takes the HIP path's member there, so that
    everything computed from p afterwards (W, b, z, q, u of the same iteration) can be compared with no
    further allowance. Returns (number of differing indices, number of indices, worst distance / slack)."""
    g = st.grid
    mem = g.members().astype(F64)
    bad = total = 0
    worst = 0.0
    for i in (layers if layers is not None else range(1, st.L)):
        lay = layer_of(i) if layer_of is not None else i + 1
        idx = P_.pdadmm_get_var(ctx, P_.VAR.PIDX, lay).astype(np.int32)
        gp = P_.pdadmm_get_var(ctx, P_.VAR.P, lay)
        assert np.array_equal(gp.view(np.uint32), g.members()[idx].view(np.uint32)), f"{what} p_{i + 1} not in Delta"
        ref = O.quantize(st.p[i], g)[0]
        total += idx.size
        rows, cols = np.nonzero(idx != ref)
        if rows.size == 0:
            continue
        bad += rows.size
        assert np.all(np.abs(idx[rows, cols] - ref[rows, cols]) == 1), f"{what} p_{i + 1}: an index is more than one level off"
        p, W, b, z = (np.asarray(a, dtype=F64) for a in (before.p[i], before.W[i], before.b[i], before.z[i]))
        q, u = np.asarray(before.q[i - 1], dtype=F64), np.asarray(before.u[i - 1], dtype=F64)
        tau = st.tau[i]
        pr = p[rows]
        r = pr @ W.T + b - z[rows]                                              # [k, n_out]
        mag_r = np.abs(pr) @ np.abs(W).T + np.abs(b) + np.abs(z[rows])
        Wc = W[:, cols]                                                          # [n_out, k]
        grad = st.nu * np.einsum("kj,jk->k", r, Wc) + u[rows, cols] + st.rho * (p[rows, cols] - q[rows, cols])
        mag_g = (st.nu * np.einsum("kj,jk->k", mag_r + np.abs(r), np.abs(Wc)) + np.abs(u[rows, cols])
                 + st.rho * (np.abs(p[rows, cols]) + np.abs(q[rows, cols])))
        v = p[rows, cols] - grad / tau
        mid = 0.5 * (mem[idx[rows, cols]] + mem[ref[rows, cols]])
        slack = 4.0 * EPS32 * (np.abs(p[rows, cols]) + mag_g / tau + np.abs(g.lo) + np.abs(v))
        ratio = np.abs(v - mid) / slack
        worst = max(worst, float(ratio.max()))
        assert np.all(ratio <= 1.0), (f"{what} p_{i + 1}: {int((ratio > 1).sum())} of {rows.size} differing indices are not at a "
                                      f"midpoint of Delta (worst distance / slack = {ratio.max():.2f})")
        if adopt:
            new_p = np.array(st.p[i], copy=True)
            new_p[rows, cols] = mem[idx[rows, cols]].astype(new_p.dtype)
            st.p[i] = new_p
    return bad, total, worst


def q_flips(P_, ctx, before, st, what=""):
    """Variant with q on Delta as well (Appendix B, last paragraph): the q-update projects
    v = (rho p_{l+1} + u_l + nu f(z_l)) / (rho + nu), so it has the same midpoint cases as the p-update.
    `before` is the oracle state ahead of the b/z/q/u phase (it holds the u the update read), `st` the state
    after it. Every q value of the HIP path must be a member of Delta; where it is not the oracle's member it
    must be the neighbouring one, with the oracle's v within rounding (4 eps32 times the magnitudes that
    enter v, including those behind W p + b, from which z_l comes) of the midpoint between the two. There the
    oracle state takes the HIP path's member and the dual step u_l <- u_l + rho (p_{l+1} - q_l) is redone
    with it. Returns the number of such elements."""
    g = st.grid
    mem32 = g.members()
    mem = mem32.astype(F64)
    step = float(g.step32)
    bad = 0
    for i in range(st.L - 1):
        gq = P_.pdadmm_get_var(ctx, P_.VAR.Q, i + 1)
        assert np.isin(gq, mem32).all(), f"{what} q_{i + 1} not in Delta"
        rows, cols = np.nonzero(gq != st.q[i].astype(F32))
        if rows.size == 0:
            continue
        bad += rows.size
        mine, theirs = gq[rows, cols].astype(F64), np.asarray(st.q[i], dtype=F64)[rows, cols]
        assert np.all(np.abs(np.abs(mine - theirs) - step) <= 1e-4 * step), f"{what} q_{i + 1}: more than one level off"
        p_next, u_old = np.asarray(st.p[i + 1], dtype=F64)[rows, cols], np.asarray(before.u[i], dtype=F64)[rows, cols]
        fz = O.act(np.asarray(st.z[i], dtype=F64)[rows, cols], st.slope)
        v = (st.rho * p_next + u_old + st.nu * fz) / (st.rho + st.nu)
        mag_a = ((np.abs(np.asarray(st.p[i], dtype=F64)[rows]) * np.abs(np.asarray(st.W[i], dtype=F64)[cols])).sum(axis=1)
                 + np.abs(np.asarray(st.b[i], dtype=F64)[cols]) + 2.0 * np.abs(np.asarray(before.z[i], dtype=F64)[rows, cols]))
        slack = 4.0 * EPS32 * ((st.rho * np.abs(p_next) + np.abs(u_old) + st.nu * (np.abs(fz) + mag_a)) / (st.rho + st.nu)
                                + np.abs(g.lo) + np.abs(v))
        ratio = np.abs(v - 0.5 * (mine + theirs)) / slack
        assert np.all(ratio <= 1.0), (f"{what} q_{i + 1}: {int((ratio > 1).sum())} of {rows.size} differing values are not at a "
                                      f"midpoint of Delta (worst distance / slack = {ratio.max():.2f})")
        new_q = np.array(st.q[i], copy=True)
        new_q[rows, cols] = mine
        new_u = np.array(st.u[i], copy=True)
        new_u[rows, cols] = u_old + st.rho * (p_next - mine)
        st.q[i], st.u[i] = new_q, new_u
    return bad


def oracle_state_from_gpu(ctx, like):
    """An oracle state holding the HIP path's current variables (fp32 values in fp64 arrays), step sizes and
    probe state, with the conventions of `like`."""
    st = like.copy()
    s = P.pdadmm_stats(ctx)
    for i in range(st.L):
        l = i + 1
        st.W[i] = P.pdadmm_get_var(ctx, P.VAR.W, l).astype(F64)
        st.b[i] = P.pdadmm_get_var(ctx, P.VAR.B, l).astype(F64)
        st.z[i] = P.pdadmm_get_var(ctx, P.VAR.Z, l).astype(F64)
        st.theta[i] = float(s["theta"][i])
        if i >= 1:
            st.p[i] = P.pdadmm_get_var(ctx, P.VAR.P, l).astype(F64)
            st.tau[i] = float(s["tau"][i])
            if st.grid is not None:
                st.p_wait[i], st.p_skip[i] = P.pdadmm_get_var(ctx, P.VAR.PROBE, l)
        if i < st.L - 1:
            st.q[i] = P.pdadmm_get_var(ctx, P.VAR.Q, l).astype(F64)
            st.u[i] = P.pdadmm_get_var(ctx, P.VAR.U, l).astype(F64)
    return st


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


def forward_flips(P_, ctx, ref, what=""):
    """-Q forward-consistent start (p_{l+1} = nearest member of Delta to f(z_l), layer after layer): the HIP
    path's indices against the oracle's. The pass is node-wise, so an index that falls on the other side of
    a midpoint changes that node's rows in all deeper layers and nothing else. Walking down the layers,
    every node that is still clean must either agree or sit within rounding (4 eps32 times the magnitudes
    behind W p + b) of a midpoint, after which it is left out. Returns the mask of nodes left out."""
    g = ref.grid
    mem = g.members().astype(F64)
    N = ref.p[0].shape[0]
    dirty = np.zeros(N, dtype=bool)
    for i in range(ref.L - 1):
        idx = P_.pdadmm_get_var(ctx, P_.VAR.PIDX, i + 2).astype(np.int32)
        gp = P_.pdadmm_get_var(ctx, P_.VAR.P, i + 2)
        assert np.array_equal(gp.view(np.uint32), g.members()[idx].view(np.uint32)), f"{what} p_{i + 2} not in Delta"
        want = O.quantize(ref.p[i + 1], g)[0]
        rows, cols = np.nonzero((idx != want) & ~dirty[:, None])
        if rows.size:
            assert np.all(np.abs(idx[rows, cols] - want[rows, cols]) == 1)
            v = O.act(ref.z[i][rows, cols], ref.slope)
            mag = (np.abs(ref.p[i][rows]) * np.abs(ref.W[i][cols])).sum(axis=1) + np.abs(ref.b[i][cols])
            mid = 0.5 * (mem[idx[rows, cols]] + mem[want[rows, cols]])
            slack = 4.0 * EPS32 * (mag + np.abs(v) + np.abs(g.lo))
            assert np.all(np.abs(v - mid) <= slack), f"{what} p_{i + 2}: a differing index is not at a midpoint of Delta"
            dirty[np.unique(rows)] = True
    return dirty
