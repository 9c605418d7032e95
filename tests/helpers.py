"""Helpers shared by the tests: build oracle states from the seeded workloads."""
from __future__ import annotations

import numpy as np

from oracle import pdadmm_oracle as O
from workloads import (get_workload, make_features, make_graph, make_labels, make_weights,
                       perturb_layers, perturb_state, scaled_workload, stream_rng)

F32, F64 = np.float32, np.float64


def grid_of(w):
    return O.Grid(*w.quant) if w.quant is not None else None


def oracle_inputs(w):
    """Graph -> A~ -> X_aug (all via the oracle), labels, starting weights."""
    rp, ci = make_graph(w.graph, w.n_nodes, w.graph_param, stream_rng(w, 0))
    arp, aci, av = O.normalize_adj(rp, ci)
    X = make_features(w)
    Xa = O.augment(arp, aci, av, X, w.hops)
    Ws, bs = make_weights(w)
    y = make_labels(w)
    return dict(rowptr=rp, colidx=ci, a_rowptr=arp, a_colidx=aci, a_vals=av, X=X, X_aug=Xa,
                W=Ws, b=bs, y=y)


def oracle_state(w, inp=None, perturbed=True, **kw):
    """Forward-consistent oracle state, optionally perturbed (all arrays fp32-representable).
    With store32=True (the oracle's memory-lean mode) the arrays stay fp32 and are replaced layer by
    layer, so that the largest workloads fit the host memory."""
    inp = oracle_inputs(w) if inp is None else inp
    g = grid_of(w)
    kw.setdefault("risk_kind", w.risk)
    st = O.init_forward(inp["X_aug"], inp["W"], inp["b"], inp["y"], w.rho, w.nu, grid=g, quantize_q=w.quant_q, slope=w.slope, **kw)
    hold = (lambda a: a) if st.store32 else (lambda a: a.astype(F64))
    if perturbed:
        quant = (lambda a: O.quantize(a, g)[1]) if g is not None else None
        for i, z, q, p, u in perturb_layers(w, st.z, st.q, quantizer=quant):
            st.z[i] = hold(z)
            if i < st.L - 1:
                st.q[i] = hold(quant(q) if w.quant_q else q)
                st.p[i + 1] = hold(p)
                st.u[i] = hold(u)
    else:
        # make every array fp32-representable so that both sides start from identical bits
        for i in range(st.L):
            st.z[i] = hold(st.z[i].astype(F32))
            if i < st.L - 1:
                st.q[i] = hold(st.q[i].astype(F32))
                st.p[i + 1] = hold(st.p[i + 1].astype(F32))
    return st


def rel_l2(a, b):
    a = np.asarray(a, dtype=F64)
    b = np.asarray(b, dtype=F64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def small(name="C1", n=240, hidden=24, n_layers=4, feat_dim=12):
    return scaled_workload(name, n, hidden=hidden, n_layers=n_layers, feat_dim=feat_dim)
