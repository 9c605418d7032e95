"""Seeded features, labels, starting weights and perturbation noise.

The perturbation turns a forward-consistent state (which is a fixed point of most of the
ADMM updates) into a generic one: it only scales noise by the root-mean-square of an
array and adds it. Nothing here evaluates the model or any ADMM update.
"""
from __future__ import annotations

import numpy as np

from .configs import Workload

# stream ids (added to the workload's seed base)
S_GRAPH, S_FEAT, S_LABEL, S_WEIGHT, S_NOISE = 0, 1, 2, 3, 4


def stream_rng(w: Workload, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(w.seed(stream)))


def make_features(w: Workload) -> np.ndarray:
    rng = stream_rng(w, S_FEAT)
    if w.feat_kind == "bernoulli01":
        return (rng.random((w.n_nodes, w.feat_dim)) < 0.01).astype(np.float32)
    if w.feat_kind == "normal":
        return rng.standard_normal((w.n_nodes, w.feat_dim), dtype=np.float32)
    raise ValueError(w.feat_kind)


def make_labels(w: Workload) -> np.ndarray:
    return stream_rng(w, S_LABEL).integers(0, w.n_classes, size=w.n_nodes).astype(np.int32)


def make_weights(w: Workload):
    """W_l ~ N(0, 2 / n_{l-1}) as fp32 [n_l, n_{l-1}], b_l = 0; l = 1..L."""
    rng = stream_rng(w, S_WEIGHT)
    dims = w.dims
    Ws, bs = [], []
    for l in range(1, len(dims)):
        std = np.float32(np.sqrt(2.0 / dims[l - 1]))
        Ws.append(rng.standard_normal((dims[l], dims[l - 1]), dtype=np.float32) * std)
        bs.append(np.zeros(dims[l], dtype=np.float32))
    return Ws, bs


def noise_like(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(shape, dtype=np.float32)


def _rms(a: np.ndarray) -> np.float32:
    return np.float32(np.sqrt(np.mean(np.square(a, dtype=np.float64))))


def perturb_layers(w: Workload, z, q, quantizer=None, scale: float = 0.1):
    """Given forward-consistent z_1..z_L and q_1..q_{L-1} (node-major arrays), yield per layer
    (l, z_l', q_l', p_{l+1}', u_l') with
        z_l' = z_l + s*rms(z_l)*n1,  q_l' = q_l + s*rms(q_l)*n2,  p_{l+1}' = q_l' + s*rms(q_l)*n3,
        u_l' = s*nu*rms(q_l)*n4,
    n* ~ N(0,1) from the workload's noise stream (the last layer has z only: the other three are None).
    `quantizer`, when given, is applied to every p (it is the caller's projection onto the grid; this
    module does not define it). z[l], q[l] are read when layer l is reached, so a caller short of memory
    may replace its arrays layer by layer while iterating."""
    rng = stream_rng(w, S_NOISE)
    L = len(z)
    s = np.float32(scale)
    for l in range(L):
        zl = z[l].astype(np.float32, copy=True)
        zl += s * _rms(zl) * noise_like(rng, zl.shape)
        if l < L - 1:
            ql = q[l].astype(np.float32, copy=True)
            r = _rms(ql)
            ql += s * r * noise_like(rng, ql.shape)
            pl = ql + s * r * noise_like(rng, ql.shape)
            if quantizer is not None:
                pl = quantizer(pl)
            ul = (s * np.float32(w.nu) * r) * noise_like(rng, ql.shape)
            yield l, zl, ql, pl.astype(np.float32, copy=False), ul.astype(np.float32, copy=False)
        else:
            yield l, zl, None, None, None


def perturb_state(w: Workload, z, q, quantizer=None, scale: float = 0.1):
    """perturb_layers collected into lists: (z, q, p_2..p_L, u_1..u_{L-1})."""
    z_out, q_out, p_out, u_out = [], [], [], []
    for l, zl, ql, pl, ul in perturb_layers(w, z, q, quantizer, scale):
        z_out.append(zl)
        if ql is not None:
            q_out.append(ql)
            p_out.append(pl)
            u_out.append(ul)
    return z_out, q_out, p_out, u_out


S_WINDOW = 100     # stream id base of the per-layer windows below (plus the layer number)


def layer_window(w: Workload, layer: int, quantizer=None, scale: float = 0.5):
    """Seeded generic (not forward-consistent) values for everything one iteration reads or writes
    around layer l = `layer` (1-based): the layer's own variables, the q/u of the layer below and the
    W/b/z/p of the layer above (whose p-update feeds this layer's q- and u-update). Plain noise with
    plausible signs and magnitudes; `quantizer` (the caller's projection) is applied to every p.
    Keys are named after the paper's variables; absent neighbours (l = 1, l = L) are left out."""
    rng = stream_rng(w, S_WINDOW + layer)
    dims, N, L = w.dims, w.n_nodes, w.n_layers
    s = np.float32(scale)
    nu = np.float32(w.nu)

    def weights(n_out, n_in):
        return rng.standard_normal((n_out, n_in), dtype=np.float32) * np.float32(np.sqrt(2.0 / n_in))

    def act(n):          # non-negative, like an activation
        a = np.abs(noise_like(rng, (N, n))) * s
        return quantizer(a).astype(np.float32, copy=False) if quantizer is not None else a

    out = {}
    n_in, n_out = dims[layer - 1], dims[layer]
    out["W"] = weights(n_out, n_in)
    out["b"] = noise_like(rng, (n_out,)) * np.float32(0.1)
    out["z"] = noise_like(rng, (N, n_out)) * s
    if layer >= 2:
        out["p"] = act(n_in)
        out["q_prev"] = np.abs(noise_like(rng, (N, n_in))) * s
        out["u_prev"] = noise_like(rng, (N, n_in)) * (np.float32(0.1) * nu)
    if layer < L:
        out["q"] = np.abs(noise_like(rng, (N, n_out))) * s
        out["u"] = noise_like(rng, (N, n_out)) * (np.float32(0.1) * nu)
        n_next = dims[layer + 1]
        out["W_next"] = weights(n_next, n_out)
        out["b_next"] = noise_like(rng, (n_next,)) * np.float32(0.1)
        out["z_next"] = noise_like(rng, (N, n_next)) * s
        out["p_next"] = act(n_out)
    return out


S_TEACHER = 5


def planted_labels(w: Workload, X_aug: np.ndarray) -> np.ndarray:
    """Learnable labels for end-to-end checks: class = argmax of a seeded random linear map of the
    augmented features the caller passes in (the uniform labels of make_labels carry no signal)."""
    T = stream_rng(w, S_TEACHER).standard_normal((X_aug.shape[1], w.n_classes))
    return np.argmax(X_aug.astype(np.float64) @ T, axis=1).astype(np.int32)
