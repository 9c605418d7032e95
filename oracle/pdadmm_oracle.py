"""CPU oracle for pdADMM-G / pdADMM-G-Q (arXiv 2105.09837). TEST INFRASTRUCTURE ONLY.

Plain numpy, fp64 arithmetic on fp32-representable inputs, written from the paper:
Section 3.1 (Problems 1-2, the augmentation X_k = H psi_k(A)), Section 3.2 (augmented
Lagrangian L_rho, Algorithm 1), Section 3.3 (Problem 3, the set Delta), Section 5.1
(renormalised adjacency, Psi = {I, A~, A~^2, A~^3}, ReLU, cross-entropy) and Appendix A/B
(the sub-problem solutions). Every phi is evaluated literally (W p + b is recomputed each
time); there is no blocking, fusion, caching or algebraic shortcut.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
It shares no code with the HIP library and does not import it.

Storage convention: the paper's n x |V| matrices are held node-major, i.e. as numpy
arrays of shape [|V|, n] (the transpose); W_l is [n_l, n_{l-1}] as in the paper, so
W_l p_l + b_l is `p @ W.T + b`.

Readings of points the paper leaves open (all are conventions, "parity unpinned" by the
paper itself; the tests pin them only through the mathematical properties they imply):
  * backtracking schedule for tau_l / theta_l (Appendix A gives only the acceptance
    condition): start each iteration at previous/eta, multiply by eta until accepted; in -Q,
    where a trial costs a product, previous/eta is probed with exponential back-off after
    rejected probes (see update_p);
  * b-update: b_l is one vector broadcast over all nodes, so the exact minimiser of phi
    over b_l is b - mean_over_nodes(W p + b - z); the printed step "gradient / nu" equals
    that only if the curvature nu*|V| is used, which is the reading taken;
  * choice between the two ReLU candidates of the z-update: the one with the smaller
    value of the z-subproblem objective, ties to the non-positive candidate;
  * FISTA for z_L: fixed number of steps, step 1/(nu + 1/2), start at z_L^k, risk = sum
    (not mean) of cross-entropy over labelled nodes; unlabelled nodes take z = W p + b;
  * Delta is a uniform grid (lo, hi, levels); the nearest-level decision is taken in fp32
    (the precision of the stored p), ties to the even index;
  * variant with p and q both on Delta (Appendix B, last paragraph): the start projects q_l too;
  * least-squares risk R(z; y) = 1/2 sum_j ||z_j - e_{y_j}||^2 over labelled nodes (Section 3.1 only asks
    R to be convex and continuous; Section 5.1 uses cross-entropy): its z_L-subproblem has a closed form.

Memory-lean mode (State.store32): every variable is STORED as fp32 (the precision the HIP path stores)
and each update reads its operands up to fp64, computes in fp64 exactly as below and rounds its result to
fp32 once. It exists so that the two largest workloads fit the host memory; the arithmetic is the same.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

F32 = np.float32
F64 = np.float64


def _f64(x):
    """Operand of an update in fp64 (no copy when it already is)."""
    return np.asarray(x, dtype=F64)


# --------------------------------------------------------------------------------------
# Graph preprocessing (Section 5.1) and augmentation (Section 3.1)
# --------------------------------------------------------------------------------------
def normalize_adj(rowptr: np.ndarray, colidx: np.ndarray):
    """A~ = (D+I)^(-1/2) (A+I) (D+I)^(-1/2), D_ii = sum_j A_ij (Section 5.1).

    Input: CSR pattern of the symmetric binary A without self-loops. Output: CSR of A~ with
    the diagonal inserted, columns ascending, values computed in fp64 as
    1/sqrt((d_i+1)(d_j+1)) and rounded once to fp32."""
    n = rowptr.size - 1
    deg = np.diff(rowptr).astype(np.int64)
    out_rowptr = np.zeros(n + 1, dtype=np.int64)
    out_rowptr[1:] = np.cumsum(deg + 1)
    out_col = np.empty(out_rowptr[-1], dtype=np.int32)
    out_val = np.empty(out_rowptr[-1], dtype=F32)
    for i in range(n):
        cols = colidx[rowptr[i]:rowptr[i + 1]].astype(np.int64)
        cols = np.sort(np.concatenate([cols, [i]]))
        w = 1.0 / np.sqrt(((deg[i] + 1) * (deg[cols] + 1)).astype(F64))
        out_col[out_rowptr[i]:out_rowptr[i + 1]] = cols
        out_val[out_rowptr[i]:out_rowptr[i + 1]] = w.astype(F32)
    return out_rowptr.astype(np.int32), out_col, out_val


def augment(rowptr, colidx, vals, X, hops: int) -> np.ndarray:
    """X_aug = [X | A~X | ... | A~^hops X] along the feature axis (Sections 3.1, 5.1).

    fp32 result with a fully specified rounding order so that it can be compared bit for
    bit: every product val*x is rounded to fp32, then added to an fp32 accumulator that
    starts at +0, strictly in the CSR (ascending column) order of the row."""
    X = np.ascontiguousarray(X, dtype=F32)
    n, d = X.shape
    out = np.empty((n, (hops + 1) * d), dtype=F32)
    out[:, :d] = X
    deg = np.diff(rowptr)
    order = np.argsort(-deg, kind="stable")       # rows sorted by decreasing length
    sorted_deg = deg[order]
    prev = X
    for k in range(1, hops + 1):
        acc = np.zeros((n, d), dtype=F32)
        for pos in range(int(deg.max()) if n else 0):
            cnt = int(np.searchsorted(-sorted_deg, -pos, side="left"))  # rows with deg > pos
            rows = order[:cnt]
            e = rowptr[rows] + pos
            prod = vals[e].astype(F32)[:, None] * prev[colidx[e]]      # fp32 multiply
            acc[rows] = acc[rows] + prod                                # fp32 add
        out[:, k * d:(k + 1) * d] = acc
        prev = acc
    return out


def augment_definition_dense(rowptr, colidx, X, hops: int) -> np.ndarray:
    """The same quantity straight from its definition, dense fp64 (small graphs only):
    builds A, D, A~ as dense matrices and multiplies matrix powers (Section 5.1)."""
    n = rowptr.size - 1
    A = np.zeros((n, n))
    for i in range(n):
        A[i, colidx[rowptr[i]:rowptr[i + 1]]] = 1.0
    dinv = np.diag(1.0 / np.sqrt(A.sum(axis=1) + 1.0))
    At = dinv @ (A + np.eye(n)) @ dinv
    Xd = X.astype(F64)
    return np.concatenate([np.linalg.matrix_power(At, k) @ Xd for k in range(hops + 1)], axis=1)


# --------------------------------------------------------------------------------------
# Projection onto Delta (Section 3.3, Appendix B)
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Grid:
    """Uniform Delta = {lo + i*step : i = 0..levels-1}; all members are fp32 numbers."""
    lo: float
    hi: float
    levels: int

    @property
    def step32(self) -> np.float32:
        return F32((F32(self.hi) - F32(self.lo)) / F32(self.levels - 1))

    def members(self) -> np.ndarray:
        i = np.arange(self.levels, dtype=F32)
        return (F32(self.lo) + (i * self.step32).astype(F32)).astype(F32)


def quantize(v, grid: Grid) -> Tuple[np.ndarray, np.ndarray]:
    """argmin_{delta in Delta} |delta - v| elementwise (Appendix B), decision in fp32:
    t = (v - lo)/step, index = round-half-even(t) clamped to [0, levels-1],
    delta = lo + index*step (product rounded, then sum rounded). NaN maps to index 0."""
    v32 = np.asarray(v).astype(F32)
    lo = F32(grid.lo)
    step = grid.step32
    with np.errstate(invalid="ignore", over="ignore"):
        t = ((v32 - lo).astype(F32) / step).astype(F32)
        r = np.rint(t)
    r = np.where(np.isnan(r), 0.0, r)
    idx = np.clip(r, 0, grid.levels - 1).astype(np.int32)
    val = (lo + (idx.astype(F32) * step).astype(F32)).astype(F32)
    return idx, val


# --------------------------------------------------------------------------------------
# State and the pieces of L_rho (Section 3.2)
# --------------------------------------------------------------------------------------
def relu(x):
    return np.maximum(x, 0.0)


def act(x, slope: float = 0.0):
    """Activation f: x for x > 0, slope*x otherwise (slope = 0: ReLU, Section 5.1; 0 < slope < 1:
    leaky ReLU, which Section 4 names as satisfying the assumption)."""
    return np.where(x > 0, x, slope * x)


@dataclass
class State:
    """All variables of Problem 2 plus the duals and the backtracking parameters.
    Python index i holds the paper's layer l = i + 1. p[0] = X is fixed."""
    W: List[np.ndarray]
    b: List[np.ndarray]
    z: List[np.ndarray]
    p: List[np.ndarray]            # p[0..L-1]  <-> p_1..p_L
    q: List[np.ndarray]            # q[0..L-2]  <-> q_1..q_{L-1}
    u: List[np.ndarray]            # u[0..L-2]
    y: np.ndarray                  # class ids, [N]
    mask: Optional[np.ndarray]     # labelled nodes (bool [N]) or None = all
    rho: float
    nu: float
    grid: Optional[Grid] = None    # pdADMM-G-Q when set
    tau: List[float] = field(default_factory=list)     # tau[i] for p[i], i >= 1
    theta: List[float] = field(default_factory=list)
    eta: float = 2.0
    bt_max_trials: int = 64
    fista_iters: int = 20
    p_trials: List[int] = field(default_factory=list)
    w_trials: List[int] = field(default_factory=list)
    quantize_q: bool = False       # variant of Appendix B (last paragraph): q_l is projected onto Delta as well
    slope: float = 0.0             # negative-side slope of the activation (0 = ReLU)
    p_wait: List[int] = field(default_factory=list)    # -Q: iterations to wait after a failed probe of tau/eta
    p_skip: List[int] = field(default_factory=list)    # -Q: iterations left until the next probe
    probe_cap: int = 16
    probe_backoff: bool = True     # -Q: False = every p-update starts at previous/eta, as in pdADMM-G
    risk_kind: str = "ce"          # "ce": cross-entropy (Section 5.1); "ls": least squares against the one-hot label
    store32: bool = False          # memory-lean mode: variables are kept as fp32 between updates

    @property
    def L(self) -> int:
        return len(self.W)

    def keep(self, x):
        """Result of an update as it is stored: fp64, or rounded once to fp32 in the memory-lean mode."""
        return np.asarray(x, dtype=F32) if self.store32 else x

    def copy(self) -> "State":
        c = lambda xs: [np.array(x, copy=True) for x in xs]
        return State(c(self.W), c(self.b), c(self.z), c(self.p), c(self.q), c(self.u), self.y,
                     self.mask, self.rho, self.nu, self.grid, list(self.tau), list(self.theta),
                     self.eta, self.bt_max_trials, self.fista_iters, list(self.p_trials),
                     list(self.w_trials), self.quantize_q, self.slope, list(self.p_wait), list(self.p_skip),
                     self.probe_cap, self.probe_backoff, self.risk_kind, self.store32)


def init_forward(X_aug, W0, b0, y, rho, nu, grid: Optional[Grid] = None, mask=None,
                 tau0: float = 1.0, theta0: float = 1.0, quantize_q: bool = False, slope: float = 0.0,
                 **kw) -> State:
    """Forward-consistent start: z_l = W_l p_l + b_l, q_l = f(z_l), p_{l+1} = q_l (projected
    onto Delta for -Q; q_l too in the variant that keeps q on the grid), u_l = 0. (The paper only
    says 'initialise'; its theorems hold from any start.)"""
    L = len(W0)
    st = State([], [], [], [], [], [], np.asarray(y), mask, float(rho), float(nu), grid,
               [tau0] * L, [theta0] * L, p_trials=[0] * L, w_trials=[0] * L,
               quantize_q=bool(quantize_q and grid is not None), slope=float(slope),
               p_wait=[0] * L, p_skip=[0] * L, **kw)
    st.W = [st.keep(np.asarray(w, dtype=F64)) for w in W0]
    st.b = [st.keep(np.asarray(v, dtype=F64)) for v in b0]
    st.p = [st.keep(np.asarray(X_aug, dtype=F64))]
    for i in range(L):
        zi = _f64(st.p[i]) @ _f64(st.W[i]).T + _f64(st.b[i])
        st.z.append(st.keep(zi))
        if i < L - 1:
            qi = act(zi, slope)
            nxt = qi
            if grid is not None:
                nxt = quantize(qi, grid)[1].astype(F64)
                if quantize_q:
                    qi = nxt.copy()
            st.q.append(st.keep(qi))
            st.p.append(st.keep(np.array(nxt, dtype=F64, copy=True)))
            st.u.append(st.keep(np.zeros_like(qi)))
    return st


def grow_layers(st: State, from_layer, W_new, b_new, **kw) -> State:
    """Greedy layer-wise training (Section 3.2, after Algorithm 1; Section 5.3 goes 2 -> 5 -> 10 layers):
    a deeper model whose layer l takes W_l, b_l from layer from_layer[l-1] of the trained model `st`
    where that entry is positive and from W_new[l-1], b_new[l-1] where it is 0; the state is the
    forward-consistent start of these weights on the same inputs, labels, rho, nu, grid and activation
    (the paper fixes neither the schedule nor the restart; step sizes start again)."""
    W, b = [], []
    for i, src in enumerate(from_layer):
        if src > 0:
            if st.W[src - 1].shape[1] != (W[-1].shape[0] if W else st.p[0].shape[1]):
                raise ValueError(f"layer {i + 1}: source layer {src} has another input width")
            W.append(st.W[src - 1].copy())
            b.append(st.b[src - 1].copy())
        else:
            W.append(np.asarray(W_new[i], dtype=F64))
            b.append(np.asarray(b_new[i], dtype=F64))
    return init_forward(st.p[0], W, b, st.y, st.rho, st.nu, grid=st.grid, mask=st.mask,
                        quantize_q=st.quantize_q, slope=st.slope, probe_backoff=st.probe_backoff,
                        risk_kind=st.risk_kind, store32=st.store32, **kw)


def phi(st: State, i: int, p=None, W=None, b=None) -> float:
    """phi for layer l = i+1 (Section 3.2): (nu/2)||z - W p - b||^2, plus for l >= 2
    <u_{l-1}, p - q_{l-1}> + (rho/2)||p - q_{l-1}||^2."""
    p = _f64(st.p[i] if p is None else p)
    W = _f64(st.W[i] if W is None else W)
    b = _f64(st.b[i] if b is None else b)
    res = _f64(st.z[i]) - (p @ W.T + b)
    val = 0.5 * st.nu * float(np.sum(res * res))
    if i >= 1:
        dpq = p - _f64(st.q[i - 1])
        val += float(np.sum(_f64(st.u[i - 1]) * dpq)) + 0.5 * st.rho * float(np.sum(dpq * dpq))
    return val


def grad_p(st: State, i: int) -> np.ndarray:
    """Gradient of phi in p_l (l = i+1 >= 2): nu W^T (W p + b - z) + u_{l-1} + rho (p - q_{l-1})."""
    p, W = _f64(st.p[i]), _f64(st.W[i])
    r = p @ W.T + _f64(st.b[i]) - _f64(st.z[i])
    return st.nu * (r @ W) + _f64(st.u[i - 1]) + st.rho * (p - _f64(st.q[i - 1]))


def grad_W(st: State, i: int) -> np.ndarray:
    """Gradient of phi in W_l: nu (W p + b - z) p^T."""
    p = _f64(st.p[i])
    r = p @ _f64(st.W[i]).T + _f64(st.b[i]) - _f64(st.z[i])
    return st.nu * (r.T @ p)


def grad_b(st: State, i: int) -> np.ndarray:
    """Gradient of phi in b_l: nu * sum over nodes of (W p + b - z)."""
    r = _f64(st.p[i]) @ _f64(st.W[i]).T + _f64(st.b[i]) - _f64(st.z[i])
    return st.nu * r.sum(axis=0)


class BacktrackingError(RuntimeError):
    pass


# --------------------------------------------------------------------------------------
# Sub-problem updates (Appendix A, B)
# --------------------------------------------------------------------------------------
def update_p(st: State, i: int) -> None:
    """p_l <- argmin U_l(p; tau) (+ indicator of Delta for -Q), tau raised until
    phi(p_new) <= U_l(p_new; tau) (Appendix A 'update p', Appendix B).

    Schedule (a convention; the paper states only the acceptance condition): pdADMM-G starts every
    update at previous/eta. For -Q every trial costs a product W d, so the smaller value previous/eta
    is only probed when it has a chance: after a probe that was rejected the next probe waits
    1, 2, 4, ... (at most probe_cap) iterations, during which the update starts at the previous tau; a
    probe that is accepted at once resets the wait. From its start value tau is multiplied by eta
    until the condition holds, in both variants. With probe_backoff = False the -Q update follows the
    plain schedule of pdADMM-G (every update starts at previous/eta)."""
    g = grad_p(st, i)
    if not np.any(g):
        st.p_trials[i] = 0
        return
    p_old = _f64(st.p[i])
    phi0 = phi(st, i)
    backoff = st.grid is not None and st.probe_backoff
    probing = not backoff or st.p_skip[i] == 0
    if not probing:
        st.p_skip[i] -= 1
    t = st.tau[i] / st.eta if probing else st.tau[i]
    for trial in range(1, st.bt_max_trials + 1):
        cand = p_old - g / t
        if st.grid is not None:
            cand = quantize(cand, st.grid)[1].astype(F64)
        d = cand - p_old
        upper = phi0 + float(np.sum(g * d)) + 0.5 * t * float(np.sum(d * d))
        if phi(st, i, p=cand) <= upper:
            st.tau[i] = t
            st.p[i] = st.keep(cand)
            st.p_trials[i] = trial
            if backoff and probing:
                if trial == 1:
                    st.p_wait[i] = 0
                else:
                    st.p_wait[i] = min(max(1, 2 * st.p_wait[i]), st.probe_cap)
                    st.p_skip[i] = st.p_wait[i]
            return
        t *= st.eta
    raise BacktrackingError(f"p-update of layer {i + 1}: no tau accepted")


def update_W(st: State, i: int) -> None:
    """W_l <- W_l - grad_W phi / theta, theta raised until phi(W_new) <= V_l(W_new; theta)."""
    G = grad_W(st, i)
    if not np.any(G):
        st.w_trials[i] = 0
        return
    W_old = _f64(st.W[i])
    phi0 = phi(st, i)
    t = st.theta[i] / st.eta
    for trial in range(1, st.bt_max_trials + 1):
        cand = W_old - G / t
        D = cand - W_old
        upper = phi0 + float(np.sum(G * D)) + 0.5 * t * float(np.sum(D * D))
        if phi(st, i, W=cand) <= upper:
            st.theta[i] = t
            st.W[i] = st.keep(cand)
            st.w_trials[i] = trial
            return
        t *= st.eta
    raise BacktrackingError(f"W-update of layer {i + 1}: no theta accepted")


def update_b(st: State, i: int) -> None:
    """b_l <- b_l - grad_b phi / (nu |V|): the exact minimiser over a broadcast bias."""
    n_nodes = st.p[i].shape[0]
    st.b[i] = st.keep(_f64(st.b[i]) - grad_b(st, i) / (st.nu * n_nodes))


def z_subproblem_value(z, a, q, z_old, slope: float = 0.0):
    """(z-a)^2 + (q - f(z))^2 + (z - z_old)^2: the z-subproblem for l < L without nu/2."""
    return (z - a) ** 2 + (q - act(z, slope)) ** 2 + (z - z_old) ** 2


def update_z_hidden(st: State, i: int) -> None:
    """Closed-form z-update for l < L (Appendix A 'update z'). ReLU: the two candidates printed
    there, min((a+z_old)/2, 0) and max((a+q+z_old)/3, 0). For f(z) = slope*z on z < 0 the same
    derivation (minimise the quadratic on each half-line, clamp at 0) gives
    min((a + z_old + slope*q)/(2 + slope^2), 0) for the non-positive side; the positive side is
    unchanged. Keep the candidate with the smaller subproblem value, ties to the non-positive one."""
    a = _f64(st.p[i]) @ _f64(st.W[i]).T + _f64(st.b[i])
    z_old, q, sl = _f64(st.z[i]), _f64(st.q[i]), st.slope
    z_neg = np.minimum((a + z_old + sl * q) / (2.0 + sl * sl), 0.0)
    z_pos = np.maximum((a + q + z_old) / 3.0, 0.0)
    h_neg = z_subproblem_value(z_neg, a, q, z_old, sl)
    h_pos = z_subproblem_value(z_pos, a, q, z_old, sl)
    st.z[i] = st.keep(np.where(h_pos < h_neg, z_pos, z_neg))


def log_softmax(z):
    m = z.max(axis=1, keepdims=True)
    e = z - m
    return e - np.log(np.exp(e).sum(axis=1, keepdims=True))


def risk(z_last, y, mask=None, kind: str = "ce") -> float:
    """R(z_L; y) summed over labelled nodes. "ce": cross-entropy, logsumexp(z_j) - z_{j, y_j} (Section 5.1);
    "ls": least squares against the one-hot label, 1/2 ||z_j - e_{y_j}||^2 (any convex continuous risk is
    admissible, Section 3.1)."""
    z_last = _f64(z_last)
    rows = np.arange(z_last.shape[0])
    if kind == "ce":
        per = -log_softmax(z_last)[rows, y]
    elif kind == "ls":
        t = np.zeros_like(z_last)
        t[rows, y] = 1.0
        per = 0.5 * np.sum((z_last - t) ** 2, axis=1)
    else:
        raise ValueError(f"unknown risk {kind!r}")
    if mask is not None:
        per = per[mask]
    return float(per.sum())


def fista_z_last(z_start, a, y, nu, iters, mask=None):
    """FISTA (Beck & Teboulle 2009) on R(z; y) + (nu/2)||z - a||^2, step 1/(nu + 1/2)."""
    n, c = a.shape
    onehot = np.zeros((n, c))
    onehot[np.arange(n), y] = 1.0
    lab = np.ones((n, 1)) if mask is None else mask.astype(F64)[:, None]
    lip = nu + 0.5
    x = z_start.copy()
    w = z_start.copy()
    t = 1.0
    for _ in range(iters):
        grad = lab * (np.exp(log_softmax(w)) - onehot) + nu * (w - a)
        x_new = w - grad / lip
        t_new = (1.0 + np.sqrt(1.0 + 4.0 * t * t)) / 2.0
        w = x_new + ((t - 1.0) / t_new) * (x_new - x)
        x, t = x_new, t_new
    if mask is not None:
        x = np.where(mask[:, None], x, a)       # exact minimiser where there is no risk term
    return x


def least_squares_z_last(a, y, nu, mask=None):
    """argmin_z 1/2 ||z - e_y||^2 + (nu/2)||z - a||^2 per labelled node: the gradient (z - e_y) + nu (z - a)
    vanishes at z = (e_y + nu a) / (1 + nu). Unlabelled nodes have no risk term: z = a."""
    n, c = a.shape
    onehot = np.zeros((n, c))
    onehot[np.arange(n), y] = 1.0
    z = (onehot + nu * a) / (1.0 + nu)
    if mask is not None:
        z = np.where(mask[:, None], z, a)
    return z


def update_z_last(st: State) -> None:
    """z_L <- argmin R(z; y) + (nu/2)||z - W_L p_L - b_L||^2 (Appendix A 'update z', the l = L line):
    FISTA for the cross-entropy risk, the closed form for the least-squares risk."""
    i = st.L - 1
    a = _f64(st.p[i]) @ _f64(st.W[i]).T + _f64(st.b[i])
    if st.risk_kind == "ls":
        st.z[i] = st.keep(least_squares_z_last(a, st.y, st.nu, st.mask))
    else:
        st.z[i] = st.keep(fista_z_last(_f64(st.z[i]), a, st.y, st.nu, st.fista_iters, st.mask))


def update_q(st: State, i: int) -> None:
    """q_l <- (rho p_{l+1} + u_l + nu f(z_l)) / (rho + nu) (Appendix A 'update q'); in the variant
    that quantises q as well, the nearest member of Delta to that value (Appendix B, last paragraph)."""
    q = (st.rho * _f64(st.p[i + 1]) + _f64(st.u[i]) + st.nu * act(_f64(st.z[i]), st.slope)) / (st.rho + st.nu)
    if st.quantize_q:
        q = quantize(q, st.grid)[1].astype(F64)
    st.q[i] = st.keep(q)


def update_u(st: State, i: int) -> None:
    """u_l <- u_l + rho (p_{l+1} - q_l)."""
    st.u[i] = st.keep(_f64(st.u[i]) + st.rho * (_f64(st.p[i + 1]) - _f64(st.q[i])))


def iterate(st: State, n_iters: int = 1) -> None:
    """Algorithm 1: phases p, W, b, z, q, (residual), u; each phase over all layers."""
    L = st.L
    for _ in range(n_iters):
        for i in range(1, L):
            update_p(st, i)
        for i in range(L):
            update_W(st, i)
        for i in range(L):
            update_b(st, i)
        for i in range(L - 1):
            update_z_hidden(st, i)
        update_z_last(st)
        for i in range(L - 1):
            update_q(st, i)
        for i in range(L - 1):
            update_u(st, i)


# --------------------------------------------------------------------------------------
# The model itself (Section 3.1, Problem 1): used to score a trained W, b
# --------------------------------------------------------------------------------------
def forward(st: State) -> np.ndarray:
    """Output layer of the GA-MLP for the current weights: p_1 = X, p_{l+1} = f(W_l p_l + b_l) for
    l < L, result W_L p_L + b_L (node-major [|V|, n_L]). The ADMM variables p, z, q are not used."""
    a = _f64(st.p[0])
    for i in range(st.L):
        z = a @ _f64(st.W[i]).T + _f64(st.b[i])
        a = act(z, st.slope)
    return z


def predict(st: State):
    """Predicted class per node (first maximum of the output row) and the output layer."""
    out = forward(st)
    return np.argmax(out, axis=1).astype(np.int32), out


def accuracy(pred, y, mask=None) -> float:
    """Share of the counted nodes (mask, or all) whose prediction equals the label."""
    hit = np.asarray(pred) == np.asarray(y)
    if mask is not None:
        hit = hit[np.asarray(mask, dtype=bool)]
    return float(hit.mean()) if hit.size else 0.0


# --------------------------------------------------------------------------------------
# Objective and residual (Section 3.2, Algorithm 1)
# --------------------------------------------------------------------------------------
def objective(st: State) -> dict:
    """Terms of L_rho: risk, (nu/2) sum ||z - W p - b||^2, (nu/2) sum ||q - f(z)||^2,
    sum <u, p_{l+1} - q_l>, (rho/2) sum ||p_{l+1} - q_l||^2; F = first three; L_rho = all."""
    L = st.L
    lin = sum(float(np.sum((_f64(st.z[i]) - _f64(st.p[i]) @ _f64(st.W[i]).T - _f64(st.b[i])) ** 2)) for i in range(L))
    actp = sum(float(np.sum((_f64(st.q[i]) - act(_f64(st.z[i]), st.slope)) ** 2)) for i in range(L - 1))
    dl = sum(float(np.sum(_f64(st.u[i]) * (_f64(st.p[i + 1]) - _f64(st.q[i])))) for i in range(L - 1))
    dq = sum(float(np.sum((_f64(st.p[i + 1]) - _f64(st.q[i])) ** 2)) for i in range(L - 1))
    out = dict(risk=risk(st.z[L - 1], st.y, st.mask, st.risk_kind), lin_pen=0.5 * st.nu * lin,
               act_pen=0.5 * st.nu * actp, dual_lin=dl, dual_quad=0.5 * st.rho * dq)
    out["F"] = out["risk"] + out["lin_pen"] + out["act_pen"]
    out["L_rho"] = out["F"] + out["dual_lin"] + out["dual_quad"]
    return out


def residual(st: State):
    """sqrt(sum_l ||p_{l+1} - q_l||_F^2) and the per-layer norms."""
    per = np.array([np.sqrt(float(np.sum((_f64(st.p[i + 1]) - _f64(st.q[i])) ** 2))) for i in range(st.L - 1)])
    return float(np.sqrt(np.sum(per ** 2))), per
