"""Pins of the CPU oracle against what the paper and the mathematics fix (CPU only).

Each test names the passage it leans on. None of them re-types the oracle's own formula:
they use brute force, closed forms, invariants from the paper's lemmas, or a different
library routine.
"""
import dataclasses

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import pdadmm_oracle as O
from tests.helpers import F32, F64, oracle_inputs, oracle_state, rel_l2, small
from workloads import make_graph, stream_rng


# ----------------------------------------------------------------------------- P1
def test_normalized_adjacency_matches_dense_definition():
    # Section 5.1: A~ = (D+I)^-1/2 (A+I) (D+I)^-1/2
    w = small(n=150)
    rp, ci = make_graph(w.graph, w.n_nodes, w.graph_param, stream_rng(w, 0))
    arp, aci, av = O.normalize_adj(rp, ci)
    A = sp.csr_matrix((np.ones(ci.size), ci, rp), shape=(150, 150)).toarray()
    d = A.sum(1) + 1
    dense = (A + np.eye(150)) / np.sqrt(np.outer(d, d))
    got = sp.csr_matrix((av.astype(F64), aci, arp), shape=(150, 150))
    assert got.has_sorted_indices
    assert np.array_equal(np.diff(arp), np.diff(rp) + 1)
    np.testing.assert_allclose(got.toarray(), dense, rtol=1e-7, atol=0)
    # structure against an independent sparse construction
    ref = sp.csr_matrix(sp.csr_matrix(A) + sp.identity(150, format="csr"))
    ref.sort_indices()
    assert np.array_equal(ref.indptr, arp) and np.array_equal(ref.indices, aci)


def test_regular_graph_rows_sum_to_one():
    # for a k-regular graph every entry is 1/(k+1) and each row has k+1 of them
    n = 40
    src = np.arange(n)
    rows = np.concatenate([src, src])
    cols = np.concatenate([(src + 1) % n, (src - 1) % n])
    A = sp.csr_matrix((np.ones(2 * n), (rows, cols)), shape=(n, n))
    A.sort_indices()
    arp, aci, av = O.normalize_adj(A.indptr.astype(np.int32), A.indices.astype(np.int32))
    assert np.all(av == F32(1.0 / 3.0))
    sums = np.add.reduceat(av.astype(F64), arp[:-1])
    np.testing.assert_allclose(sums, 1.0, rtol=1e-6)


@pytest.mark.parametrize("kind", ["er", "pa"])
def test_augmentation_matches_dense_matrix_powers(kind):
    # Sections 3.1 / 5.1: X_k = A~^k X stacked along features, k = 0..hops
    w = dataclasses.replace(small(n=200, feat_dim=9), graph=kind, graph_param=(3,), hops=3)
    inp = oracle_inputs(w)
    dense = O.augment_definition_dense(inp["rowptr"], inp["colidx"], inp["X"], 3)
    got = inp["X_aug"]
    assert got.dtype == F32 and got.shape == (200, 36)
    assert np.array_equal(got[:, :9], inp["X"])
    err = np.linalg.norm(got - dense) / np.linalg.norm(dense)
    assert err <= 1e-6
    # and against scipy's sparse product (a different routine, fp64)
    At = sp.csr_matrix((inp["a_vals"].astype(F64), inp["a_colidx"], inp["a_rowptr"]), shape=(200, 200))
    x3 = At @ (At @ (At @ inp["X"].astype(F64)))
    np.testing.assert_allclose(got[:, 27:], x3, rtol=2e-5, atol=2e-6)


def test_augmentation_rounding_order_is_sequential_fp32():
    # the fp32 result must equal a scalar left-to-right fp32 loop over the row's entries
    w = small(n=60, feat_dim=5)
    inp = oracle_inputs(w)
    arp, aci, av, X = inp["a_rowptr"], inp["a_colidx"], inp["a_vals"], inp["X"].astype(F32)
    X = (X + stream_rng(w, 9).standard_normal(X.shape).astype(F32)).astype(F32)
    got = O.augment(arp, aci, av, X, 1)[:, 5:]
    for i in range(60):
        for c in range(5):
            acc = F32(0.0)
            for e in range(arp[i], arp[i + 1]):
                acc = F32(acc + F32(av[e] * X[aci[e], c]))
            assert acc.tobytes() == got[i, c].tobytes()


# ----------------------------------------------------------------------------- P2
def _brute_min(fun, lo, hi, n=400001):
    grid = np.linspace(lo, hi, n)
    vals = fun(grid)
    k = int(np.argmin(vals))
    return grid[k], vals[k]


@pytest.mark.parametrize("slope", [0.0, 0.01, 0.3])
def test_z_update_is_the_scalar_minimiser(slope):
    # Appendix A 'update z', l < L: min_z (z-a)^2 + (q - f(z))^2 + (z - z_old)^2, f = ReLU (slope 0) or
    # leaky ReLU (Section 4 names it as admissible; its closed form follows the printed derivation)
    rng = np.random.default_rng(7)
    cases = rng.normal(size=(300, 3)) * np.array([1.5, 1.0, 1.5])
    special = np.array([[0.0, 0.0, 0.0], [1.0, 0.5, -1.0], [-1.0, 1.0, 0.0], [0.3, -0.8, 0.2],
                        [-0.4, -0.3, -0.1], [2.0, 0.0, -2.0], [-1.0, 3.0, -1.0]])
    cases = np.vstack([cases, special])
    a, q, z_old = cases[:, 0], cases[:, 1], cases[:, 2]
    w = small()
    st = oracle_state(w, perturbed=False)
    # drive the oracle's own routine through a one-layer-wide fake state
    n = cases.shape[0]
    fake = dataclasses.replace(st, W=[np.zeros((1, 1))], b=[np.zeros(1)], z=[z_old[:, None].copy()],
                               p=[np.zeros((n, 1))], q=[q[:, None].copy()], u=[np.zeros((n, 1))])
    fake.b[0] = np.zeros(1)
    # a = W p + b must equal the wanted a: use p = a, W = 1
    fake.W[0] = np.ones((1, 1))
    fake.p[0] = a[:, None].copy()
    fake.slope = slope
    O.update_z_hidden(fake, 0)
    z_new = fake.z[0][:, 0]
    for k in range(n):
        f = lambda z: (z - a[k]) ** 2 + (q[k] - np.where(z > 0, z, slope * z)) ** 2 + (z - z_old[k]) ** 2
        zb, hb = _brute_min(f, -6.0, 6.0)
        assert f(z_new[k]) <= hb + 1e-12
        # unless two minima tie within the grid resolution the minimiser itself agrees
        s = a[k] + z_old[k]
        tn = s + slope * q[k]
        near_tie = tn < 0 < s + q[k] and abs((s + q[k]) ** 2 / 3 - tn * tn / (2 + slope * slope)) < 1e-3
        if not near_tie:
            assert abs(z_new[k] - zb) < 1e-4


def test_z_update_tie_goes_to_nonpositive_branch():
    # s<0<s+q with (s+q)^2/3 == s^2/2 exactly in fp64 is hard to hit; instead check the
    # degenerate tie s = 0, q = 0 (both candidates are 0) and a constructed near-tie order
    st = oracle_state(small(), perturbed=False)
    a = np.array([[0.0, -1.0]])
    z_old = np.array([[0.0, -1.0]])
    s = -2.0
    qtie = -s + np.sqrt(1.5) * abs(s)        # (s+q)^2/3 == s^2/2 up to rounding
    fake = dataclasses.replace(st, W=[np.eye(2)], b=[np.zeros(2)], z=[z_old.copy()], p=[a.copy()],
                               q=[np.array([[0.0, qtie]])], u=[np.zeros((1, 2))])
    O.update_z_hidden(fake, 0)
    assert fake.z[0][0, 0] == 0.0
    zc = fake.z[0][0, 1]
    assert zc == -1.0 or abs(zc - (s + qtie) / 3) < 1e-12      # either minimiser is valid at a tie


# ----------------------------------------------------------------------------- P3
def test_q_update_is_the_scalar_minimiser_and_dual_identity():
    # Appendix A 'update q': min_q u (p - q) + (rho/2)(p-q)^2 + (nu/2)(q - relu(z))^2
    w = small()
    st = oracle_state(w)
    st.rho, st.nu = 0.7, 0.3
    O.update_q(st, 1)
    rng = np.random.default_rng(3)
    for _ in range(40):
        j, c = rng.integers(st.q[1].shape[0]), rng.integers(st.q[1].shape[1])
        p, u, z = st.p[2][j, c], st.u[1][j, c], st.z[1][j, c]
        f = lambda q: u * (p - q) + 0.35 * (p - q) ** 2 + 0.15 * (q - max(z, 0.0)) ** 2
        qb, fb = _brute_min(f, st.q[1][j, c] - 2, st.q[1][j, c] + 2, 200001)
        assert f(st.q[1][j, c]) <= fb + 1e-12 and abs(qb - st.q[1][j, c]) < 1e-4


@pytest.mark.parametrize("name,slope", [("C1", 0.0), ("C5", 0.0), ("C1", 0.2)])
def test_dual_equals_nu_times_q_minus_activation(name, slope):
    # Lemma (q optimality): u_l^k = nu (q_l^k - f(z_l^k)) for every k >= 1
    w = dataclasses.replace(small(name, n=120, hidden=16, n_layers=4, feat_dim=6), slope=slope)
    st = oracle_state(w)
    assert st.slope == slope
    for _ in range(3):
        O.iterate(st)
        for i in range(st.L - 1):
            fz = np.where(st.z[i] > 0, st.z[i], slope * st.z[i])
            np.testing.assert_allclose(st.u[i], st.nu * (st.q[i] - fz), rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- P4
def test_gradients_by_finite_differences():
    # expanded gradients of phi in p, W, b (Appendix, proof of the Lipschitz lemmas)
    st = oracle_state(small(n=40, hidden=7, feat_dim=3))
    rng = np.random.default_rng(0)
    i = 2
    gp, gW, gb = O.grad_p(st, i), O.grad_W(st, i), O.grad_b(st, i)
    eps = 1e-6
    for _ in range(10):
        j, c = rng.integers(gp.shape[0]), rng.integers(gp.shape[1])
        d = np.zeros_like(st.p[i]); d[j, c] = eps
        fd = (O.phi(st, i, p=st.p[i] + d) - O.phi(st, i, p=st.p[i] - d)) / (2 * eps)
        assert abs(fd - gp[j, c]) <= 1e-6 * max(1.0, abs(gp[j, c]))
        r, c = rng.integers(gW.shape[0]), rng.integers(gW.shape[1])
        d = np.zeros_like(st.W[i]); d[r, c] = eps
        fd = (O.phi(st, i, W=st.W[i] + d) - O.phi(st, i, W=st.W[i] - d)) / (2 * eps)
        assert abs(fd - gW[r, c]) <= 1e-6 * max(1.0, abs(gW[r, c]))
        r = rng.integers(gb.size)
        d = np.zeros_like(st.b[i]); d[r] = eps
        fd = (O.phi(st, i, b=st.b[i] + d) - O.phi(st, i, b=st.b[i] - d)) / (2 * eps)
        assert abs(fd - gb[r]) <= 1e-6 * max(1.0, abs(gb[r]))


def test_phi_is_exactly_quadratic_in_p_and_W():
    st = oracle_state(small(n=50, hidden=9, feat_dim=4))
    rng = np.random.default_rng(1)
    i = 1
    d = rng.normal(size=st.p[i].shape)
    lhs = O.phi(st, i, p=st.p[i] + d) - O.phi(st, i) - np.sum(O.grad_p(st, i) * d)
    rhs = 0.5 * st.nu * np.sum((d @ st.W[i].T) ** 2) + 0.5 * st.rho * np.sum(d * d)
    assert abs(lhs - rhs) <= 1e-9 * abs(rhs)
    D = rng.normal(size=st.W[i].shape)
    lhs = O.phi(st, i, W=st.W[i] + D) - O.phi(st, i) - np.sum(O.grad_W(st, i) * D)
    rhs = 0.5 * st.nu * np.sum((st.p[i] @ D.T) ** 2)
    assert abs(lhs - rhs) <= 1e-9 * abs(rhs)


@pytest.mark.parametrize("name", ["C1", "C5"])
def test_backtracking_accepts_smallest_admissible_step_parameter(name):
    # Appendix A: tau must satisfy phi(p_new) <= U_l(p_new; tau); our schedule takes the first
    # tau on the grid previous/eta * eta^j that does, so tau/eta must fail unless it was trial 1.
    w = small(name, n=100, hidden=12, n_layers=4, feat_dim=5)
    st = oracle_state(w)
    searched_p = searched_w = 0
    for it in range(4):
        if it == 1:
            # start far below the admissible range so that the search has to climb: only then does the
            # accepted value show that every term of the condition is in place
            st.tau = [1e-5] * st.L
            st.theta = [1e-5] * st.L
        before = st.copy()
        for i in range(1, st.L):
            O.update_p(st, i)
            searched_p += st.p_trials[i] > 2
        for i in range(1, st.L):
            g = O.grad_p(before, i)
            def cond(t):
                cand = before.p[i] - g / t
                if before.grid is not None:
                    cand = O.quantize(cand, before.grid)[1].astype(F64)
                d = cand - before.p[i]
                return O.phi(before, i, p=cand) <= O.phi(before, i) + np.sum(g * d) + 0.5 * t * np.sum(d * d)
            assert cond(st.tau[i])
            if st.p_trials[i] > 1:
                assert not cond(st.tau[i] / st.eta)
            # Lemma (optimality 1), first inequality: decrease >= (tau/2)||dp||^2 (non-Q)
            if before.grid is None:
                dec = O.phi(before, i) - O.phi(before, i, p=st.p[i])
                assert dec >= 0.5 * st.tau[i] * np.sum((st.p[i] - before.p[i]) ** 2) * (1 - 1e-9)
            else:
                assert O.phi(before, i, p=st.p[i]) <= O.phi(before, i) * (1 + 1e-12) + 1e-12
        mid = st.copy()
        for i in range(st.L):
            O.update_W(st, i)
            searched_w += st.w_trials[i] > 2
        for i in range(st.L):
            G = O.grad_W(mid, i)
            def condw(t):
                D = -G / t
                return O.phi(mid, i, W=mid.W[i] + D) <= O.phi(mid, i) + np.sum(G * D) + 0.5 * t * np.sum(D * D)
            assert condw(st.theta[i])
            if st.w_trials[i] > 1:
                assert not condw(st.theta[i] / st.eta)
            dec = O.phi(mid, i) - O.phi(mid, i, W=st.W[i])
            assert dec >= 0.5 * st.theta[i] * np.sum((st.W[i] - mid.W[i]) ** 2) * (1 - 1e-9)
        for i in range(st.L):
            O.update_b(st, i)
        for i in range(st.L - 1):
            O.update_z_hidden(st, i)
        O.update_z_last(st)
        for i in range(st.L - 1):
            O.update_q(st, i)
        for i in range(st.L - 1):
            O.update_u(st, i)
    assert searched_p >= st.L - 1 and searched_w >= st.L


# ----------------------------------------------------------------------------- P5
def test_b_update_is_stationary_and_decreases_enough():
    st = oracle_state(small(n=80, hidden=10, feat_dim=4))
    for i in range(st.L):
        before = O.phi(st, i)
        b_old = st.b[i].copy()
        O.update_b(st, i)
        assert np.max(np.abs(O.grad_b(st, i))) <= 1e-12 * max(1.0, np.max(np.abs(st.b[i]))) * st.p[i].shape[0]
        # Lemma (optimality 1), third inequality
        assert before - O.phi(st, i) >= 0.5 * st.nu * np.sum((st.b[i] - b_old) ** 2) * (1 - 1e-9)


# ----------------------------------------------------------------------------- P6
def test_fista_converges_to_the_stationary_point():
    # z_L-subproblem: softmax(z) - onehot + nu (z - a) = 0 at the minimiser
    rng = np.random.default_rng(5)
    n, c, nu = 30, 6, 0.05
    a = rng.normal(size=(n, c)) * 2
    y = rng.integers(0, c, size=n)
    z = O.fista_z_last(np.zeros((n, c)), a, y, nu, 20000)
    onehot = np.eye(c)[y]
    g = np.exp(O.log_softmax(z)) - onehot + nu * (z - a)
    assert np.max(np.abs(g)) < 1e-9


def test_fista_two_classes_matches_logistic_prox_by_bisection():
    rng = np.random.default_rng(6)
    n, nu = 25, 0.2
    a = rng.normal(size=(n, 2)) * 1.5
    y = rng.integers(0, 2, size=n)
    z = O.fista_z_last(a.copy(), a, y, nu, 5000)
    # with 2 classes: z = a + s*(+1,-1)*sign, where the scalar margin m = z_y - z_other solves
    # m - m0 = (2/nu) * sigmoid(-m), m0 = a_y - a_other  (stationarity of CE + prox)
    for j in range(n):
        m0 = a[j, y[j]] - a[j, 1 - y[j]]
        lo, hi = m0, m0 + 2.0 / nu
        for _ in range(200):
            mid = 0.5 * (lo + hi)
            if mid - m0 - (2.0 / nu) / (1.0 + np.exp(mid)) > 0:
                hi = mid
            else:
                lo = mid
        m = 0.5 * (lo + hi)
        assert abs((z[j, y[j]] - z[j, 1 - y[j]]) - m) < 1e-8
        assert abs(z[j].sum() - a[j].sum()) < 1e-9        # the mean direction is untouched


def test_fista_first_two_steps_are_plain_gradient_steps():
    # Beck & Teboulle's recursion starts with t_1 = 1, so the first extrapolation coefficient (t_1 - 1)/t_2
    # vanishes: two FISTA steps are two gradient steps of size 1/(nu + 1/2) on R(z; y) + (nu/2)||z - a||^2.
    # The gradient here comes from central differences of that objective, not from the oracle's formula.
    # From the third step on the extrapolation is active, so three steps must differ from three such steps.
    rng = np.random.default_rng(11)
    n, c, nu = 5, 4, 0.3
    a, z0 = rng.standard_normal((n, c)), rng.standard_normal((n, c))
    y = rng.integers(0, c, n)
    h = lambda z: O.risk(z, y) + 0.5 * nu * float(np.sum((z - a) ** 2))

    def fd_grad(z, eps=1e-6):
        g = np.zeros_like(z)
        for j in range(z.shape[0]):
            for k in range(z.shape[1]):
                e = np.zeros_like(z)
                e[j, k] = eps
                g[j, k] = (h(z + e) - h(z - e)) / (2 * eps)
        return g

    gd = [z0]
    for _ in range(3):
        gd.append(gd[-1] - fd_grad(gd[-1]) / (nu + 0.5))
    np.testing.assert_allclose(O.fista_z_last(z0, a, y, nu, 1), gd[1], atol=1e-8)
    np.testing.assert_allclose(O.fista_z_last(z0, a, y, nu, 2), gd[2], atol=1e-8)
    x3 = O.fista_z_last(z0, a, y, nu, 3)
    assert np.max(np.abs(x3 - gd[3])) > 1e-4
    # ... and the third step extrapolates FORWARD along the last move: x_3 is the gradient step taken from
    # x_2 + beta (x_2 - x_1) with 0 < beta < 1 (beta = (t_2 - 1)/t_3 = 0.28...); recover beta by a 1-D search
    def step_from(beta):
        wv = gd[2] + beta * (gd[2] - gd[1])
        return wv - fd_grad(wv) / (nu + 0.5)
    from scipy.optimize import minimize_scalar
    betas = np.linspace(0.0, 1.0, 101)
    errs = [np.sum((step_from(bv) - x3) ** 2) for bv in betas]
    coarse = float(betas[int(np.argmin(errs))])
    fit = minimize_scalar(lambda bv: np.sum((step_from(bv) - x3) ** 2), bounds=(coarse - 0.01, coarse + 0.01),
                          method="bounded", options=dict(xatol=1e-10))
    t2 = (1 + 5 ** 0.5) / 2
    t3 = (1 + (1 + 4 * t2 * t2) ** 0.5) / 2
    assert np.max(np.abs(step_from(fit.x) - x3)) < 1e-6 and abs(fit.x - (t2 - 1) / t3) < 1e-5


def test_fista_unlabelled_nodes_take_linear_output_and_step_is_safe():
    rng = np.random.default_rng(8)
    n, c = 12, 5
    a = rng.normal(size=(n, c))
    y = rng.integers(0, c, size=n)
    mask = np.arange(n) % 2 == 0
    z = O.fista_z_last(rng.normal(size=(n, c)), a, y, 0.1, 20, mask)
    assert np.array_equal(z[~mask], a[~mask])
    # curvature of cross-entropy is at most 1/2: lambda_max(diag(s) - s s^T) <= 1/2
    for _ in range(200):
        s = rng.dirichlet(np.ones(c) * rng.uniform(0.1, 3))
        assert np.linalg.eigvalsh(np.diag(s) - np.outer(s, s)).max() <= 0.5 + 1e-12
    # risk is the summed cross-entropy: compare with a direct evaluation
    direct = sum(np.log(np.exp(z[j]).sum()) - z[j, y[j]] for j in range(n) if mask[j])
    assert abs(O.risk(z, y, mask) - direct) < 1e-10


def test_fista_decreases_the_subproblem_monotonically_enough():
    rng = np.random.default_rng(9)
    n, c, nu = 20, 4, 0.01
    a = rng.normal(size=(n, c))
    y = rng.integers(0, c, size=n)
    f = lambda z: O.risk(z, y) + 0.5 * nu * np.sum((z - a) ** 2)
    vals = [f(O.fista_z_last(a.copy(), a, y, nu, t)) for t in (0, 5, 20, 100, 1000)]
    assert vals[1] < vals[0] and vals[2] < vals[1] and vals[3] < vals[2] and vals[4] <= vals[3] + 1e-9


# ----------------------------------------------------------------------------- P7
@pytest.mark.parametrize("grid", [O.Grid(-1.0, 1.0, 256), O.Grid(-1.0, 20.0, 22), O.Grid(0.0, 3.0, 7)])
def test_quantizer_is_nearest_member(grid):
    # Appendix B: p <- argmin_{delta in Delta} |delta - v|
    rng = np.random.default_rng(11)
    mem = grid.members()
    assert mem.dtype == F32 and mem.size == grid.levels and np.all(np.diff(mem) > 0)
    span = grid.hi - grid.lo
    v = (rng.uniform(grid.lo - 0.3 * span, grid.hi + 0.3 * span, size=20000)).astype(F32)
    mids = ((mem[:-1].astype(F64) + mem[1:].astype(F64)) / 2).astype(F32)
    v = np.concatenate([v, mem, mids, np.nextafter(mids, F32(np.inf)), np.nextafter(mids, F32(-np.inf)),
                        np.array([np.inf, -np.inf, 0.0, -0.0], dtype=F32)])
    idx, val = O.quantize(v, grid)
    assert idx.min() >= 0 and idx.max() < grid.levels
    assert np.array_equal(val.view(np.uint32), mem[idx].view(np.uint32))       # p in Delta, bit for bit
    fin = np.isfinite(v)
    brute = np.argmin(np.abs(mem.astype(F64)[None, :] - v.astype(F64)[fin, None]), axis=1)
    dist_got = np.abs(mem.astype(F64)[idx[fin]] - v.astype(F64)[fin])
    dist_best = np.abs(mem.astype(F64)[brute] - v.astype(F64)[fin])
    # identical except within rounding of a midpoint, where either neighbour is a minimiser
    assert np.all(dist_got <= dist_best + 4 * np.finfo(F32).eps * np.maximum(1.0, np.abs(v[fin])))
    assert np.mean(idx[fin] == brute) > 0.99
    assert O.quantize(np.array([np.nan], dtype=F32), grid)[0][0] == 0


@pytest.mark.parametrize("grid", [O.Grid(-1.0, 1.0, 65536), O.Grid(-3.0, 5.0, 1000)])
def test_quantizer_is_nearest_member_on_fine_grids(grid):
    # the 16-bit case of Section 5.5 (65536 levels): nearest member by bisection into the sorted members
    # and a comparison of the two neighbours in fp64
    rng = np.random.default_rng(12)
    mem = grid.members()
    assert mem.dtype == F32 and mem.size == grid.levels and np.all(np.diff(mem) > 0)
    span = grid.hi - grid.lo
    mids = ((mem[:-1].astype(F64) + mem[1:].astype(F64)) / 2).astype(F32)
    v = np.concatenate([rng.uniform(grid.lo - 0.3 * span, grid.hi + 0.3 * span, size=50000).astype(F32), mem, mids,
                        np.nextafter(mids, F32(np.inf)), np.nextafter(mids, F32(-np.inf))])
    idx, val = O.quantize(v, grid)
    assert idx.min() >= 0 and idx.max() < grid.levels
    assert np.array_equal(val.view(np.uint32), mem[idx].view(np.uint32))
    m64, v64 = mem.astype(F64), v.astype(F64)
    hi = np.clip(np.searchsorted(m64, v64), 1, grid.levels - 1)
    lo = hi - 1
    brute = np.where(np.abs(m64[lo] - v64) <= np.abs(m64[hi] - v64), lo, hi)
    dist_got, dist_best = np.abs(m64[idx] - v64), np.abs(m64[brute] - v64)
    assert np.all(dist_got <= dist_best + 4 * np.finfo(F32).eps * np.maximum(1.0, np.abs(v64)))
    # equal indices wherever the decision is not within fp32 rounding of a midpoint (t = (v - lo)/step is formed in
    # fp32: at t near 65535 one ulp of t is 0.004 of a step, and so is one ulp of v - lo near 2)
    away = np.abs(np.abs(m64[lo] - v64) - np.abs(m64[hi] - v64)) > 0.05 * float(grid.step32)
    assert away[:50000].mean() > 0.9          # (the random values; the rest sit on members and midpoints)
    assert np.array_equal(idx[away], brute[away])


def test_quantized_run_keeps_p_in_delta():
    w = small("C5", n=90, hidden=10, n_layers=4, feat_dim=4)
    st = oracle_state(w)
    mem = st.grid.members()
    for _ in range(3):
        O.iterate(st)
        for i in range(1, st.L):
            assert np.isin(st.p[i].astype(F32), mem).all()
            assert np.array_equal(st.p[i].astype(F32).astype(F64), st.p[i])


# ----------------------------------------------------------------------------- P8
def test_lagrangian_is_monotone_when_lemma_condition_holds():
    # Lemma 1: rho > max(4 nu S^2, (sqrt(17)+1) nu / 2) (S = 1 for ReLU) => L_rho non-increasing.
    # nu = 0.01, rho = 1 is the setting of the paper's convergence experiment (Section 5.3).
    w = dataclasses.replace(small(n=150, hidden=16, n_layers=5, feat_dim=6), rho=1.0, nu=0.01)
    st = oracle_state(w, fista_iters=300)
    vals, res = [O.objective(st)["L_rho"]], [O.residual(st)[0]]
    for _ in range(40):
        O.iterate(st)
        vals.append(O.objective(st)["L_rho"])
        res.append(O.residual(st)[0])
    vals = np.array(vals)
    assert np.all(np.diff(vals) <= 1e-9 * np.abs(vals[:-1]))
    # residual ||p_{l+1} - q_l|| shrinks (Theorem 1 / 3: it converges to 0)
    assert res[-1] < 0.05 * res[0] and np.mean(res[-5:]) < np.mean(res[5:10])


def test_phase_by_phase_sufficient_decrease():
    # Lemma (optimality 1): each primal phase lowers L_rho by the stated quadratic amount
    w = dataclasses.replace(small(n=100, hidden=12, n_layers=4, feat_dim=5), rho=1.0, nu=0.01)
    st = oracle_state(w, fista_iters=2000)
    for _ in range(2):
        L0 = O.objective(st)["L_rho"]
        z_old = [z.copy() for z in st.z]
        for i in range(st.L - 1):
            O.update_z_hidden(st, i)
        O.update_z_last(st)
        L1 = O.objective(st)["L_rho"]
        dz = sum(np.sum((st.z[i] - z_old[i]) ** 2) for i in range(st.L))
        assert L0 - L1 >= 0.5 * st.nu * dz * (1 - 1e-6) - 1e-9
        O.iterate(st)


# ----------------------------------------------------------------------------- P9
def test_forward_consistent_start_changes_only_the_last_layer_first():
    # with z = W p + b, q = f(z), p_{l+1} = q_l, u = 0 every residual and gradient vanishes,
    # so one iteration may only move z_L; the change then spreads backwards layer by layer
    w = small(n=70, hidden=8, n_layers=5, feat_dim=4)
    inp = oracle_inputs(w)
    st = O.init_forward(inp["X_aug"], inp["W"], inp["b"], inp["y"], w.rho, w.nu)
    ref = st.copy()
    O.iterate(st)
    L = st.L
    for i in range(L):
        np.testing.assert_allclose(st.W[i], ref.W[i], rtol=0, atol=1e-12)
        np.testing.assert_allclose(st.b[i], ref.b[i], rtol=0, atol=1e-12)
        if i < L - 1:
            np.testing.assert_allclose(st.z[i], ref.z[i], rtol=0, atol=1e-12)
            np.testing.assert_allclose(st.q[i], ref.q[i], rtol=0, atol=1e-12)
            np.testing.assert_allclose(st.u[i], ref.u[i], rtol=0, atol=1e-12)
            np.testing.assert_allclose(st.p[i + 1], ref.p[i + 1], rtol=0, atol=1e-12)
    assert np.max(np.abs(st.z[L - 1] - ref.z[L - 1])) > 1e-3
    O.iterate(st)
    assert np.max(np.abs(st.W[L - 1] - ref.W[L - 1])) > 0           # layer L now moves
    np.testing.assert_allclose(st.W[0], ref.W[0], rtol=0, atol=1e-10)   # layer 1 still untouched
    np.testing.assert_allclose(st.z[0], ref.z[0], rtol=0, atol=1e-10)


def test_backtracking_schedule_convention():
    # convention (the paper states only the acceptance condition): every iteration restarts at
    # previous/eta and multiplies by eta per rejected trial, so tau, theta stay powers of eta
    st = oracle_state(small(n=60, hidden=8, feat_dim=4))
    for _ in range(4):
        tau0, th0 = list(st.tau), list(st.theta)
        O.iterate(st)
        for i in range(1, st.L):
            assert st.p_trials[i] >= 1 and st.tau[i] == tau0[i] / st.eta * st.eta ** (st.p_trials[i] - 1)
        for i in range(st.L):
            assert st.w_trials[i] >= 1 and st.theta[i] == th0[i] / st.eta * st.eta ** (st.w_trials[i] - 1)


def test_quantized_start_keeps_p_on_the_grid_and_q_only_in_the_variant():
    # Problem 3: p_l in Delta for l >= 2 from the start on; q_l is a free variable (q_l = f(z_l) at the
    # forward-consistent start) unless the variant of Appendix B's last paragraph keeps it on Delta too.
    w = small("C5", n=120, hidden=10, n_layers=4, feat_dim=5)
    inp = oracle_inputs(w)
    for both in (False, True):
        st = oracle_state(dataclasses.replace(w, quant_q=both), inp, perturbed=False)
        mem = st.grid.members().astype(F64)
        half = 0.5 * float(st.grid.step32)
        for i in range(1, st.L):
            fz = O.act(st.z[i - 1])
            dist = np.abs(fz[..., None] - mem)
            nearest = mem[np.argmin(dist, axis=-1)]
            clear = np.abs(np.sort(dist, axis=-1)[..., 0] - np.sort(dist, axis=-1)[..., 1]) > 1e-6 * half
            assert np.isin(st.p[i], mem).all()
            assert np.array_equal(st.p[i][clear], nearest[clear])          # brute-force nearest member
            if both:
                assert np.array_equal(st.q[i - 1], st.p[i])
            else:
                assert np.allclose(st.q[i - 1], fz, rtol=0, atol=1e-6)
                assert not np.isin(st.q[i - 1], mem).all()


def test_risk_is_stable_for_large_outputs():
    # R = logsumexp(z) - z_y (Section 3.1 uses the cross-entropy): for z = (1000, 0) it is 0 for label 0
    # and 1000 for label 1; a naive exp overflows here.
    z = np.array([[1000.0, 0.0], [-1000.0, 0.0], [0.0, 0.0]])
    with np.errstate(over="raise", invalid="raise"):
        assert abs(O.risk(z[:1], np.array([0]))) < 1e-12
        assert abs(O.risk(z[:1], np.array([1])) - 1000.0) < 1e-9
        assert abs(O.risk(z, np.array([1, 0, 0])) - (1000.0 + 1000.0 + np.log(2.0))) < 1e-9
        out = O.fista_z_last(z, z.copy(), np.array([1, 0, 0]), 0.1, 3)
    assert np.isfinite(out).all()


@pytest.mark.parametrize("name", ["C1", "C5"])
def test_iteration_takes_the_updates_in_the_order_of_algorithm_1(name):
    # Algorithm 1: p_l (l = 2..L) from the old W, b, z, q, u; then W_l from the new p; b_l from the new p, W;
    # z_l from the new p, W, b; q_l from the new p_{l+1}, z_l and the old u_l; last u_l from the new p, q.
    # Each update below is applied to a state that holds exactly those versions; the sweep must agree.
    w = small(name, n=90, hidden=9, n_layers=4, feat_dim=4)
    st = oracle_state(w)
    ref = st.copy()
    O.iterate(st, 1)
    L = ref.L
    old = ref.copy()
    for i in range(1, L):
        O.update_p(ref, i)
    for i in range(1, L):        # the p-updates of different layers do not see each other
        solo = old.copy()
        O.update_p(solo, i)
        assert np.array_equal(solo.p[i], ref.p[i])
    assert all(np.array_equal(ref.W[i], old.W[i]) for i in range(L))
    for i in range(L):
        O.update_W(ref, i)
    for i in range(L):
        O.update_b(ref, i)
    assert all(np.array_equal(ref.z[i], old.z[i]) for i in range(L))
    for i in range(L - 1):
        O.update_z_hidden(ref, i)
    O.update_z_last(ref)
    assert all(np.array_equal(ref.u[i], old.u[i]) for i in range(L - 1))
    for i in range(L - 1):
        O.update_q(ref, i)
    for i in range(L - 1):
        O.update_u(ref, i)
    for name_, a, b in [("p", st.p, ref.p), ("W", st.W, ref.W), ("b", st.b, ref.b), ("z", st.z, ref.z),
                        ("q", st.q, ref.q), ("u", st.u, ref.u)]:
        for i in range(len(a)):
            assert np.array_equal(a[i], b[i]), (name_, i)
    # the W-update has used the NEW p: its gradient at the old p would have given another W
    # (in -Q a small step can project back onto the old p; then there is nothing to tell apart)
    probe = old.copy()
    O.update_W(probe, 1)
    moved = not np.array_equal(old.p[1], st.p[1])
    assert moved or name == "C5"
    assert np.array_equal(probe.W[1], st.W[1]) == (not moved)


def test_objective_terms_and_residual_on_a_hand_computed_state():
    # Problem 2 / Section 3.2 on one node, widths 1-1-1-2, every term worked out by hand:
    #   layer 1: W p + b = 1*2 + 0.5 = 2.5, z = 2      -> (z - Wp - b)^2 = 0.25; q = 1.5, f(z) = 2 -> 0.25
    #            p_2 = 1, u_1 = 0.2                      -> u (p - q) = -0.1, (p - q)^2 = 0.25
    #   layer 2: 2*1 - 1 = 1, z = -1                     -> 4;              q = 0.5, f(z) = 0 -> 0.25
    #            p_3 = 3.5, u_2 = -1                     -> -3,             (p - q)^2 = 9
    #   layer 3: a = (3.5, -3.5), z = (0, ln 3)          -> 12.25 + (ln 3 + 3.5)^2
    #            softmax(z) = (1/4, 3/4), label 0        -> R = ln 4
    nu, rho = 0.1, 3.0
    W = [np.array([[1.0]]), np.array([[2.0]]), np.array([[1.0], [-1.0]])]
    b = [np.array([0.5]), np.array([-1.0]), np.array([0.0, 0.0])]
    st = O.init_forward(np.array([[2.0]]), W, b, np.array([0]), rho, nu)
    st.z = [np.array([[2.0]]), np.array([[-1.0]]), np.array([[0.0, np.log(3.0)]])]
    st.q = [np.array([[1.5]]), np.array([[0.5]])]
    st.p = [np.array([[2.0]]), np.array([[1.0]]), np.array([[3.5]])]
    st.u = [np.array([[0.2]]), np.array([[-1.0]])]
    o = O.objective(st)
    lin = 0.25 + 4.0 + 12.25 + (np.log(3.0) + 3.5) ** 2
    want = dict(risk=np.log(4.0), lin_pen=0.05 * lin, act_pen=0.05 * 0.5, dual_lin=-3.1, dual_quad=1.5 * 9.25)
    for k, v in want.items():
        assert abs(o[k] - v) < 1e-12, (k, o[k], v)
    assert abs(o["F"] - (np.log(4.0) + 0.05 * lin + 0.025)) < 1e-12
    assert abs(o["L_rho"] - (np.log(4.0) + 0.05 * lin + 0.025 - 3.1 + 13.875)) < 1e-12
    tot, per = O.residual(st)
    assert abs(tot - np.sqrt(9.25)) < 1e-12 and np.allclose(per, [0.5, 3.0], atol=1e-15)
    # phi of Section 3.2 on the same numbers: layer 2 = (nu/2)*4 + u_1 (p_2 - q_1) + (rho/2)(p_2 - q_1)^2
    assert abs(O.phi(st, 1) - (0.05 * 4.0 - 0.1 + 1.5 * 0.25)) < 1e-12
    assert abs(O.phi(st, 0) - 0.05 * 0.25) < 1e-12


# ----------------------------------------------------------------------------- the model (Problem 1)
def test_forward_pass_reproduces_a_network_with_a_known_function():
    # Section 3.1 / Problem 1. Two layers built by hand: W_1 = [I; -I] splits x into (x+, x-),
    # W_2 = [I, -I] recombines them, so the output is x itself; a third layer adds a known bias.
    rng = np.random.default_rng(5)
    n, d = 50, 6
    X = rng.standard_normal((n, d))
    I = np.eye(d)
    W = [np.vstack([I, -I]), np.hstack([I, -I])]
    b = [np.zeros(2 * d), np.zeros(d)]
    y = rng.integers(0, d, n)
    st = O.init_forward(X, W, b, y, 1.0, 1.0)
    out = O.forward(st)
    np.testing.assert_allclose(out, X, atol=1e-15)
    pred, _ = O.predict(st)
    assert np.array_equal(pred, np.argmax(X, axis=1))
    # max(x_0, x_1) = x_1 + relu(x_0 - x_1): a one-hidden-layer network, checked node by node
    W = [np.array([[1.0, -1.0], [0.0, 1.0], [0.0, -1.0]]), np.array([[1.0, 1.0, -1.0], [0.0, 0.0, 0.0]])]
    b = [np.zeros(3), np.array([0.0, 0.25])]
    X2 = rng.standard_normal((n, 2))
    st = O.init_forward(X2, W, b, np.zeros(n, dtype=int), 1.0, 1.0)
    out = O.forward(st)
    for j in range(n):
        assert abs(out[j, 0] - max(X2[j, 0], X2[j, 1])) < 1e-15 and out[j, 1] == 0.25
    pred, _ = O.predict(st)
    assert np.array_equal(pred, (np.maximum(X2[:, 0], X2[:, 1]) <= 0.25).astype(np.int32))
    # accuracy counts masked nodes only
    m = np.zeros(n, dtype=bool)
    m[:10] = True
    assert O.accuracy(pred, pred, m) == 1.0 and O.accuracy(pred, 1 - pred, m) == 0.0
    assert abs(O.accuracy(pred, np.where(np.arange(n) < 5, 1 - pred, pred), m) - 0.5) < 1e-15


def test_forward_pass_ignores_the_admm_variables():
    # the perturbed p, z, q must not enter the prediction: only X, W, b do
    w = small(n=120)
    inp = oracle_inputs(w)
    a = oracle_state(w, inp, perturbed=False)
    b = oracle_state(w, inp, perturbed=True)
    assert np.array_equal(O.forward(a), O.forward(b))
    # at the forward-consistent start the ADMM variable z_L is the model's output
    np.testing.assert_allclose(O.forward(a), a.z[-1], rtol=1e-6, atol=1e-6)


def test_growing_by_identity_layers_keeps_the_function():
    # Greedy layer-wise schedule (Section 3.2): a fresh hidden layer W = I, b = 0 placed after a ReLU layer
    # computes relu(relu(x)) = relu(x), so the grown model must reproduce the trained one's output exactly,
    # and its start must be forward-consistent (zero residuals, zero duals).
    w = small(n=150, hidden=12, n_layers=3, feat_dim=5)
    inp = oracle_inputs(w)
    mask = np.arange(w.n_nodes) % 3 != 0
    st = O.init_forward(inp["X_aug"], inp["W"], inp["b"], inp["y"], 1.0, 0.01, mask=mask)
    O.iterate(st, 5)
    h = w.hidden
    eye, zero = np.eye(h), np.zeros(h)
    deep = O.grow_layers(st, [1, 2, 0, 0, 3], [None, None, eye, eye, None], [None, None, zero, zero, None])
    assert deep.L == 5
    np.testing.assert_allclose(O.forward(deep), O.forward(st), rtol=0, atol=1e-12)
    assert np.array_equal(O.predict(deep)[0], O.predict(st)[0])
    for i, src in enumerate([1, 2, 0, 0, 3]):
        if src:
            assert np.array_equal(deep.W[i], st.W[src - 1]) and deep.W[i] is not st.W[src - 1]
            assert np.array_equal(deep.b[i], st.b[src - 1])
    for i in range(deep.L):
        assert np.max(np.abs(deep.p[i] @ deep.W[i].T + deep.b[i] - deep.z[i])) < 1e-12
        if i < deep.L - 1:
            assert not deep.u[i].any() and np.array_equal(deep.p[i + 1], deep.q[i])
    assert deep.tau == [1.0] * 5 and deep.theta == [1.0] * 5
    # the problem itself is carried over: penalties, labels, mask, activation, grid
    assert (deep.rho, deep.nu, deep.slope, deep.grid, deep.quantize_q) == (1.0, 0.01, st.slope, None, False)
    assert deep.mask is st.mask and np.array_equal(deep.y, st.y) and np.array_equal(deep.p[0], st.p[0])
    # training the grown model goes on decreasing the objective from that start
    f0 = O.objective(deep)["L_rho"]
    O.iterate(deep, 3)
    assert O.objective(deep)["L_rho"] < f0
    # a source layer of another shape is refused
    with pytest.raises(ValueError):
        O.grow_layers(st, [2, 1, 3], [None] * 3, [None] * 3)


def test_variant_with_p_and_q_on_the_grid():
    # Appendix B, last paragraph: q_l <- nearest member of Delta to the closed-form q.
    w = dataclasses.replace(small("C5", n=200, hidden=16, n_layers=4, feat_dim=6), quant_q=True)
    inp = oracle_inputs(w)
    st = oracle_state(w, inp)
    assert st.quantize_q
    mem = st.grid.members().astype(F64)
    ref = st.copy()
    ref.quantize_q = False
    for k in range(3):
        # one iteration of both; up to the q-update they see the same state
        for i in range(1, st.L):
            O.update_p(st, i); O.update_p(ref, i)
        for i in range(st.L):
            O.update_W(st, i); O.update_W(ref, i)
        for i in range(st.L):
            O.update_b(st, i); O.update_b(ref, i)
        for i in range(st.L - 1):
            O.update_z_hidden(st, i); O.update_z_hidden(ref, i)
        O.update_z_last(st); O.update_z_last(ref)
        for i in range(st.L - 1):
            O.update_q(st, i); O.update_q(ref, i)
            assert np.isin(st.q[i], mem).all()                       # q in Delta
            # it is the nearest member to the unquantised closed form (brute force over Delta), except
            # where that value sits within fp32 rounding of a midpoint
            v = ref.q[i]
            brute = mem[np.argmin(np.abs(v[..., None] - mem), axis=-1)]
            differ = st.q[i] != brute
            if differ.any():
                gap = np.abs(np.abs(v[differ] - st.q[i][differ]) - np.abs(v[differ] - brute[differ]))
                assert np.all(gap <= 1e-6)
            assert differ.sum() <= max(2, 1e-4 * differ.size)
        for i in range(st.L - 1):
            O.update_u(st, i); O.update_u(ref, i)
            # dual ascent with the projected q
            assert np.all(np.isfinite(st.u[i]))
        # continue both from the variant's state
        ref = st.copy()
        ref.quantize_q = False
    assert all(np.isin(st.p[i], mem).all() for i in range(1, st.L))


def test_leaky_activation_whole_iteration_properties():
    # with a leaky ReLU the same lemmas apply (Section 4: it satisfies the assumption, S = 1):
    # monotone L_rho under Lemma 1's condition, and every phase decreases it
    w = dataclasses.replace(small("C1", n=160, hidden=20, n_layers=4, feat_dim=8), slope=0.1, rho=1.0, nu=0.01)
    st = oracle_state(w)
    prev = O.objective(st)["L_rho"]
    for k in range(6):
        O.iterate(st)
        cur = O.objective(st)["L_rho"]
        assert cur <= prev + 1e-9 * abs(prev), (k, prev, cur)
        prev = cur
    # the objective's activation term uses the same f
    i = 1
    fz = np.where(st.z[i] > 0, st.z[i], 0.1 * st.z[i])
    direct = 0.5 * st.nu * sum(float(np.sum((st.q[j] - np.where(st.z[j] > 0, st.z[j], 0.1 * st.z[j])) ** 2))
                               for j in range(st.L - 1))
    assert abs(O.objective(st)["act_pen"] - direct) <= 1e-12 * max(1.0, direct)


def _literal_condition(st, i, t, taken=None):
    """Appendix A / B, 'update p' typed out for one trial value t of tau: candidate = nearest member of
    Delta to p - grad/t (brute force over Delta); returns (candidate, phi(candidate) <= U_l(candidate; t)).
    With `taken` (the oracle's own new p) the condition is evaluated there instead, after checking that it
    is a nearest member too (at a midpoint of Delta two members are)."""
    p = st.p[i]
    W, b, z, q, u = st.W[i], st.b[i], st.z[i], st.q[i - 1], st.u[i - 1]

    def phi_of(pp):
        r = z - pp @ W.T - b
        return 0.5 * st.nu * np.sum(r * r) + np.sum(u * (pp - q)) + 0.5 * st.rho * np.sum((pp - q) ** 2)

    g = st.nu * ((p @ W.T + b - z) @ W) + u + st.rho * (p - q)
    mem = st.grid.members().astype(F64)
    v = (p - g / t).astype(F32)                                     # the decision is taken in fp32
    cand = mem[np.argmin(np.abs(v[..., None].astype(F64) - mem), axis=-1)]
    if taken is not None:
        assert np.isin(taken, mem).all()
        assert np.all(np.abs(taken - v) <= np.abs(cand - v) + 1e-6) and np.mean(taken != cand) <= 1e-3
        cand = taken
    d = cand - p
    upper = phi_of(p) + np.sum(g * d) + 0.5 * t * np.sum(d * d)
    return cand, phi_of(cand) <= upper


def test_quantized_probe_back_off_against_the_plain_schedule():
    # Appendix A fixes only the acceptance condition phi(p_new) <= U_l(p_new; tau). The plain schedule (every
    # update starts at previous/eta) is the reference; the back-off schedule skips the start value previous/eta
    # in some updates to save a product. Property, update by update along a back-off run: (1) the accepted
    # tau satisfies the condition evaluated literally; (2) where the probe was not skipped both schedules give
    # the same tau and p; (3) where it was skipped, either the condition fails at previous/eta - then the plain
    # schedule arrives at the same tau and p - or it holds: a missed probe, the only way the two differ.
    # Missed probes must be rare.
    w = small("C5", n=150, hidden=16, n_layers=4, feat_dim=6)
    st = oracle_state(w)
    updates = skipped = missed = trials = 0
    for k in range(40):
        for i in range(1, st.L):
            before = st.copy()
            plain = st.copy()
            plain.probe_backoff = False
            O.update_p(st, i)
            O.update_p(plain, i)
            if st.p_trials[i] == 0:
                continue                                             # vanishing gradient: nothing to do
            updates += 1
            trials += st.p_trials[i]
            _, ok = _literal_condition(before, i, st.tau[i], taken=st.p[i])
            assert ok                                                # (1)
            was_skipped = before.p_skip[i] > 0
            if not was_skipped:
                assert plain.tau[i] == st.tau[i] and np.array_equal(plain.p[i], st.p[i])    # (2)
                continue
            skipped += 1
            _, ok_smaller = _literal_condition(before, i, before.tau[i] / st.eta)
            if ok_smaller:                                           # (3) a missed probe
                missed += 1
                assert plain.tau[i] == before.tau[i] / st.eta
            else:
                assert plain.tau[i] == st.tau[i] and np.array_equal(plain.p[i], st.p[i])
                assert plain.p_trials[i] == st.p_trials[i] + 1       # the plain schedule paid one more product
        for i in range(st.L):
            O.update_W(st, i)
        for i in range(st.L):
            O.update_b(st, i)
        for i in range(st.L - 1):
            O.update_z_hidden(st, i)
        O.update_z_last(st)
        for i in range(st.L - 1):
            O.update_q(st, i)
        for i in range(st.L - 1):
            O.update_u(st, i)
    assert skipped > 0.3 * updates                                   # the back-off is exercised
    assert missed <= 0.1 * skipped, (missed, skipped)
    assert trials / updates < 1.5                                    # probing every time sits near 2 once tau settles


def test_plain_schedule_of_the_quantized_variant_starts_every_update_at_previous_over_eta():
    w = small("C5", n=150, hidden=16, n_layers=3, feat_dim=6)
    st = oracle_state(w, probe_backoff=False)
    for k in range(12):
        before = st.copy()
        O.iterate(st)
        for i in range(1, st.L):
            if st.p_trials[i]:
                assert st.tau[i] == before.tau[i] / st.eta * st.eta ** (st.p_trials[i] - 1)
            assert st.p_wait[i] == 0 and st.p_skip[i] == 0           # the back-off state is never touched
            _, ok = _literal_condition_after(before, st, i)
            assert ok


def _literal_condition_after(before, after, i):
    # the p-update of layer i reads only variables of iteration k (Algorithm 1: p comes first)
    return _literal_condition(before, i, after.tau[i], taken=after.p[i]) if after.p_trials[i] else (None, True)


def test_memory_lean_mode_stores_fp32_and_follows_the_fp64_run():
    # store32: variables are rounded to fp32 once per update (the storage precision of the HIP path) and every
    # update is still computed in fp64: the run must shadow the all-fp64 run at fp32 rounding level, with the
    # same step-size decisions, for both variants.
    for name in ("C3", "C5"):
        w = small(name, n=400, hidden=40, n_layers=4, feat_dim=8)
        inp = oracle_inputs(w)
        a, b = oracle_state(w, inp), oracle_state(w, inp, store32=True)
        for k in range(6):
            O.iterate(a)
            O.iterate(b)
            assert all(x.dtype == F32 for x in b.W + b.b + b.z + b.p + b.q + b.u)
            assert all(x.dtype == F64 for x in a.W + a.b + a.z + a.q + a.u)
            assert a.tau == b.tau and a.theta == b.theta and a.p_trials == b.p_trials
            oa, ob = O.objective(a), O.objective(b)
            assert abs(oa["L_rho"] - ob["L_rho"]) <= 1e-6 * abs(oa["L_rho"])
            assert abs(O.residual(a)[0] - O.residual(b)[0]) <= 1e-5 * O.residual(a)[0]
            for x, y in zip(a.z + a.q + a.u + a.W, b.z + b.q + b.u + b.W):
                assert rel_l2(y, x) <= 1e-5       # not bit-level: a -Q index may flip at a midpoint
        c = b.copy()
        assert c.store32 and all(x.dtype == F32 for x in c.z)


def test_least_squares_risk_closed_form_against_scalar_brute_force():
    # R(z; y) = 1/2 ||z - e_y||^2: the z_L-subproblem of Appendix A is separable per element,
    # h(z) = 1/2 (z - t)^2 + (nu/2)(z - a)^2 with t = 1 for the labelled class and 0 otherwise.
    rng = np.random.default_rng(5)
    n, c, nu = 40, 5, 0.37
    a = rng.standard_normal((n, c)) * 3
    y = rng.integers(0, c, size=n)
    mask = rng.random(n) < 0.7
    z = O.least_squares_z_last(a, y, nu, mask)
    t = np.zeros((n, c)); t[np.arange(n), y] = 1.0
    grid = np.linspace(-12, 12, 480001)                              # 5e-5 spacing
    for j in range(0, n, 3):
        for k in range(c):
            if mask[j]:
                h = 0.5 * (grid - t[j, k]) ** 2 + 0.5 * nu * (grid - a[j, k]) ** 2
                assert abs(grid[np.argmin(h)] - z[j, k]) <= 5e-5
            else:
                assert z[j, k] == a[j, k]                            # no risk term: the minimiser of the penalty alone
    # the risk value itself, by hand: two nodes, three classes
    zz = np.array([[1.0, 0.0, 0.0], [0.5, 0.5, 2.0]])
    assert O.risk(zz, np.array([0, 1]), kind="ls") == 0.5 * (0.25 + 0.25 + 4.0)
    assert O.risk(zz, np.array([0, 1]), mask=np.array([True, False]), kind="ls") == 0.0


def test_least_squares_risk_whole_iteration_properties():
    # the same lemmas hold for any convex risk: monotone L_rho under Lemma 1's condition, dual identity
    # u = nu (q - f(z)); and the exact z_L-update makes the z-phase decrease hold without FISTA slack
    w = dataclasses.replace(small("C1", n=160, hidden=20, n_layers=4, feat_dim=8), rho=1.0, nu=0.01)
    st = oracle_state(w, risk_kind="ls")
    prev = O.objective(st)["L_rho"]
    for k in range(8):
        O.iterate(st)
        ob = O.objective(st)
        assert ob["L_rho"] <= prev + 1e-12 * abs(prev), (k, prev, ob["L_rho"])
        prev = ob["L_rho"]
        for i in range(st.L - 1):
            assert np.max(np.abs(st.u[i] - st.nu * (st.q[i] - np.maximum(st.z[i], 0)))) <= 1e-12
        t = np.zeros_like(st.z[-1]); t[np.arange(t.shape[0]), st.y] = 1.0
        assert abs(ob["risk"] - 0.5 * np.sum((st.z[-1] - t) ** 2)) <= 1e-12 * max(1.0, ob["risk"])
        # stationarity of the z_L-subproblem
        a = st.p[-1] @ st.W[-1].T + st.b[-1]
        assert np.max(np.abs((st.z[-1] - t) + st.nu * (st.z[-1] - a))) <= 1e-12


def test_golden_writer_runs_layers_side_by_side_with_the_same_result():
    # tests/golden/write_golden.py spreads the per-layer updates of a phase over forked child processes for the two
    # largest workloads: same function calls, same order of phases, so the same run as O.iterate
    import importlib.util
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "write_golden.py")
    spec = importlib.util.spec_from_file_location("write_golden", path)
    wg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(wg)
    for name in ("C3", "C5"):
        w = small(name, n=300, hidden=24, n_layers=5, feat_dim=6)
        a = oracle_state(w, store32=True)
        b = a.copy()
        for k in range(4):
            O.iterate(a)
            wg.iterate_layers_side_by_side(b, 3)
            assert a.tau == b.tau and a.theta == b.theta and a.p_trials == b.p_trials and a.p_skip == b.p_skip
            for x, y in zip(a.W + a.b + a.z + a.p + a.q + a.u, b.W + b.b + b.z + b.p + b.q + b.u):
                assert np.array_equal(x, y)
