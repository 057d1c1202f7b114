"""Pins for the CPU oracle: each test ties an oracle function to something the paper or
the mathematics fixes -- never to the oracle's own formula retyped.

Citations are to the paper: Sec. 1 / Eq. 1 (problem and scaling iteration), Algorithm 1
(iteration order, init, row partition), Proposition 1 (blocked == centralised),
Sec. 5.3.2 (multitarget), Sec. 3.3 (damping), App. "Convergence proofs" (Hilbert metric,
fixed point), App. toy portfolio example (printed cost and plan).
"""
import os

import numpy as np
import pytest
import scipy.optimize
import scipy.special

HERE = os.path.dirname(os.path.abspath(__file__))


def problem(n, seed, d=2, eps=0.1, symmetric=False):
    rng = np.random.default_rng(seed)
    x = rng.uniform(size=(n, d))
    y = x.copy() if symmetric else rng.uniform(size=(n, d)) + 0.3
    a = rng.uniform(0.5, 1.5, n); a /= a.sum()
    b = a.copy() if symmetric else rng.uniform(0.5, 1.5, n)
    b /= b.sum()
    C = ((x[:, None, :] - y[None, :, :]) ** 2).sum(-1)      # NumPy, not the oracle
    K = np.exp(-C / eps)
    return x, y, a, b, C, K


def primal_objective(P, C, eps):
    """Eq. 1: <P,C> + eps * sum P (log P - 1)."""
    return float((P * C).sum() + eps * (P * (np.log(P) - 1.0)).sum())


def dual_objective(f, g, a, b, C, eps):
    """Lagrangian dual of Eq. 1: <f,a> + <g,b> - eps * sum exp((f_i + g_j - C_ij)/eps)."""
    return float(f @ a + g @ b - eps * np.exp((f[:, None] + g[None, :] - C) / eps).sum())


# ---------------------------------------------------------------- setup ----

def test_cost_and_gibbs_against_numpy(orc):
    x, y, a, b, C, K = problem(37, 1, d=5)
    assert np.allclose(orc.cost_sqeuclid(x, y), C, rtol=1e-14, atol=0)
    assert np.allclose(orc.gibbs(C, 0.1), K, rtol=1e-14, atol=0)
    Kn, cmax = orc.gibbs_from_points(x, y, 0.07, True)
    assert cmax == pytest.approx(C.max(), rel=1e-15)
    assert np.allclose(Kn, np.exp(-(C / C.max()) / 0.07), rtol=1e-14, atol=0)
    # the asymmetric cost catches a swapped (x, y) or transposed output
    assert not np.allclose(C, C.T)


def test_gibbs_f32_variant_is_the_rounded_f64_kernel(orc):
    x, y, a, b, C, K = problem(64, 2, d=3)
    for norm in (False, True):
        K64, cmax = orc.gibbs_from_points(x, y, 0.05, norm)
        K32, cmax32 = orc.gibbs_from_points_f32(x, y, 0.05, norm)
        assert K32.dtype == np.float32 and cmax32 == cmax
        assert np.array_equal(K32, K64.astype(np.float32))
    assert orc.max_sqeuclid(x, y) == pytest.approx(C.max(), rel=1e-15)
    assert orc.max_sqeuclid(x[:5], y) == pytest.approx(C[:5].max(), rel=1e-15)   # rectangular
    # d > 1 on clouds of different extent (a wrong stride in either operand shows), maximum below 1
    rng = np.random.default_rng(17)
    xs = 0.1 * rng.uniform(size=(23, 4)) * np.array([1.0, 5.0, 0.2, 3.0]); ys = 0.1 * rng.uniform(size=(31, 4))
    want = ((xs[:, None, :] - ys[None, :, :]) ** 2).sum(-1).max()
    assert want < 1.0 and orc.max_sqeuclid(xs, ys) == pytest.approx(want, rel=1e-14)


# ------------------------------------------- single steps vs library routines

def test_products_against_numpy_matmul(orc):
    """x -> K x and x -> K^T x (Sec. 3.1) against NumPy's matmul on an asymmetric K."""
    x, y, a, b, C, K = problem(53, 3)
    rng = np.random.default_rng(0)
    v = rng.uniform(0.5, 2.0, 53); u = rng.uniform(0.5, 2.0, 53)
    assert np.allclose(orc.row_products(K, v), K @ v, rtol=1e-13)
    assert np.allclose(orc.col_products(K, u), K.T @ u, rtol=1e-13)
    assert not np.allclose(K @ v, K.T @ v, rtol=1e-3)       # a transposed operand would show
    # ranges: a row slab and a column slab
    assert np.allclose(orc.row_products(K, v, 10, 31), (K @ v)[10:31], rtol=1e-13)
    assert np.allclose(orc.col_products(K, u, 0, 53, 7, 20), (K.T @ u)[7:20], rtol=1e-13)
    assert np.allclose(orc.col_products(K, u, 10, 31), K[10:31].T @ u[10:31], rtol=1e-13)
    # more columns than one of the loop's column chunks, ragged last chunk, rectangular slab
    Kb = rng.uniform(0.1, 1.0, (90, 700)); ub = rng.uniform(0.5, 2.0, 90); vb = rng.uniform(0.5, 2.0, 700)
    assert np.allclose(orc.col_products(Kb, ub), Kb.T @ ub, rtol=1e-13)
    assert np.allclose(orc.col_products(Kb, ub, 5, 80, 100, 650), (Kb[5:80].T @ ub[5:80])[100:650], rtol=1e-13)
    assert np.allclose(orc.row_products(Kb, vb), Kb @ vb, rtol=1e-13)


def test_first_iteration_against_numpy(orc):
    """Algorithm 1 from u = v = 1: u1 = a ./ (K 1), v1 = b ./ (K^T u1); order u then v."""
    x, y, a, b, C, K = problem(41, 4)
    u1 = a / (K @ np.ones(41)); v1 = b / (K.T @ u1)
    u, v = orc.sinkhorn_dense(K, a, b, 1)
    assert np.allclose(u, u1, rtol=1e-13) and np.allclose(v, v1, rtol=1e-13)
    u2 = a / (K @ v1); v2 = b / (K.T @ u2)
    u, v = orc.sinkhorn_dense(K, a, b, 2)
    assert np.allclose(u, u2, rtol=1e-13) and np.allclose(v, v2, rtol=1e-13)
    # zero iterations leave the init untouched
    u, v = orc.sinkhorn_dense(K, a, b, 0)
    assert np.array_equal(u, np.ones(41)) and np.array_equal(v, np.ones(41))


def test_lse_against_scipy(orc):
    rng = np.random.default_rng(5)
    for scale in (1.0, 50.0, 700.0):
        z = rng.normal(size=200) * scale
        assert orc.lse(z) == pytest.approx(scipy.special.logsumexp(z), rel=1e-14)
    assert orc.lse(np.array([-2000.0, -2001.0])) == pytest.approx(-2000.0 + np.log1p(np.exp(-1.0)))


# -------------------------------------------------- what the definition fixes

def test_marginals_exact_after_each_half_step(orc):
    """P = diag(u) K diag(v): P 1 = a right after the u-update, P^T 1 = b right after the
    v-update (Sec. 1, scaling form)."""
    x, y, a, b, C, K = problem(64, 6)
    u, v = orc.sinkhorn_dense(K, a, b, 3)
    P = u[:, None] * K * v[None, :]
    assert np.allclose(P.sum(0), b, rtol=1e-13)             # last update was v
    assert not np.allclose(P.sum(1), a, rtol=1e-6)          # rows are not yet exact
    u_next = a / (K @ v)                                    # the u-update that follows
    assert np.allclose((u_next[:, None] * K * v[None, :]).sum(1), a, rtol=1e-13)
    assert np.allclose(orc.row_marginal(K, u, v), P.sum(1), rtol=1e-13)
    assert np.allclose(orc.col_marginal(K, u, v), P.sum(0), rtol=1e-13)
    e1, e2 = orc.marginal_error(K, a, u, v)
    assert e1 == pytest.approx(np.abs(P.sum(1) - a).sum(), rel=1e-12)
    assert e2 == pytest.approx(np.sqrt(((P.sum(1) - a) ** 2).sum()), rel=1e-12)


def test_constant_cost_gives_product_plan(orc):
    """C == kappa  =>  after one iteration P = a b^T / (1^T a), and it is a fixed point."""
    n, kappa, eps = 17, 0.37, 0.05
    rng = np.random.default_rng(7)
    a = rng.uniform(0.5, 1.5, n); a /= a.sum()
    b = rng.uniform(0.5, 1.5, n); b /= b.sum()
    K = orc.gibbs(np.full((n, n), kappa), eps)
    k = np.exp(-kappa / eps)
    u, v = orc.sinkhorn_dense(K, a, b, 1)
    assert np.allclose(u, a / (k * n), rtol=1e-13)
    assert np.allclose(v, b * n / a.sum(), rtol=1e-13)
    assert np.allclose(u[:, None] * K * v[None, :], np.outer(a, b), rtol=1e-13)
    u2, v2 = orc.sinkhorn_dense(K, a, b, 5)
    assert np.allclose(u2, u, rtol=1e-13) and np.allclose(v2, v, rtol=1e-13)


def test_two_by_two_brute_force_optimum(orc):
    """n = 2: the feasible set of Eq. 1 is one-dimensional; minimise the objective over it
    with a library scalar minimiser and compare with the converged scaling iteration."""
    C = np.array([[0.10, 0.70], [0.45, 0.05]])
    a = np.array([0.35, 0.65]); b = np.array([0.6, 0.4])
    eps = 0.2

    def plan(p):
        return np.array([[p, a[0] - p], [b[0] - p, a[1] - b[0] + p]])

    lo = max(0.0, b[0] - a[1]) + 1e-12
    hi = min(a[0], b[0]) - 1e-12
    res = scipy.optimize.minimize_scalar(lambda p: primal_objective(plan(p), C, eps),
                                         bounds=(lo, hi), method="bounded",
                                         options={"xatol": 1e-14})
    K = orc.gibbs(C, eps)
    u, v = orc.sinkhorn_dense(K, a, b, 2000)
    P = u[:, None] * K * v[None, :]
    assert np.allclose(P, plan(res.x), atol=2e-7)
    # brute force on a grid as well: nothing on the segment beats the Sinkhorn plan
    grid = np.linspace(lo, hi, 20001)
    best = min(primal_objective(plan(p), C, eps) for p in grid)
    assert primal_objective(P, C, eps) <= best + 1e-12


def test_three_by_three_brute_force_optimum(orc):
    """n = 3: with both marginals fixed the plan has 4 free entries; minimise Eq. 1 over them
    with a library minimiser (derivative-free, then polished) from the product plan."""
    rng = np.random.default_rng(8)
    C = rng.uniform(0.0, 1.0, (3, 3))
    a = np.array([0.2, 0.5, 0.3]); b = np.array([0.4, 0.25, 0.35])
    eps = 0.3

    def plan(p):
        P = np.empty((3, 3))
        P[:2, :2] = p.reshape(2, 2)
        P[:2, 2] = a[:2] - P[:2, :2].sum(1)
        P[2, :2] = b[:2] - P[:2, :2].sum(0)
        P[2, 2] = a[2] - P[2, :2].sum()
        return P

    def obj(p):
        P = plan(p)
        return primal_objective(P, C, eps) if (P > 0).all() else np.inf

    p0 = np.outer(a, b)[:2, :2].ravel()
    res = scipy.optimize.minimize(obj, p0, method="Nelder-Mead",
                                  options={"xatol": 1e-12, "fatol": 1e-16, "maxiter": 20000})
    res = scipy.optimize.minimize(obj, res.x, method="BFGS", options={"gtol": 1e-12})
    K = orc.gibbs(C, eps)
    u, v = orc.sinkhorn_dense(K, a, b, 3000)
    P = u[:, None] * K * v[None, :]
    assert np.allclose(P, plan(res.x), atol=1e-6)
    assert primal_objective(P, C, eps) <= res.fun + 1e-12


def test_dual_ascent_and_zero_gap(orc):
    """Each half-step maximises the dual exactly in one block => the dual value never
    decreases; at convergence it equals the primal value of Eq. 1 at P."""
    x, y, a, b, C, K = problem(12, 9, eps=0.1)
    eps = 0.1
    u, v = np.ones(12), np.ones(12)
    prev = dual_objective(eps * np.log(u), eps * np.log(v), a, b, C, eps)
    for t in range(30):
        u, v = orc.sinkhorn_dense(K, a, b, 1, u0=u, v0=v)
        cur = dual_objective(eps * np.log(u), eps * np.log(v), a, b, C, eps)
        assert cur >= prev - 1e-13
        prev = cur
    u, v = orc.sinkhorn_dense(K, a, b, 3000)
    P = u[:, None] * K * v[None, :]
    D = dual_objective(eps * np.log(u), eps * np.log(v), a, b, C, eps)
    assert D == pytest.approx(primal_objective(P, C, eps), abs=1e-12)
    # any other feasible plan is worse (weak duality, brute force over random feasible moves)
    rng = np.random.default_rng(0)
    for _ in range(200):
        i, k = rng.choice(12, 2, replace=False); j, l = rng.choice(12, 2, replace=False)
        step = 0.5 * min(P[i, j], P[k, l], P[i, l], P[k, j]) * rng.uniform(-1, 1)
        Q = P.copy()
        Q[i, j] += step; Q[k, l] += step; Q[i, l] -= step; Q[k, j] -= step
        assert primal_objective(Q, C, eps) >= primal_objective(P, C, eps) - 1e-14


def test_fixed_point_and_gauge(orc):
    """At convergence both scaling equations hold at once; a different init gauge (u0 = s,
    v0 = 1/s .. any positive start) reaches the same plan (App. convergence, uniqueness of P*)."""
    x, y, a, b, C, K = problem(20, 10, eps=0.2)
    u, v = orc.sinkhorn_dense(K, a, b, 4000)
    assert np.allclose(u, a / (K @ v), rtol=1e-12) and np.allclose(v, b / (K.T @ u), rtol=1e-12)
    rng = np.random.default_rng(1)
    u2, v2 = orc.sinkhorn_dense(K, a, b, 4000, u0=rng.uniform(0.1, 10, 20), v0=rng.uniform(0.1, 10, 20))
    assert np.allclose(u[:, None] * K * v[None, :], u2[:, None] * K * v2[None, :], rtol=1e-10)
    ratio = u2 / u
    assert np.allclose(ratio, ratio[0], rtol=1e-9) and np.allclose(v2 / v, 1.0 / ratio[0], rtol=1e-9)


def test_symmetric_special_case(orc):
    """x = y and a = b (the paper's own experimental setting, symmetric C): the optimal plan
    is symmetric and u is proportional to v."""
    x, y, a, b, C, K = problem(24, 11, eps=0.15, symmetric=True)
    assert np.allclose(C, C.T)
    u, v = orc.sinkhorn_dense(K, a, b, 5000)
    P = u[:, None] * K * v[None, :]
    assert np.allclose(P, P.T, rtol=1e-9, atol=1e-15)
    assert np.allclose(u / v, (u / v)[0], rtol=1e-9)


def test_hilbert_metric_contracts(orc):
    """d_H(u^{t+1}, u^t) is non-increasing (x -> Kx contracts, x -> a./x is an isometry)."""
    def d_h(p, q):
        r = p / q
        return np.log(r.max()) - np.log(r.min())
    x, y, a, b, C, K = problem(30, 12, eps=0.05)
    us = [np.ones(30)]
    u, v = np.ones(30), np.ones(30)
    for _ in range(25):
        u, v = orc.sinkhorn_dense(K, a, b, 1, u0=u, v0=v)
        us.append(u)
    d = [d_h(us[t + 1], us[t]) for t in range(1, 25)]
    assert all(d[t + 1] <= d[t] * (1 + 1e-12) for t in range(len(d) - 1))
    assert d[-1] < d[0]


# ------------------------------------------------------------ identities ---

@pytest.mark.parametrize("c", [1, 2, 4, 8])
def test_blocked_equals_centralised(orc, c):
    """Proposition 1: the row-partitioned iterates coincide with the centralised ones."""
    x, y, a, b, C, K = problem(48, 13)
    u, v = orc.sinkhorn_dense(K, a, b, 25)
    ua, va = orc.sinkhorn_blocked(K, a, b, 25, c, 0)
    assert np.array_equal(ua, u) and np.array_equal(va, v)  # same sums, same order
    ub, vb = orc.sinkhorn_blocked(K, a, b, 25, c, 1)
    assert np.allclose(ub, u, rtol=1e-13) and np.allclose(vb, v, rtol=1e-13)
    with pytest.raises(ValueError):
        orc.sinkhorn_blocked(K, a, b, 1, 5, 0)              # n = c m is required


def test_resume_equals_straight_run(orc):
    x, y, a, b, C, K = problem(33, 14)
    u, v = orc.sinkhorn_dense(K, a, b, 40)
    u1, v1 = orc.sinkhorn_dense(K, a, b, 15)
    u2, v2 = orc.sinkhorn_dense(K, a, b, 25, u0=u1, v0=v1)
    assert np.array_equal(u2, u) and np.array_equal(v2, v)


def test_f32_storage_is_promoted_entrywise(orc):
    x, y, a, b, C, K = problem(40, 15)
    K32 = K.astype(np.float32)
    u, v = orc.sinkhorn_dense(K32, a, b, 20)
    u64, v64 = orc.sinkhorn_dense(K32.astype(np.float64), a, b, 20)
    assert np.array_equal(u, u64) and np.array_equal(v, v64)


def test_batched_column_equals_single_run(orc):
    """Multitarget form (Sec. 5.3.2): column k of the stacked run is the run on (a_k, b_k)."""
    x, y, a, b, C, K = problem(26, 16)
    rng = np.random.default_rng(3)
    m = 5
    A = rng.exponential(size=(26, m)); A /= A.sum(0)
    B = rng.exponential(size=(26, m)); B /= B.sum(0)
    U, V = orc.sinkhorn_batched(K, A, B, 30)
    for k in range(m):
        u, v = orc.sinkhorn_dense(K, A[:, k], B[:, k], 30)
        assert np.allclose(U[:, k], u, rtol=1e-13) and np.allclose(V[:, k], v, rtol=1e-13)
    # first step against a library GEMM
    U1, V1 = orc.sinkhorn_batched(K, A, B, 1)
    Uref = A / (K @ np.ones((26, m)))
    assert np.allclose(U1, Uref, rtol=1e-13) and np.allclose(V1, B / (K.T @ Uref), rtol=1e-13)


def test_batched_damped_column_equals_single_damped_run(orc):
    x, y, a, b, C, K = problem(22, 29, eps=0.3)
    K = K + 0.05 * np.random.default_rng(1).uniform(size=K.shape)      # K != K^T: a transposed walk would show
    rng = np.random.default_rng(6)
    m = 4
    A = rng.exponential(size=(22, m)); A /= A.sum(0)
    B = rng.exponential(size=(22, m)); B /= B.sum(0)
    for geometric in (False, True):
        U, V = orc.sinkhorn_batched_damped(K, A, B, 17, 0.55, geometric)
        for k in range(m):
            u, v = orc.sinkhorn_dense_damped(K, A[:, k], B[:, k], 17, 0.55, geometric)
            assert np.allclose(U[:, k], u, rtol=1e-13) and np.allclose(V[:, k], v, rtol=1e-13)
        U1, V1 = orc.sinkhorn_batched_damped(K, A, B, 9, 1.0, geometric)   # eta = 1: the plain iteration
        U0, V0 = orc.sinkhorn_batched(K, A, B, 9)
        assert np.allclose(U1, U0, rtol=1e-13) and np.allclose(V1, V0, rtol=1e-13)


def test_batched_tolerance_mode(orc):
    """The stacked run stops at the first poll where EVERY target is below the tolerance: its
    error is the largest of the per-target errors (NumPy, from the plan), its iterates are those
    of the fixed-count run, and with a poll every iteration it stops where the slowest
    single-target run stops (the L1 marginal error of Sinkhorn never increases)."""
    x, y, a, b, C, K = problem(30, 23, eps=0.3)
    rng = np.random.default_rng(4)
    m = 6
    A = rng.exponential(size=(30, m)); A /= A.sum(0)
    B = rng.exponential(size=(30, m)); B /= B.sum(0)
    U, V, done, err = orc.sinkhorn_batched_tol(K, A, B, 500, 1e-8, check_every=1)
    assert 1 < done < 500 and err < 1e-8
    errs = [np.abs((U[:, k, None] * K * V[None, :, k]).sum(1) - A[:, k]).sum() for k in range(m)]
    assert err == pytest.approx(max(errs), rel=1e-5)                     # cancellation-limited
    Uf, Vf = orc.sinkhorn_batched(K, A, B, done)
    assert np.array_equal(U, Uf) and np.array_equal(V, Vf)
    singles = [orc.sinkhorn_dense_tol(K, A[:, k], B[:, k], 500, 1e-8, check_every=1)[2] for k in range(m)]
    assert done == max(singles) and min(singles) < done                   # the targets differ
    # polling interval and cap
    _, _, done5, err5 = orc.sinkhorn_batched_tol(K, A, B, 500, 1e-8, check_every=5)
    assert done5 % 5 == 0 and done <= done5 < done + 5 and err5 < 1e-8
    _, _, done_cap, err_cap = orc.sinkhorn_batched_tol(K, A, B, 3, 1e-30, check_every=2)
    assert done_cap == 3 and err_cap > 1e-30
    # one target: the dense tolerance run
    U1, V1, d1, e1 = orc.sinkhorn_batched_tol(K, A[:, :1], B[:, :1], 500, 1e-8, check_every=3)
    us, vs, ds, es = orc.sinkhorn_dense_tol(K, A[:, 0], B[:, 0], 500, 1e-8, check_every=3)
    assert d1 == ds and e1 == pytest.approx(es, rel=1e-9) and np.allclose(U1[:, 0], us, rtol=1e-13)


def test_log_domain_relaxed_updates(orc):
    """Both relaxations of Sec. 3.3 in the log domain against the dense damped iteration
    (f = eps log u, a fp64 identity at moderate eps), eta = 1 against the plain log iteration,
    and one arithmetic step written out with SciPy's logsumexp."""
    from scipy.special import logsumexp
    rng = np.random.default_rng(8)
    n, d, eps = 40, 3, 0.4
    x = rng.uniform(size=(n, d)); y = rng.uniform(size=(n, d))
    a = rng.uniform(0.5, 1.5, n); a /= a.sum()
    b = rng.uniform(0.5, 1.5, n); b /= b.sum()
    K = np.exp(-orc.cost_sqeuclid(x, y) / eps)
    for geometric in (False, True):
        u, v = orc.sinkhorn_dense_damped(K, a, b, 25, 0.6, geometric)
        f, g = orc.sinkhorn_log_points_damped(x, y, eps, a, b, 25, 0.6, geometric)
        assert np.allclose(f, eps * np.log(u), rtol=0, atol=1e-12) and np.allclose(g, eps * np.log(v), rtol=0, atol=1e-12)
        f1, g1 = orc.sinkhorn_log_points_damped(x, y, eps, a, b, 9, 1.0, geometric)
        f0, g0, _, _ = orc.sinkhorn_log_points(x, y, eps, a, b, 9)
        assert np.allclose(f1, f0, rtol=0, atol=1e-14) and np.allclose(g1, g0, rtol=0, atol=1e-14)
    # first arithmetic f-step from f = g = 0 by hand
    C = orc.cost_sqeuclid(x, y)
    f_new = eps * np.log(a) - eps * logsumexp(-C / eps, axis=1)
    want = eps * logsumexp(np.stack([np.log(0.3) + np.zeros(n), np.log(0.7) + f_new / eps]), axis=0)
    f, g = orc.sinkhorn_log_points_damped(x, y, eps, a, b, 1, 0.7, False)
    assert np.allclose(f, want, rtol=0, atol=1e-13)
    # small eps: the arithmetic form must not overflow where exp(f / eps) would
    fs, gs = orc.sinkhorn_log_points_damped(x, y, 1e-4, a, b, 5, 0.5, False)
    assert np.isfinite(fs).all() and np.isfinite(gs).all() and np.abs(fs / 1e-4).max() > 710   # exp would overflow


def test_tolerance_mode_polling(orc):
    x, y, a, b, C, K = problem(32, 17, eps=0.3)
    u, v, done, err = orc.sinkhorn_dense_tol(K, a, b, 500, 1e-9, check_every=7)
    assert done % 7 == 0 and done < 500 and err < 1e-9
    P = u[:, None] * K * v[None, :]
    assert err == pytest.approx(np.abs(P.sum(1) - a).sum(), rel=1e-4)   # cancellation-limited
    # one poll earlier the error was still above the tolerance
    u7, v7 = orc.sinkhorn_dense(K, a, b, done - 7)
    assert np.abs((u7[:, None] * K * v7[None, :]).sum(1) - a).sum() >= 1e-9
    # the cap binds when the tolerance is unreachable
    _, _, done, err = orc.sinkhorn_dense_tol(K, a, b, 10, 1e-300, check_every=4)
    assert done == 10 and err > 0


def test_stop_rule_on_the_two_norm(orc):
    """The paper's own metric, err_a = ||P1 - a||_2 (Sec. 5.4): the stop iteration is the first
    poll at which NumPy's evaluation of that norm on the plain iteration's state is below the
    threshold; it comes no later than the 1-norm's, and the three forms agree on it."""
    x, y, a, b, C, K = problem(40, 23, eps=0.3)
    tol, ce = 1e-7, 3
    u, v, done, err = orc.sinkhorn_dense_tol(K, a, b, 500, tol, check_every=ce, l2=True)
    norms = []
    for t in range(ce, done + 1, ce):
        ut, vt = orc.sinkhorn_dense(K, a, b, t)
        norms.append(np.linalg.norm((ut[:, None] * K * vt[None, :]).sum(1) - a))
    assert done % ce == 0 and norms[-1] < tol and all(e >= tol for e in norms[:-1])
    assert err == pytest.approx(norms[-1], rel=1e-6)
    u1, v1, done1, err1 = orc.sinkhorn_dense_tol(K, a, b, 500, tol, check_every=ce)
    assert done <= done1 and err1 < tol
    ut, vt = orc.sinkhorn_dense(K, a, b, done)
    assert np.array_equal(u, ut) and np.array_equal(v, vt)
    # log domain: same state, same count, same error
    f, g, done_l, err_l = orc.sinkhorn_log_points(x, y, 0.3, a, b, 500, tol, ce, l2=True)
    assert done_l == done and err_l == pytest.approx(err, rel=1e-4)
    # multitarget: the slowest column decides, each column in its own 2-norm
    rng = np.random.default_rng(3)
    A = rng.uniform(0.5, 1.5, (40, 5)) ** 3; A /= A.sum(0)
    B = rng.uniform(0.5, 1.5, (40, 5)) ** 3; B /= B.sum(0)
    U, V, done_b, err_b = orc.sinkhorn_batched_tol(K, A, B, 500, tol, ce, l2=True)
    singles = [orc.sinkhorn_dense_tol(K, A[:, k], B[:, k], 500, tol, check_every=ce, l2=True) for k in range(5)]
    assert done_b == max(s[2] for s in singles)
    col = [np.linalg.norm((U[:, k, None] * K * V[None, :, k]).sum(1) - A[:, k]) for k in range(5)]
    assert err_b == pytest.approx(max(col), rel=1e-5) and err_b < tol


# ------------------------------------------------------------ log domain ---

def test_log_domain_equals_dense(orc):
    """f = eps log u, g = eps log v: the log-sum-exp form is the logarithm of the iteration."""
    x, y, a, b, C, K = problem(28, 18, d=4, eps=0.1)
    u, v = orc.sinkhorn_dense(K, a, b, 35)
    f, g = orc.sinkhorn_log_cost(C, 0.1, a, b, 35)
    assert np.allclose(f, 0.1 * np.log(u), rtol=0, atol=1e-13)
    assert np.allclose(g, 0.1 * np.log(v), rtol=0, atol=1e-13)
    fp, gp, done, _ = orc.sinkhorn_log_points(x, y, 0.1, a, b, 35)
    assert done == 35
    assert np.allclose(fp, f, rtol=0, atol=1e-13) and np.allclose(gp, g, rtol=0, atol=1e-13)


def test_log_domain_survives_where_dense_underflows(orc):
    """Small eps: K underflows to 0 in fp64 yet the potentials stay finite and the plan
    exp((f+g-C)/eps) has exact column sums after a g-update."""
    rng = np.random.default_rng(19)
    n, d, eps = 40, 16, 0.002
    x = rng.uniform(size=(n, d)); y = rng.uniform(size=(n, d))
    a = np.full(n, 1.0 / n); b = np.full(n, 1.0 / n)
    C = ((x[:, None, :] - y[None, :, :]) ** 2).sum(-1)
    assert np.exp(-C / eps).min() == 0.0
    f, g, done, _ = orc.sinkhorn_log_points(x, y, eps, a, b, 50)
    assert np.isfinite(f).all() and np.isfinite(g).all()
    logP = (f[:, None] + g[None, :] - C) / eps
    assert np.allclose(np.exp(scipy.special.logsumexp(logP, axis=0)), b, rtol=1e-11)
    rows = orc.log_row_marginal_points(x, f, y, g, eps)
    assert np.allclose(rows, np.exp(scipy.special.logsumexp(logP, axis=1)), rtol=1e-11)


def test_log_update_rows_against_scipy(orc):
    rng = np.random.default_rng(20)
    n, d, eps = 50, 6, 0.05
    x = rng.uniform(size=(n, d)); y = rng.uniform(size=(n, d))
    a = rng.uniform(0.5, 1.5, n); a /= a.sum()
    g = rng.normal(size=n) * 0.1
    C = ((x[:, None, :] - y[None, :, :]) ** 2).sum(-1)
    ref = eps * np.log(a) - eps * scipy.special.logsumexp((g[None, :] - C) / eps, axis=1)
    assert np.allclose(orc.log_update_points(x, a, y, g, eps), ref, rtol=0, atol=1e-14)
    rows = np.array([3, 17, 49, 0])
    assert np.allclose(orc.log_update_points(x, a, y, g, eps, rows), ref[rows], rtol=0, atol=1e-14)
    # the g-update is the same routine with the clouds' roles swapped (cost is symmetric in them)
    f = rng.normal(size=n) * 0.1
    refg = eps * np.log(a) - eps * scipy.special.logsumexp((f[:, None] - C) / eps, axis=0)
    assert np.allclose(orc.log_update_points(y, a, x, f, eps), refg, rtol=0, atol=1e-14)


def test_log_tolerance_mode(orc):
    rng = np.random.default_rng(21)
    n, d, eps = 60, 3, 0.2
    x = rng.uniform(size=(n, d)); y = rng.uniform(size=(n, d))
    a = np.full(n, 1.0 / n); b = np.full(n, 1.0 / n)
    f, g, done, err = orc.sinkhorn_log_points(x, y, eps, a, b, 400, tol=1e-8, check_every=5)
    assert done % 5 == 0 and done < 400 and err < 1e-8
    C = ((x[:, None, :] - y[None, :, :]) ** 2).sum(-1)
    P = np.exp((f[:, None] + g[None, :] - C) / eps)
    assert err == pytest.approx(np.abs(P.sum(1) - a).sum(), rel=1e-6, abs=1e-16)


# --------------------------------------------------------------- damping ---

def test_damped_updates(orc):
    """Sec. 3.3: eta = 1 is the plain iteration; one arithmetic step is the convex combination;
    one geometric step is linear interpolation of the log scalings; both keep the fixed point."""
    x, y, a, b, C, K = problem(22, 22, eps=0.2)
    u, v = orc.sinkhorn_dense(K, a, b, 9)
    for geo in (False, True):
        ud, vd = orc.sinkhorn_dense_damped(K, a, b, 9, 1.0, geo)
        assert np.allclose(ud, u, rtol=1e-13) and np.allclose(vd, v, rtol=1e-13)
    rng = np.random.default_rng(2)
    u0 = rng.uniform(0.5, 2, 22); v0 = rng.uniform(0.5, 2, 22)
    eta = 0.3
    ua, va = orc.sinkhorn_dense_damped(K, a, b, 1, eta, False, u0=u0, v0=v0)
    ua_ref = (1 - eta) * u0 + eta * a / (K @ v0)
    assert np.allclose(ua, ua_ref, rtol=1e-13)
    assert np.allclose(va, (1 - eta) * v0 + eta * b / (K.T @ ua_ref), rtol=1e-13)
    ug, vg = orc.sinkhorn_dense_damped(K, a, b, 1, eta, True, u0=u0, v0=v0)
    ug_ref = np.exp((1 - eta) * np.log(u0) + eta * np.log(a / (K @ v0)))
    assert np.allclose(ug, ug_ref, rtol=1e-13)
    assert np.allclose(vg, np.exp((1 - eta) * np.log(v0) + eta * np.log(b / (K.T @ ug_ref))), rtol=1e-13)
    us, vs = orc.sinkhorn_dense(K, a, b, 4000)
    Pstar = us[:, None] * K * vs[None, :]
    for geo in (False, True):
        ud, vd = orc.sinkhorn_dense_damped(K, a, b, 6000, 0.5, geo)
        assert np.allclose(ud[:, None] * K * vd[None, :], Pstar, rtol=1e-8)


# ------------------------------------------------- the paper's toy example ---

def _read_toy():
    vals = {}
    with open(os.path.join(HERE, "golden", "toy_portfolio.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, rest = line.split(":")
            vals[key.strip()] = np.array([float(t) for t in rest.split()])
    return vals


def test_toy_portfolio_example(orc):
    """App. "Toy portfolio example: numerical details": printed C, marginals from the shifted
    returns, eps = 0.01, and the printed plan.  What the printed numbers do fix: the marginals
    are the normalised shifted returns; the printed plan's column sums equal b to 3 s.f.; its
    support pattern (mass on (1,1), (2,1), (3,3)) is the one the converged iteration finds.
    The printed entries themselves are NOT reproducible from the printed inputs (their row
    sums differ from a), so they pin nothing more than that."""
    t = _read_toy()
    C = t["C"].reshape(3, 3)
    a = t["x_shifted"] / t["x_shifted"].sum()
    b = t["xp_shifted"] / t["xp_shifted"].sum()
    Pprint = t["P_star"].reshape(3, 3)
    eps = float(t["eps"][0])
    assert np.allclose(Pprint.sum(0), b, rtol=1e-2)
    assert not np.allclose(Pprint.sum(1), a, rtol=0.5)
    K = orc.gibbs(C, eps)
    u, v = orc.sinkhorn_dense(K, a, b, 500)
    P = u[:, None] * K * v[None, :]
    assert np.allclose(P.sum(1), a, rtol=1e-9) and np.allclose(P.sum(0), b, rtol=1e-12)
    assert set(map(tuple, np.argwhere(Pprint > 0.05))) <= set(map(tuple, np.argwhere(P > 0.01)))
    assert P[2, 2] == pytest.approx(Pprint[2, 2], rel=2e-2)


# ------------------------------------- bounded-delay emulation (Algorithm 3) ---

def test_async_emulation_with_one_client_is_the_damped_iteration(orc):
    """c = 1: there are no remote slices, so any delay gives the centralised relaxed iteration
    of Sec. 3.3."""
    x, y, a, b, C, K = problem(30, 30, eps=0.2)
    for eta in (1.0, 0.5):
        ud, vd = orc.sinkhorn_dense_damped(K, a, b, 12, eta, False)
        for tau, w in ((0, 1), (3, 1), (2, 4)):
            ua, va = orc.sinkhorn_async_emulated(K, a, b, 12, 1, eta, tau, w)
            assert np.allclose(ua, ud, rtol=1e-13) and np.allclose(va, vd, rtol=1e-13)


def test_async_emulation_first_iterations_by_hand(orc):
    """Two iterations of Algorithm 3 written out with NumPy for c = 2, tau = 1, eta = 0.7:
    remote slices are still the initial ones in both iterations, own slices are current."""
    n, m, eta = 8, 4, 0.7
    x, y, a, b, C, K = problem(n, 31, eps=0.3)
    u0 = np.ones(n); v0 = np.ones(n)
    hist = [(u0, v0)]
    for t in (1, 2):
        pu, pv = hist[-1]
        su, sv = hist[0]                      # s(t) = 0 for t <= tau + 1
        nu, nv = pu.copy(), pv.copy()
        for j in range(2):
            I = slice(j * m, (j + 1) * m)
            view = sv.copy(); view[I] = pv[I]
            nu[I] = (1 - eta) * pu[I] + eta * a[I] / (K[I, :] @ view)
            view = su.copy(); view[I] = nu[I]
            nv[I] = (1 - eta) * pv[I] + eta * b[I] / (K[:, I].T @ view)
        hist.append((nu, nv))
    ua, va = orc.sinkhorn_async_emulated(K, a, b, 2, 2, eta, 1, 1)
    assert np.allclose(ua, hist[-1][0], rtol=1e-13) and np.allclose(va, hist[-1][1], rtol=1e-13)
    # third iteration sees the peers' slices from the end of iteration 1
    pu, pv = hist[2]; su, sv = hist[1]
    nu, nv = pu.copy(), pv.copy()
    for j in range(2):
        I = slice(j * m, (j + 1) * m)
        view = sv.copy(); view[I] = pv[I]
        nu[I] = (1 - eta) * pu[I] + eta * a[I] / (K[I, :] @ view)
        view = su.copy(); view[I] = nu[I]
        nv[I] = (1 - eta) * pv[I] + eta * b[I] / (K[:, I].T @ view)
    ua, va = orc.sinkhorn_async_emulated(K, a, b, 3, 2, eta, 1, 1)
    assert np.allclose(ua, nu, rtol=1e-13) and np.allclose(va, nv, rtol=1e-13)


@pytest.mark.parametrize("c,tau,w,eta", [(4, 2, 1, 1.0), (4, 3, 2, 0.5), (8, 1, 3, 1.0)])
def test_async_emulation_converges_to_the_sinkhorn_plan(orc, c, tau, w, eta):
    """Proposition 2: under bounded delay the scalings converge to a Sinkhorn fixed point
    (unique up to the scalar gauge), i.e. to the same plan P*."""
    x, y, a, b, C, K = problem(32, 32, eps=0.25)
    us, vs = orc.sinkhorn_dense(K, a, b, 4000)
    Pstar = us[:, None] * K * vs[None, :]
    ua, va = orc.sinkhorn_async_emulated(K, a, b, 3000, c, eta, tau, w)
    assert np.allclose(ua[:, None] * K * va[None, :], Pstar, rtol=1e-7)
    r = ua / us
    assert np.allclose(r, r[0], rtol=1e-7)


# ----------------- synchronous local steps w (Sec. 3.1 Remark; App. "local steps") ---

def test_local_steps_w1_is_algorithm_1_and_one_client_is_centralised(orc):
    """The appendix on local steps: w = 1 is fully synchronous Sinkhorn -- the very values of
    the row-partitioned iteration as printed in Algorithm 1; and with one client there is no
    peer whose slice could be stale, so any w gives the centralised iteration."""
    x, y, a, b, C, K = problem(24, 60, eps=0.2)
    for c in (1, 2, 4, 8):
        ub, vb = orc.sinkhorn_blocked(K, a, b, 9, c, 0)
        ul, vl = orc.sinkhorn_local_steps(K, a, b, 9, c, 1)
        assert np.array_equal(ul, ub) and np.array_equal(vl, vb)
    ud, vd = orc.sinkhorn_dense(K, a, b, 9)
    for w in (2, 3, 9, 50):
        ul, vl = orc.sinkhorn_local_steps(K, a, b, 9, 1, w)
        assert np.array_equal(ul, ud) and np.array_equal(vl, vd)
    with pytest.raises(ValueError):
        orc.sinkhorn_local_steps(K, a, b, 1, 5, 1)      # 5 does not divide 24
    with pytest.raises(ValueError):
        orc.sinkhorn_local_steps(K, a, b, 1, 2, 0)


def test_local_steps_first_rounds_by_hand(orc):
    """c = 2 clients, w = 2, written out with NumPy on per-client views: iteration 1 is local
    (each client sees the peer's initial slices), iteration 2 gathers u before the v-update and v
    after it, iteration 3 is local again on the gathered views, iteration 4 gathers.  The
    asymmetric K tells the row slab from the column slab."""
    n, m = 10, 5
    x, y, a, b, C, K = problem(n, 61, eps=0.3)
    I = [slice(0, m), slice(m, n)]
    uview = [np.ones(n), np.ones(n)]; vview = [np.ones(n), np.ones(n)]
    states = []
    for k in (1, 2, 3, 4):
        for j in (0, 1):
            uview[j][I[j]] = a[I[j]] / (K[I[j], :] @ vview[j])
        if k % 2 == 0:
            uview[0][I[1]] = uview[1][I[1]]; uview[1][I[0]] = uview[0][I[0]]
        for j in (0, 1):
            vview[j][I[j]] = b[I[j]] / (K[:, I[j]].T @ uview[j])
        if k % 2 == 0:
            vview[0][I[1]] = vview[1][I[1]]; vview[1][I[0]] = vview[0][I[0]]
        states.append((np.concatenate([uview[0][I[0]], uview[1][I[1]]]),
                       np.concatenate([vview[0][I[0]], vview[1][I[1]]])))
    for k in (1, 2, 3, 4):
        ul, vl = orc.sinkhorn_local_steps(K, a, b, k, 2, 2)
        assert np.allclose(ul, states[k - 1][0], rtol=1e-13) and np.allclose(vl, states[k - 1][1], rtol=1e-13)
    # the local iterations really differ from Algorithm 1 (stale peers), the schedule matters
    u1, v1 = orc.sinkhorn_dense(K, a, b, 4)
    assert not np.allclose(states[3][0], u1, rtol=1e-3)
    # a run is resumable at a collective: 4 iterations == 2 + 2 with the state passed through
    ua, va = orc.sinkhorn_local_steps(K, a, b, 2, 2, 2)
    ub, vb = orc.sinkhorn_local_steps(K, a, b, 2, 2, 2, ua, va)
    u4, v4 = orc.sinkhorn_local_steps(K, a, b, 4, 2, 2)
    assert np.array_equal(ub, u4) and np.array_equal(vb, v4)


def test_local_steps_before_the_first_collective_equal_the_delay_emulation(orc):
    """Until the first collective a client has its own slices current and the peers' initial
    ones: exactly what the bounded-delay schedule (undamped, no exchange yet) prescribes.  The
    two functions are written separately; the emulation is pinned by its own hand-written case."""
    x, y, a, b, C, K = problem(24, 62, eps=0.25)
    for c in (2, 3, 4):
        ul, vl = orc.sinkhorn_local_steps(K, a, b, 5, c, 6)
        ue, ve = orc.sinkhorn_async_emulated(K, a, b, 5, c, 1.0, 0, 6)
        assert np.allclose(ul, ue, rtol=1e-14) and np.allclose(vl, ve, rtol=1e-14)
    # at the collective iteration they part: here the v-update sees every peer's fresh u
    ul, vl = orc.sinkhorn_local_steps(K, a, b, 6, 3, 6)
    ue, ve = orc.sinkhorn_async_emulated(K, a, b, 6, 3, 1.0, 0, 6)
    assert np.allclose(ul, ue, rtol=1e-14) and not np.allclose(vl, ve, rtol=1e-6)
    # ... exactly as one more step of Algorithm 1's v-update on the gathered u would
    assert np.allclose(vl, b / (K.T @ ul), rtol=1e-13)


@pytest.mark.parametrize("c,w", [(2, 2), (4, 3), (8, 5)])
def test_local_steps_converge_to_the_sinkhorn_plan(orc, c, w):
    """The appendix reports that w > 1 slows the iteration but still reaches the tolerance: the
    limit is a Sinkhorn fixed point, i.e. the same plan P* (scalings up to the scalar gauge)."""
    x, y, a, b, C, K = problem(32, 63, eps=0.25)
    us, vs = orc.sinkhorn_dense(K, a, b, 4000)
    Pstar = us[:, None] * K * vs[None, :]
    ul, vl = orc.sinkhorn_local_steps(K, a, b, 6000, c, w)
    assert np.allclose(ul[:, None] * K * vl[None, :], Pstar, rtol=1e-7)
    r = ul / us
    assert np.allclose(r, r[0], rtol=1e-7)


# ------------------------------------------------------------ plan objective ---

def test_plan_objective_against_numpy_and_duality(orc):
    """Eq. 1 evaluated at P = diag(u) K diag(v): against NumPy on the explicit plan, and at
    convergence against the dual value (an independent formula)."""
    x, y, a, b, C, K = problem(14, 40, eps=0.15)
    eps = 0.15
    rng = np.random.default_rng(4)
    l = rng.normal(size=14)
    u, v = orc.sinkhorn_dense(K, a, b, 7)
    P = u[:, None] * K * v[None, :]
    out = orc.plan_objective(K, C, eps, u, v, l)
    assert out[0] == pytest.approx((P * C).sum(), rel=1e-13)
    assert out[1] == pytest.approx((P * (np.log(P) - 1)).sum(), rel=1e-13)
    assert out[2] == pytest.approx(primal_objective(P, C, eps), rel=1e-13)
    assert out[3] == pytest.approx(P.sum(), rel=1e-13)
    assert out[4] == pytest.approx((P * l[None, :]).sum(), rel=1e-12)
    u, v = orc.sinkhorn_dense(K, a, b, 5000)
    out = orc.plan_objective(K, C, eps, u, v)
    assert out[2] == pytest.approx(dual_objective(eps * np.log(u), eps * np.log(v), a, b, C, eps), abs=1e-12)
    assert out[4] == 0.0


# ------------------------------- radius search of the robust-risk example ---

def _two_by_two_root():
    """n = 2: with both marginals fixed the plan has one free entry p.  A scaling of K has
    P11 P22 / (P12 P21) = K11 K22 / (K12 K21) = exp(-lambda (c11 + c22 - c12 - c21)/eps) (the
    column term l_j cancels), so the lambda that yields a chosen p is known in closed form."""
    a = np.array([0.35, 0.65]); b = np.array([0.55, 0.45])
    c = np.array([[0.1, 0.9], [0.7, 0.2]])
    eps = 0.05
    p = 0.30                                        # P11; then P12 = a1 - p, P21 = b1 - p, P22 = a2 - b1 + p
    P = np.array([[p, a[0] - p], [b[0] - p, a[1] - b[0] + p]])
    assert (P > 0).all()
    ratio = P[0, 0] * P[1, 1] / (P[0, 1] * P[1, 0])
    lam = -eps * np.log(ratio) / (c[0, 0] + c[1, 1] - c[0, 1] - c[1, 0])
    return a, b, c, eps, P, lam, float((P * c).sum())


def test_radius_search_two_by_two_closed_form(orc):
    a, b, c, eps, P, lam_star, delta = _two_by_two_root()
    l = np.array([0.02, -0.03])
    lam, cost, loss, steps, u, v, K = orc.radius_search(c, l, a, b, eps, delta, 0.0, 1.0, 60, 0.0, 3000)
    assert 0.0 < lam_star < 1.0 and 40 <= steps <= 60
    assert lam == pytest.approx(lam_star, abs=1e-10)
    assert np.allclose(u[:, None] * K * v[None, :], P, rtol=1e-8)
    assert cost == pytest.approx(delta, rel=1e-9) and loss == pytest.approx(float(b @ l), rel=1e-12)
    # a tolerance on g stops the search early, at a lambda whose cost is within it
    lam2, cost2, _, steps2, _, _, _ = orc.radius_search(c, l, a, b, eps, delta, 0.0, 1.0, 60, 1e-4, 3000)
    assert steps2 < 20 and abs(cost2 - delta) <= 1e-4


def test_gibbs_lambda_and_the_role_of_l(orc):
    """lambda = 0 leaves K_ij = exp(l_j/eps), whose scaling is the independent coupling a b^T,
    so <P, c> = a^T c b.  For any lambda, l only rescales the columns of K: the converged plan is
    the same as with l = 0, and sum_ij P_ij l_j = b^T l after any v-update."""
    x, y, a, b, C, _ = problem(9, 77, eps=0.2)
    eps = 0.2
    rng = np.random.default_rng(5)
    l = rng.uniform(-0.3, 0.3, 9)
    assert np.allclose(orc.gibbs_lambda(C, 0.7, l, eps), np.exp(-(0.7 * C - l[None, :]) / eps), rtol=1e-14)
    assert np.allclose(orc.gibbs_lambda(C, 0.7, None, eps), np.exp(-0.7 * C / eps), rtol=1e-14)   # no l: l = 0
    K32 = orc.gibbs_lambda(C, 0.7, l, eps, True)
    assert np.array_equal(K32, K32.astype(np.float32).astype(np.float64))
    lam, cost, loss, steps, u, v, K = orc.radius_search(C, l, a, b, eps, 0.0, 0.0, 0.0, 1, 0.0, 5)
    assert lam == 0.0 and steps == 1
    assert cost == pytest.approx(float(a @ C @ b), rel=1e-12)
    assert np.allclose(u[:, None] * K * v[None, :], np.outer(a, b), rtol=1e-12)
    r1 = orc.radius_search(C, l, a, b, eps, 0.0, 0.8, 0.8, 1, 0.0, 3000)
    r0 = orc.radius_search(C, None, a, b, eps, 0.0, 0.8, 0.8, 1, 0.0, 3000)
    P1 = r1[4][:, None] * r1[6] * r1[5][None, :]
    P0 = r0[4][:, None] * r0[6] * r0[5][None, :]
    assert np.allclose(P1, P0, rtol=1e-10)
    assert r1[1] == pytest.approx(r0[1], rel=1e-10)
    assert r1[2] == pytest.approx(float(b @ l), rel=1e-12) and r0[2] == 0.0


def test_radius_search_against_scipy_root_of_the_log_domain_cost(orc):
    """The transport cost of the optimal plan falls as lambda grows; the root that SciPy finds
    for g(lambda) evaluated through the log-domain iteration on C_lambda (NumPy builds the cost)
    is the one the bisection returns."""
    x, y, a, b, C, _ = problem(12, 91, eps=0.1)
    eps = 0.1
    l = np.random.default_rng(6).uniform(-0.2, 0.2, 12)

    def cost_at(lam):
        Cl = lam * C - l[None, :]
        f, g = orc.sinkhorn_log_cost(Cl, eps, a, b, 400)[:2]
        P = np.exp((f[:, None] + g[None, :] - Cl) / eps)
        return float((P * C).sum())

    costs = [cost_at(t) for t in (0.0, 0.5, 1.0, 2.0, 4.0)]
    assert all(c1 > c2 for c1, c2 in zip(costs, costs[1:]))
    assert costs[0] == pytest.approx(float(a @ C @ b), rel=1e-10)
    delta = 0.5 * (costs[1] + costs[3])
    root = scipy.optimize.brentq(lambda t: cost_at(t) - delta, 0.0, 4.0, xtol=1e-12)
    lam, cost, loss, steps, u, v, K = orc.radius_search(C, l, a, b, eps, delta, 0.0, 4.0, 45, 0.0, 400)
    assert lam == pytest.approx(root, abs=1e-9) and cost == pytest.approx(delta, rel=1e-9)
    # every solve is Algorithm 1 from u = v = 1 on the kernel of its lambda: the scalings handed back
    # are those of the plain iteration on the K handed back (the gauge, not only the plan)
    lam, cost, loss, steps, u, v, K = orc.radius_search(C, l, a, b, eps, delta, 0.0, 4.0, 6, 0.0, 25)
    assert steps == 6 and np.array_equal(K, orc.gibbs_lambda(C, lam, l, eps))
    up, vp = orc.sinkhorn_dense(K, a, b, 25)
    assert np.array_equal(u, up) and np.array_equal(v, vp)


# ---------------------------------------- 2D block grid (HPC baseline appendix) ---

def test_grid_iteration_is_the_centralised_one(orc):
    """Block products reduced along block rows / block columns only regroup the sums: every grid
    gives the centralised iterates to rounding; with one block column the grouping is exactly
    that of the row-slab flow; the first iteration matches NumPy block matmuls."""
    x, y, a, b, C, K = problem(48, 48, eps=0.2)
    uc, vc = orc.sinkhorn_dense(K, a, b, 30)
    for p_r, p_c in ((1, 1), (2, 3), (4, 4), (6, 2), (48, 1), (1, 48), (8, 16)):
        u, v = orc.sinkhorn_grid(K, a, b, 30, p_r, p_c)
        assert np.allclose(u, uc, rtol=1e-13) and np.allclose(v, vc, rtol=1e-13)
    u1, v1 = orc.sinkhorn_grid(K, a, b, 30, 1, 1)
    assert np.array_equal(u1, uc) and np.array_equal(v1, vc)
    for c in (2, 4, 8):
        ub, vb = orc.sinkhorn_blocked(K, a, b, 30, c, 1)
        ug, vg = orc.sinkhorn_grid(K, a, b, 30, c, 1)
        assert np.array_equal(ub, ug) and np.array_equal(vb, vg)
    p_r, p_c = 4, 3
    rows = np.split(np.arange(48), p_r); cols = np.split(np.arange(48), p_c)
    v0 = np.ones(48)
    q = np.concatenate([sum(K[np.ix_(R, J)] @ v0[J] for J in cols) for R in rows])
    u_np = a / q
    r = np.concatenate([sum(K[np.ix_(R, J)].T @ u_np[R] for R in rows) for J in cols])
    v_np = b / r
    u, v = orc.sinkhorn_grid(K, a, b, 1, p_r, p_c)
    assert np.allclose(u, u_np, rtol=1e-14) and np.allclose(v, v_np, rtol=1e-14)
    with pytest.raises(ValueError):
        orc.sinkhorn_grid(K, a, b, 1, 5, 2)
    with pytest.raises(ValueError):
        orc.sinkhorn_grid(K, a, b, 1, 2, 7)


# ------------------------------------------------ privacy layer (DP appendix) ---

def test_philox_known_answers(orc):
    with open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) as fh:
        rows = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(t, 16) for t in r]
        assert list(orc.philox4x32_10(w[0:4], w[4:6])) == w[6:10]


def test_dp_normals_are_standard_normal_and_counter_based(orc):
    import scipy.stats
    z = orc.dp_normals(11, 4, 0, 200000)
    assert scipy.stats.kstest(z, "norm").pvalue > 1e-3
    r2 = z[0::2] ** 2 + z[1::2] ** 2                      # a Box-Muller pair: chi-square, 2 dof
    assert scipy.stats.kstest(r2, "chi2", args=(2,)).pvalue > 1e-3
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 0.01
    other = orc.dp_normals(11, 5, 0, 200000)              # another release, another seed: unrelated streams
    assert abs(np.corrcoef(z, other)[0, 1]) < 0.01
    assert abs(np.corrcoef(z, orc.dp_normals(12, 4, 0, 200000))[0, 1]) < 0.01
    # counter-based: any sub-range can be drawn on its own, in any order
    assert np.array_equal(orc.dp_normals(11, 4, 777, 100), z[777:877])
    assert np.array_equal(orc.dp_normals(11, 4, 2 ** 34 + 3, 5), orc.dp_normals(11, 4, 2 ** 34, 8)[3:])
    # the map from element to generator call, written out: elements 4q .. 4q+3 come from call q with
    # counter (q, release) and key seed; Box-Muller on (x0, x1) and on (x2, x3), uniforms (x + 1/2) 2^-32
    seed, release = (5 << 32) + 11, (3 << 32) + 4
    z = orc.dp_normals(seed, release, 0, 12)
    for q in range(3):
        w = orc.philox4x32_10([q, 0, release & 0xFFFFFFFF, release >> 32], [seed & 0xFFFFFFFF, seed >> 32])
        for pair in range(2):
            u1 = (float(w[2 * pair]) + 0.5) / 2.0 ** 32; u2 = (float(w[2 * pair + 1]) + 0.5) / 2.0 ** 32
            r = np.sqrt(-2.0 * np.log(u1))
            assert z[4 * q + 2 * pair] == pytest.approx(r * np.cos(2 * np.pi * u2), rel=1e-13, abs=1e-14)
            assert z[4 * q + 2 * pair + 1] == pytest.approx(r * np.sin(2 * np.pi * u2), rel=1e-13, abs=1e-14)


def test_dp_release_clip_and_noise(orc):
    rng = np.random.default_rng(8)
    X = np.exp(rng.normal(scale=3.0, size=(50, 6)))
    L = np.log(X)
    # no clip, no noise: identity up to exp(log(.))
    assert np.allclose(orc.dp_release(X, np.inf, 0.0, 1, 0), X, rtol=1e-14)
    assert np.allclose(orc.dp_release(X, 0.0, 0.0, 1, 0), X, rtol=1e-14)
    # clip only: rows keep their direction, norms become min(norm, S)
    S = 5.0
    Lc = np.log(orc.dp_release(X, S, 0.0, 1, 0))
    norms = np.linalg.norm(L, axis=1)
    assert (norms > S).any() and (norms < S).any()
    assert np.allclose(np.linalg.norm(Lc, axis=1), np.minimum(norms, S), rtol=1e-12)
    assert np.allclose(Lc * norms[:, None], L * np.linalg.norm(Lc, axis=1)[:, None], rtol=1e-10, atol=1e-12)
    # l2 sensitivity of the clipped release is at most 2 S, whatever the inputs
    Y = np.exp(rng.normal(scale=30.0, size=(50, 6)))
    assert (np.linalg.norm(Lc - np.log(orc.dp_release(Y, S, 0.0, 1, 0)), axis=1) <= 2 * S + 1e-9).all()
    # one target: the row clip is a clamp of the log-scaling to [-S, S]
    x1 = np.exp(rng.normal(scale=3.0, size=40))
    assert np.allclose(np.log(orc.dp_release(x1, 2.0, 0.0, 1, 0))[:, 0], np.clip(np.log(x1), -2.0, 2.0), rtol=1e-12)
    assert np.allclose(np.log(orc.dp_release(x1, 0.25, 0.0, 1, 0))[:, 0], np.clip(np.log(x1), -0.25, 0.25), rtol=1e-12)
    # noise only: the log-scalings move by sigma times the release's normal numbers, element i*m + k
    sigma = 0.3
    Ln = np.log(orc.dp_release(X, np.inf, sigma, 21, 9))
    assert np.allclose(Ln - L, sigma * orc.dp_normals(21, 9, 0, X.size).reshape(X.shape), rtol=0, atol=1e-12)
    # both: clip first, then add
    Lb = np.log(orc.dp_release(X, S, sigma, 21, 9))
    assert np.allclose(Lb - Lc, sigma * orc.dp_normals(21, 9, 0, X.size).reshape(X.shape), rtol=0, atol=1e-12)


def test_batched_dp_iteration(orc):
    x, y, a, b, C, K = problem(24, 61, eps=0.3)
    rng = np.random.default_rng(9)
    A = rng.uniform(0.5, 1.5, (24, 3)); A /= A.sum(0)
    B = rng.uniform(0.5, 1.5, (24, 3)); B /= B.sum(0)
    U0, V0 = orc.sinkhorn_batched(K, A, B, 7)
    U1, V1 = orc.sinkhorn_batched_dp(K, A, B, 7, np.inf, np.inf, 0.0, 0.0, 5)
    assert np.allclose(U1, U0, rtol=1e-12) and np.allclose(V1, V0, rtol=1e-12)
    # two iterations by hand: NumPy products, the oracle's release
    S_u, S_v, s_u, s_v, seed = 4.0, 3.0, 0.05, 0.02, 77
    U = np.ones((24, 3)); V = np.ones((24, 3))
    for t in range(2):
        U = orc.dp_release(A / (K @ V), S_u, s_u, seed, 10 + 2 * t)
        V = orc.dp_release(B / (K.T @ U), S_v, s_v, seed, 10 + 2 * t + 1)
    Ud, Vd = orc.sinkhorn_batched_dp(K, A, B, 2, S_u, S_v, s_u, s_v, seed, release0=10)
    assert np.allclose(Ud, U, rtol=1e-12) and np.allclose(Vd, V, rtol=1e-12)
    # resume: 2 + 3 iterations with the release counter carried on equal 5
    U5, V5 = orc.sinkhorn_batched_dp(K, A, B, 5, S_u, S_v, s_u, s_v, seed, release0=10)
    Ur, Vr = orc.sinkhorn_batched_dp(K, A, B, 3, S_u, S_v, s_u, s_v, seed, release0=14, U0=Ud, V0=Vd)
    assert np.array_equal(Ur, U5) and np.array_equal(Vr, V5)


def test_rdp_accountant_closed_form(orc):
    """With c = T (2S)^2 / (2 sigma^2) the bound c p + log(1/delta)/(p - 1) is minimised at
    p* = 1 + sqrt(log(1/delta)/c) with value c + 2 sqrt(c log(1/delta))."""
    S, sigma, T, delta = 4.0, 50.0, 2000, 1e-5
    c = T * (2 * S) ** 2 / (2 * sigma ** 2)
    p_star = 1 + np.sqrt(np.log(1 / delta) / c)
    best = c + 2 * np.sqrt(c * np.log(1 / delta))
    eps, p = orc.rdp_epsilon(S, sigma, T, delta, [1.5, p_star, 8.0, 64.0])
    assert p == p_star and eps == pytest.approx(best, rel=1e-13)
    grid = np.concatenate([1 + np.arange(1, 100) / 10.0, np.arange(12, 64)])
    eps_g, p_g = orc.rdp_epsilon(S, sigma, T, delta, grid)
    assert best <= eps_g <= 1.01 * best and abs(p_g - p_star) <= 0.1
    assert orc.rdp_epsilon(S, sigma, T, delta, [0.5, 0.9, 1.0, 2.0])[1] == 2.0  # orders <= 1 are not RDP orders
    # additive composition: twice the releases, twice the Renyi term
    e1 = orc.rdp_epsilon(S, sigma, T, delta, [3.0])[0] - np.log(1 / delta) / 2
    e2 = orc.rdp_epsilon(S, sigma, 2 * T, delta, [3.0])[0] - np.log(1 / delta) / 2
    assert e2 == pytest.approx(2 * e1, rel=1e-13)
