"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

Two kinds of cases.  The `*_full_*` tests follow a configuration for its own length: the oracle
runs all 1000 (configuration 3) or 300 (configuration 5) iterations, or the configuration-4 law
to its stop rule, in chunks that print a progress line, and the GPU's state is compared element
by element at every chunk boundary -- direct relative error, both marginals, and the error with
the uniform-rescaling direction taken out (see gpu_util.gauge_free).  The older cases combine a
short run from the cold start with one-step consistency at a late state: the oracle recomputes
sampled entries of the next update from the GPU's own previous half-step.
"""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev, gauge_free, relerr, say

pytestmark = pytest.mark.gpu


def test_cfg3_n32768_c8_equals_c1_and_oracle(orc):
    w = workloads.make(3)
    n = w.n
    K, _ = orc.gibbs_from_points_f32(w.x, w.y, w.eps, True)
    Kd = dev(K); a = dev(w.a); b = dev(w.b)

    def run(c, iters, u=None, v=None, flow=api.FSK_FLOW_FUSED):
        opts = api.make_opts(n, torch.float32, c=c, max_iters=iters, flow=flow)
        ws = api.alloc_workspace(opts)
        u = torch.ones(n, device="cuda") if u is None else u.clone()
        v = torch.ones(n, device="cuda") if v is None else v.clone()
        api.fsk_sinkhorn_dense(opts, Kd, a, b, u, v, ws)
        torch.cuda.synchronize()
        return u, v

    # (i) 20 iterations against the oracle, blocked and centralised
    uo, vo = orc.sinkhorn_blocked(K, w.a, w.b, 20, 8, 1)
    for c in (8, 1):
        u, v = run(c, 20)
        assert relerr(u.cpu().numpy(), uo) <= 1e-4 and relerr(v.cpu().numpy(), vo) <= 1e-4

    # the full 1000 iterations: every c reproduces c = 1 bit for bit in the fused flow (Proposition
    # 1): the strips a block is cut into are the same 128 rows whatever c is
    u1, v1 = run(1, 1000)
    for c in (2, 4, 8, 64, 256):
        uc, vc = run(c, 1000)
        assert torch.equal(uc, u1) and torch.equal(vc, v1), c
    u8, v8 = run(8, 999)
    # the two-pass flow is bitwise independent of c at full size as well (one iteration suffices)
    ut1, vt1 = run(1, 1, u8, v8, flow=api.FSK_FLOW_TWO_PASS)
    ut8, vt8 = run(8, 1, u8, v8, flow=api.FSK_FLOW_PAPER)
    assert torch.equal(ut1, ut8) and torch.equal(vt1, vt8)

    # (ii) iteration 1000 from the GPU's state after 999, sampled rows and columns
    u9, v9 = run(8, 1, u8, v8)
    rng = np.random.default_rng(3)
    rows = np.sort(rng.choice(n, 512, replace=False))
    cols = np.sort(rng.choice(n, 512, replace=False))
    v8h = v8.cpu().numpy(); u9h = u9.cpu().numpy(); v9h = v9.cpu().numpy()
    q = np.array([orc.row_products(K, v8h, i, i + 1)[0] for i in rows])
    assert relerr(u9h[rows], w.a[rows].astype(np.float64) / q) <= 1e-4
    r = np.array([orc.col_products(K, u9h, 0, n, j, j + 1)[0] for j in cols])
    assert relerr(v9h[cols], w.b[cols].astype(np.float64) / r) <= 1e-4
    # column marginal exact after the v-update, row marginal converged
    assert relerr(v9h[cols] * r, w.b[cols]) <= 1e-4
    qn = np.array([orc.row_products(K, v9h, i, i + 1)[0] for i in rows])
    assert np.max(np.abs(u9h[rows] * qn - w.a[rows]) / w.a[rows]) <= 1e-3


def test_cfg4_n65536_log_domain(orc):
    w = workloads.make(4)
    n, d, eps = w.n, w.d, w.eps
    x, y, a, b = dev(w.x), dev(w.y), dev(w.a), dev(w.b)

    def run(iters, f=None, g=None, tol=0.0, check_every=1):
        opts = api.make_opts(n, torch.float32, max_iters=iters, tol=tol, check_every=check_every)
        ws = api.alloc_workspace(opts, api.FSK_MODE_LOG, d)
        f = torch.zeros(n, device="cuda") if f is None else f.clone()
        g = torch.zeros(n, device="cuda") if g is None else g.clone()
        done, err = api.fsk_sinkhorn_log_points(opts, x, y, eps, a, b, f, g, ws)
        torch.cuda.synchronize()
        return f, g, done, err

    # (i) two full oracle iterations from the cold start
    fo, go, _, _ = orc.sinkhorn_log_points(w.x, w.y, eps, w.a, w.b, 2)
    f, g, _, _ = run(2)
    assert np.max(np.abs(f.cpu().numpy() - fo)) / eps <= 1e-4
    assert np.max(np.abs(g.cpu().numpy() - go)) / eps <= 1e-4

    # (ii) one-step consistency at t = 100 on sampled rows / columns
    f99, g99, _, _ = run(99)
    f100, g100, _, _ = run(1, f99, g99)
    rng = np.random.default_rng(4)
    rows = np.sort(rng.choice(n, 256, replace=False))
    g99h = g99.cpu().numpy().astype(np.float64); f100h = f100.cpu().numpy().astype(np.float64)
    g100h = g100.cpu().numpy().astype(np.float64)
    f_ref = orc.log_update_points(w.x, w.a, w.y, g99h, eps, rows)
    assert np.max(np.abs(f100h[rows] - f_ref)) / eps <= 1e-4
    g_ref = orc.log_update_points(w.y, w.b, w.x, f100h, eps, rows)
    assert np.max(np.abs(g100h[rows] - g_ref)) / eps <= 1e-4

    # a tolerance this law reaches: the run stops at a poll before the cap, the reported error is
    # below it, and the oracle's evaluation of the handed-back state on sampled rows agrees
    ft, gt, done_t, err_t = run(2000, tol=2e-3, check_every=10)
    assert 0 < done_t < 2000 and done_t % 10 == 0 and err_t < 2e-3
    rm = orc.log_row_marginal_points(w.x, ft.cpu().numpy().astype(np.float64), w.y,
                                     gt.cpu().numpy().astype(np.float64), eps, rows)
    est = np.abs(rm - w.a[rows]).sum() * (n / rows.size)
    assert 0.5 * err_t <= est <= 2.0 * err_t
    # ... and ten iterations earlier (the previous poll) the error was still above it
    fp_, gp_, _, _ = run(done_t - 10)
    rm = orc.log_row_marginal_points(w.x, fp_.cpu().numpy().astype(np.float64), w.y,
                                     gp_.cpu().numpy().astype(np.float64), eps, rows)
    assert np.abs(rm - w.a[rows]).sum() * (n / rows.size) > 0.6 * 2e-3

    # the stop rule of the configuration: L1 row-marginal error < 1e-6 or 2000 iterations
    f, g, done, err = run(2000, f100, g100, tol=1e-6, check_every=50)
    assert done % 50 == 0 and np.isfinite(err)
    assert (err < 1e-6) or done == 2000
    fh = f.cpu().numpy().astype(np.float64); gh = g.cpu().numpy().astype(np.float64)
    rm = orc.log_row_marginal_points(w.x, fh, w.y, gh, eps, rows)
    est = np.abs(rm - w.a[rows]).sum() * (n / rows.size)      # sampled estimate of the L1 error
    assert est <= max(5 * err, 5e-6)
    cm = orc.log_row_marginal_points(w.y, gh, w.x, fh, eps, rows)
    assert np.max(np.abs(cm - w.b[rows]) / w.b[rows]) <= 1e-4

    # the cap binds because of the law's convergence rate, not because of fp32 potentials: the
    # all-fp64 interface follows the same error curve to the same cap
    def run64(iters, tol, every):
        opts = api.make_opts(n, torch.float64, max_iters=iters, tol=tol, check_every=every)
        ws = api.alloc_workspace(opts, api.FSK_MODE_LOG, d)
        f = torch.zeros(n, dtype=torch.float64, device="cuda"); g = torch.zeros_like(f)
        done, err = api.fsk_sinkhorn_log_points(opts, dev(w.x.astype(np.float64)), dev(w.y.astype(np.float64)),
                                                eps, dev(w.a.astype(np.float64)), dev(w.b.astype(np.float64)),
                                                f, g, ws)
        return done, err
    _, _, done32, err32 = run(2000, tol=1e-6, check_every=500)
    done64, err64 = run64(2000, 1e-6, 500)
    assert done32 == done64 == 2000 and err64 > 1e-6
    assert err32 == pytest.approx(err64, rel=1e-2)


def test_cfg5_n16384_m64_batched(orc):
    w = workloads.make(5)
    n, m = w.n, w.m
    K, _ = orc.gibbs_from_points_f32(w.x, w.y, w.eps, False)
    Kd = dev(K); A = dev(w.a); B = dev(w.b)

    def run(iters, U=None, V=None):
        opts = api.make_opts(n, torch.float32, m=m, max_iters=iters)
        ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
        U = torch.ones(n, m, device="cuda") if U is None else U.clone()
        V = torch.ones(n, m, device="cuda") if V is None else V.clone()
        api.fsk_sinkhorn_batched(opts, Kd, A, B, U, V, ws)
        torch.cuda.synchronize()
        return U, V

    Uo, Vo = orc.sinkhorn_batched(K, w.a, w.b, 2)
    U, V = run(2)
    assert relerr(U.cpu().numpy(), Uo) <= 1e-4 and relerr(V.cpu().numpy(), Vo) <= 1e-4

    U299, V299 = run(299)
    U300, V300 = run(1, U299, V299)
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(n, 128, replace=False))
    V299h = V299.cpu().numpy(); U300h = U300.cpu().numpy(); V300h = V300.cpu().numpy()
    for k in (0, 17, 63):
        q = np.array([orc.row_products(K, V299h[:, k], i, i + 1)[0] for i in rows])
        assert relerr(U300h[rows, k], w.a[rows, k].astype(np.float64) / q) <= 1e-4
        r = np.array([orc.col_products(K, U300h[:, k], 0, n, j, j + 1)[0] for j in rows])
        assert relerr(V300h[rows, k], w.b[rows, k].astype(np.float64) / r) <= 1e-4


def test_multitarget_instance_n5000_m500(orc):
    """The multitarget experiment's own shape (Sec. 5.3.2: n = 5000, N = 500 targets, 15
    iterations; the paper runs it in fp64), all column groups in one launch, whole trajectory
    against the oracle.  Both precisions get the same fp32-representable K, A, B, so one oracle
    run serves both."""
    n, m, iters = 5000, 500, 15
    w = workloads.make(5, n=n, m=m, seed=5500)
    K, _ = orc.gibbs_from_points_f32(w.x, w.y, w.eps, False)
    A = np.ascontiguousarray(w.a.astype(np.float32)); B = np.ascontiguousarray(w.b.astype(np.float32))
    Uo, Vo = orc.sinkhorn_batched(K, A, B, iters)
    for td, nd, tol in ((torch.float32, np.float32, 1e-4), (torch.float64, np.float64, 1e-10)):
        opts = api.make_opts(n, td, m=m, max_iters=iters)
        ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
        U = torch.ones(n, m, dtype=td, device="cuda"); V = torch.ones(n, m, dtype=td, device="cuda")
        Kd = torch.empty(n, n + 8, dtype=td, device="cuda")[:, :n]
        Kd.copy_(dev(K))
        api.fsk_sinkhorn_batched(opts, Kd, dev(A.astype(nd)), dev(B.astype(nd)), U, V, ws)
        torch.cuda.synchronize()
        assert relerr(U.cpu().numpy(), Uo) <= tol and relerr(V.cpu().numpy(), Vo) <= tol


def test_cfg3_full_1000_iterations_against_oracle(orc, capsys):
    """Configuration 3 for its own length: 1000 iterations, c = 8, fused flow, against the
    oracle's row-slab iteration (contributions added in block order) on u, v and both marginals;
    compared every 100 iterations so that a drift shows where it starts."""
    w = workloads.make(3)
    n, T, step = w.n, w.iters, 100
    K, _ = orc.gibbs_from_points_f32(w.x, w.y, w.eps, True)
    Kd = dev(K); a = dev(w.a); b = dev(w.b)

    def run(iters, flow=api.FSK_FLOW_FUSED):
        opts = api.make_opts(n, torch.float32, c=8, max_iters=iters, flow=flow)
        ws = api.alloc_workspace(opts)
        u = torch.ones(n, device="cuda"); v = torch.ones(n, device="cuda")
        api.fsk_sinkhorn_dense(opts, Kd, a, b, u, v, ws)
        rm = torch.empty(n, device="cuda"); cm = torch.empty(n, device="cuda")
        api.fsk_marginals(opts, Kd, a, u, v, rm, cm, ws)
        torch.cuda.synchronize()
        return u.cpu().numpy(), v.cpu().numpy(), rm.cpu().numpy(), cm.cpu().numpy()

    uo = vo = None
    worst = 0.0
    for t in range(step, T + 1, step):
        uo, vo = orc.sinkhorn_blocked(K, w.a, w.b, step, 8, 1, uo, vo)   # resumes exactly (fp64 state)
        u, v, rm, cm = run(t)
        eu, ev = relerr(u, uo), relerr(v, vo)
        gu, du = gauge_free(u, uo); gv, dv = gauge_free(v, vo)
        say(capsys, f"cfg3 t={t}: relerr u {eu:.2e} v {ev:.2e}; gauge-free u {gu:.2e} v {gv:.2e}; "
                    f"uniform drift u {du:.2e} v {dv:.2e}")
        assert eu <= 1e-4 and ev <= 1e-4 and gu <= 1e-4 and gv <= 1e-4
        worst = max(worst, eu, ev)
    # both marginals of the final state against the oracle's
    assert relerr(rm, orc.row_marginal(K, uo, vo)) <= 1e-4
    assert relerr(cm, orc.col_marginal(K, uo, vo)) <= 1e-4
    say(capsys, f"cfg3 full run: worst relative error on u, v over the checkpoints {worst:.2e}")
    # Algorithm 1 as printed (row slabs, then column slabs), the same 1000 iterations
    u, v, rm, cm = run(T, flow=api.FSK_FLOW_PAPER)
    eu, ev = relerr(u, uo), relerr(v, vo)
    gu, du = gauge_free(u, uo); gv, dv = gauge_free(v, vo)
    say(capsys, f"cfg3 t={T}, Algorithm-1 flow: relerr u {eu:.2e} v {ev:.2e}; gauge-free u {gu:.2e} v {gv:.2e}; "
                f"uniform drift u {du:.2e} v {dv:.2e}")
    assert eu <= 1e-4 and ev <= 1e-4 and gu <= 1e-4 and gv <= 1e-4
    assert relerr(cm, orc.col_marginal(K, uo, vo)) <= 1e-4


def test_cfg5_full_300_iterations_against_oracle(orc, capsys):
    """Configuration 5 for its own length: 300 iterations of the 64 stacked targets, compared
    every 30 iterations; the rescaling direction is taken out per target."""
    w = workloads.make(5)
    n, m, T, step = w.n, w.m, w.iters, 30
    K, _ = orc.gibbs_from_points_f32(w.x, w.y, w.eps, False)
    Kd = dev(K); A = dev(w.a); B = dev(w.b)

    def run(iters):
        opts = api.make_opts(n, torch.float32, m=m, max_iters=iters)
        ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
        U = torch.ones(n, m, device="cuda"); V = torch.ones(n, m, device="cuda")
        api.fsk_sinkhorn_batched(opts, Kd, A, B, U, V, ws)
        torch.cuda.synchronize()
        return U.cpu().numpy(), V.cpu().numpy()

    Uo = Vo = None
    for t in range(step, T + 1, step):
        Uo, Vo = orc.sinkhorn_batched(K, w.a, w.b, step, Uo, Vo)
        U, V = run(t)
        eu, ev = relerr(U, Uo), relerr(V, Vo)
        gu, du = gauge_free(U, Uo); gv, dv = gauge_free(V, Vo)
        say(capsys, f"cfg5 t={t}: relerr U {eu:.2e} V {ev:.2e}; gauge-free U {gu:.2e} V {gv:.2e}; "
                    f"largest uniform drift of a target U {du:.2e} V {dv:.2e}")
        assert eu <= 1e-4 and ev <= 1e-4 and gu <= 1e-4 and gv <= 1e-4
    # row marginals of the final state, three targets: U_ik (K V)_ik against the oracle's
    for k in (0, 31, 63):
        got = U[:, k].astype(np.float64) * orc.row_products(K, V[:, k])
        assert relerr(got, Uo[:, k] * orc.row_products(K, Vo[:, k])) <= 1e-4


def test_cfg4_law_to_its_stop_rule_against_oracle(orc, capsys):
    """The configuration-4 law at n = 4096 (x, y ~ U[0,1]^16, eps = 0.01, a = b = 1/n) run to a
    stop rule against the oracle under the same polling.  The configuration's own rule (L1 error
    below 1e-6 or 2000 iterations) ends at the cap for this law, in fp64 too, so a looser
    tolerance that IS reached goes first: there the stop iteration is compared and the potentials
    at the GPU's stop iteration; then both sides go on to the cap."""
    w = workloads.make(4, n=4096)
    n, d, eps, every = w.n, w.d, w.eps, 50
    x, y, a, b = dev(w.x), dev(w.y), dev(w.a), dev(w.b)

    def run(iters, tol):
        opts = api.make_opts(n, torch.float32, max_iters=iters, tol=tol, check_every=every)
        ws = api.alloc_workspace(opts, api.FSK_MODE_LOG, d)
        f = torch.zeros(n, device="cuda"); g = torch.zeros(n, device="cuda")
        done, err = api.fsk_sinkhorn_log_points(opts, x, y, eps, a, b, f, g, ws)
        torch.cuda.synchronize()
        return f.cpu().numpy().astype(np.float64), g.cpu().numpy().astype(np.float64), done, err

    def compare(tag, f, g, fo, go):
        ef, eg = np.max(np.abs(f - fo)) / eps, np.max(np.abs(g - go)) / eps
        # u = exp(f/eps): log(u/u_oracle) = (f - f_oracle)/eps, so the rescaling direction is a
        # constant shift of f (and the opposite one of g)
        df, dg = (f - fo) / eps, (g - go) / eps
        gf, gg = np.max(np.abs(df - df.mean())), np.max(np.abs(dg - dg.mean()))
        say(capsys, f"cfg4 law {tag}: |df|/eps {ef:.2e} |dg|/eps {eg:.2e}; gauge-free {gf:.2e} {gg:.2e}; "
                    f"uniform shift {df.mean():.2e} {dg.mean():.2e}")
        assert ef <= 1e-4 and eg <= 1e-4 and gf <= 1e-4 and gg <= 1e-4

    # (a) a tolerance both sides reach
    tol = 5e-4
    fo, go, done_o, err_o = orc.sinkhorn_log_points(w.x, w.y, eps, w.a, w.b, 2000, tol, every)
    say(capsys, f"cfg4 law: oracle stops after {done_o} iterations at L1 error {err_o:.3e} (tol {tol})")
    assert 0 < done_o < 2000 and err_o < tol
    f, g, done, err = run(2000, tol)
    assert done % every == 0 and err < tol
    assert abs(done - done_o) <= every          # fp32 exponentials may cross the threshold one poll apart
    if done != done_o:
        fo, go, _, _ = orc.sinkhorn_log_points(w.x, w.y, eps, w.a, w.b, done)
        done_o = done
    else:
        assert err == pytest.approx(err_o, rel=2e-2)
    compare(f"at the stop iteration {done}", f, g, fo, go)

    # (b) the configuration's rule: 1e-6 or 2000 iterations; the oracle resumes from (a)
    fo, go, more, err_o = orc.sinkhorn_log_points(w.x, w.y, eps, w.a, w.b, 2000 - done_o, 1e-6, every, fo, go)
    say(capsys, f"cfg4 law: oracle at {done_o + more} iterations, L1 error {err_o:.3e}")
    f, g, done, err = run(2000, 1e-6)
    assert done == done_o + more                # both at the cap (or both at the same poll)
    assert (err < 1e-6) == (err_o < 1e-6)
    assert err == pytest.approx(err_o, rel=5e-2)
    compare(f"after {done} iterations", f, g, fo, go)
