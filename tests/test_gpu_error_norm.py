"""Tolerance mode on the paper's own metric, ||P1 - a||_2 (fsk_opts.err_norm = FSK_NORM_L2), in
the dense, register-resident, log-domain and multitarget calls, against the oracle's rule."""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev, relerr, run_dense

pytestmark = pytest.mark.gpu
L2 = api.FSK_NORM_L2


@pytest.mark.parametrize("flow", [api.FSK_FLOW_FUSED, api.FSK_FLOW_TWO_PASS, api.FSK_FLOW_PAPER,
                                  api.FSK_FLOW_RESIDENT])
def test_dense_stop_rule_on_the_two_norm(orc, flow):
    w = workloads.make(1, n=300)                                  # fp64
    K, _ = orc.gibbs_from_points(w.x, w.y, w.eps, False)
    tol, ce = 1e-9, 7
    uo, vo, done_o, err_o = orc.sinkhorn_dense_tol(K, w.a, w.b, 5000, tol, check_every=ce, l2=True)
    _, _, done_1, _ = orc.sinkhorn_dense_tol(K, w.a, w.b, 5000, tol, check_every=ce)
    assert done_o < done_1                                        # the two norms stop at different polls here
    u, v, done, err = run_dense(K, w.a, w.b, 5000, flow=flow, tol=tol, check_every=ce, err_norm=L2)
    assert done == done_o and err < tol and err == pytest.approx(err_o, rel=1e-3)
    assert relerr(u, uo) <= 1e-10 and relerr(v, vo) <= 1e-10
    assert err == pytest.approx(orc.marginal_error(K, w.a, u, v)[1], rel=1e-3)
    uf, vf, _, _ = run_dense(K, w.a, w.b, done, flow=flow)        # the state of the fixed-count run
    assert np.array_equal(u, uf) and np.array_equal(v, vf)
    # the cap: the last iteration is polled in the chosen norm
    u, v, done, err = run_dense(K, w.a, w.b, 10, flow=flow, tol=1e-300, check_every=4, err_norm=L2)
    assert done == 10 and err == pytest.approx(orc.marginal_error(K, w.a, u, v)[1], rel=1e-6)


def test_dense_fp32_blocks_two_norm(orc):
    w3 = workloads.make(3, n=512)
    K3, _ = orc.gibbs_from_points_f32(w3.x, w3.y, w3.eps, True)
    uo, vo, done_o, err_o = orc.sinkhorn_dense_tol(K3, w3.a, w3.b, 3000, 2e-6, check_every=1, l2=True)
    for flow, c in ((api.FSK_FLOW_FUSED, 8), (api.FSK_FLOW_PAPER, 4)):
        u, v, done, err = run_dense(K3, w3.a, w3.b, 3000, flow=flow, c=c, tol=2e-6, check_every=1, err_norm=L2)
        assert abs(done - done_o) <= 1 and err < 2e-6
        assert err == pytest.approx(orc.marginal_error(K3, w3.a, u, v)[1], rel=0.05, abs=2e-8)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_log_domain_stop_rule_on_the_two_norm(orc, dtype):
    w = workloads.make(4, n=700)
    eps = 0.05
    tol = 3e-7 if dtype == np.float32 else 1e-8
    td = torch.float64 if dtype == np.float64 else torch.float32
    fo, go, done_o, err_o = orc.sinkhorn_log_points(w.x, w.y, eps, w.a, w.b, 3000, tol=tol, check_every=5, l2=True)
    opts = api.make_opts(700, td, max_iters=3000, tol=tol, check_every=5, err_norm=L2)
    ws = api.alloc_workspace(opts, api.FSK_MODE_LOG, w.x.shape[1])
    f = torch.zeros(700, dtype=td, device="cuda"); g = torch.zeros(700, dtype=td, device="cuda")
    cast = lambda t: dev(np.ascontiguousarray(t.astype(dtype)))
    done, err = api.fsk_sinkhorn_log_points(opts, cast(w.x), cast(w.y), eps, cast(w.a), cast(w.b), f, g, ws)
    assert done % 5 == 0 and err < tol
    rows = orc.log_row_marginal_points(w.x, f.double().cpu().numpy(), w.y, g.double().cpu().numpy(), eps)
    if dtype == np.float64:
        assert done == done_o and err == pytest.approx(err_o, rel=1e-4)
        assert err == pytest.approx(np.linalg.norm(rows - w.a), rel=1e-4)
    else:
        assert abs(done - done_o) <= 5
        assert err == pytest.approx(np.linalg.norm(rows - w.a), rel=0.1, abs=3e-8)


@pytest.mark.parametrize("dtype,n,m", [(np.float64, 300, 70), (np.float32, 515, 33)])
def test_multitarget_stop_rule_on_the_two_norm(orc, dtype, n, m):
    rng = np.random.default_rng(4100 + n)
    x = rng.uniform(size=(n, 2)); y = rng.uniform(size=(n, 2))
    K64, _ = orc.gibbs_from_points(x, y, 0.3, False)
    K = np.ascontiguousarray(K64.astype(dtype))
    A = rng.uniform(0.5, 1.5, (n, m)) ** 3; A = np.ascontiguousarray((A / A.sum(0)).astype(dtype))
    B = rng.uniform(0.5, 1.5, (n, m)) ** 3; B = np.ascontiguousarray((B / B.sum(0)).astype(dtype))
    tol, ce = (1e-10, 3) if dtype == np.float64 else (3e-7, 2)
    Uo, Vo, done_o, err_o = orc.sinkhorn_batched_tol(K, A, B, 400, tol, ce, l2=True)
    td = torch.float64 if dtype == np.float64 else torch.float32
    opts = api.make_opts(n, td, m=m, max_iters=400, tol=tol, check_every=ce, err_norm=L2)
    ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
    pack = 16 // np.dtype(dtype).itemsize
    full = torch.full((n, (n + pack - 1) // pack * pack), float("nan"), dtype=td, device="cuda")
    full[:, :n] = dev(K)
    U = torch.ones(n, m, dtype=td, device="cuda"); V = torch.ones(n, m, dtype=td, device="cuda")
    done, err = api.fsk_sinkhorn_batched_tol(opts, full[:, :n], dev(A), dev(B), U, V, ws)
    U = U.cpu().numpy(); V = V.cpu().numpy()
    assert done_o < 400 and err < tol and done % ce == 0
    worst = max(orc.marginal_error(K, A[:, k], U[:, k], V[:, k])[1] for k in range(m))
    if dtype == np.float64:
        assert done == done_o and err == pytest.approx(err_o, rel=1e-4)
        assert relerr(U, Uo) <= 1e-10 and relerr(V, Vo) <= 1e-10
        assert err == pytest.approx(worst, rel=1e-3)
    else:
        assert abs(done - done_o) <= ce
        assert err == pytest.approx(worst, rel=0.1, abs=3e-8)


def test_unknown_norm_is_refused():
    opts = api.make_opts(64, torch.float32, max_iters=1, err_norm=7)
    X = torch.ones(64, 64, device="cuda"); x = torch.ones(64, device="cuda")
    with pytest.raises(api.FskError) as e:
        api.fsk_sinkhorn_dense(opts, X, x, x, x.clone(), x.clone(), api.alloc_workspace(api.make_opts(64)))
    assert e.value.status == api.FSK_EINVAL
