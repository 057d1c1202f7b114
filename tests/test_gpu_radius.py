"""GPU parity of the robust-risk kernel builder and the bisection radius search against the
oracle (appendix "Enforcing the Wasserstein radius")."""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev, relerr, tdtype

pytestmark = pytest.mark.gpu


def _problem(orc, n, dtype, seed):
    w = workloads.make(2, n=n)
    c64 = orc.cost_sqeuclid(w.x, w.y); c64 /= c64.max()
    c = np.ascontiguousarray(c64.astype(dtype))
    l = np.random.default_rng(seed).uniform(-0.05, 0.05, n).astype(dtype)
    return w, c, l


def _padded(n, td, fill=float("nan")):
    """n x n view of a matrix whose row pitch is a multiple of 16 bytes."""
    pack = 16 // torch.empty((), dtype=td).element_size()
    ld = (n + pack - 1) // pack * pack
    return torch.full((n, ld), fill, dtype=td, device="cuda")[:, :n]


@pytest.mark.parametrize("dtype,n", [(np.float32, 1030), (np.float64, 515)])
def test_kernel_from_cost_lambda(orc, dtype, n):
    w, c, l = _problem(orc, n, dtype, 1)
    td = tdtype(dtype)
    opts = api.make_opts(n, td)
    pack = 16 // np.dtype(dtype).itemsize
    ld = (n + pack - 1) // pack * pack
    K = torch.full((n, ld), float("nan"), dtype=td, device="cuda")
    cd = torch.zeros((n, ld), dtype=td, device="cuda"); cd[:, :n] = dev(c)
    for lam, lv in ((0.37, l), (2.5, None)):
        api.fsk_kernel_from_cost_lambda(opts, cd[:, :n], lam, None if lv is None else dev(lv), 0.1, K[:, :n])
        torch.cuda.synchronize()
        ref = orc.gibbs_lambda(c.astype(np.float64), lam, None if lv is None else lv.astype(np.float64), 0.1)
        # one rounding of the stored value plus the conditioning of exp at |argument| <= (lam + 0.05)/0.1
        ulp = np.finfo(dtype).eps
        bound = 2 * ulp + (lam + 0.05) / 0.1 * np.finfo(np.float64).eps * 2
        assert relerr(K[:, :n].cpu().numpy(), ref) <= bound
    assert torch.isnan(K[:, n:]).all()


@pytest.mark.parametrize("dtype,n,c_blocks,flow,tol", [
    (np.float32, 1024, 1, api.FSK_FLOW_FUSED, 1e-4),
    (np.float32, 1030, 5, api.FSK_FLOW_PAPER, 1e-4),
    (np.float64, 512, 4, api.FSK_FLOW_FUSED, 1e-10),
])
def test_radius_search_matches_oracle(orc, dtype, n, c_blocks, flow, tol):
    w, c, l = _problem(orc, n, dtype, 2)
    eps, iters, steps = 0.1, 60, 14
    c64 = c.astype(np.float64); l64 = l.astype(np.float64)
    a64 = w.a.astype(dtype).astype(np.float64); b64 = w.b.astype(dtype).astype(np.float64)
    # a radius between the costs at the ends of the bracket, from the oracle
    hi_cost = orc.radius_search(c64, l64, a64, b64, eps, 0.0, 0.0, 0.0, 1, 0.0, iters)[1]
    lo_cost = orc.radius_search(c64, l64, a64, b64, eps, 0.0, 3.0, 3.0, 1, 0.0, iters)[1]
    delta = 0.6 * lo_cost + 0.4 * hi_cost
    as_f32 = dtype == np.float32
    lam_o, cost_o, loss_o, steps_o, u_o, v_o, _ = orc.radius_search(
        c64, l64, a64, b64, eps, delta, 0.0, 3.0, steps, 0.0, iters, as_f32)

    td = tdtype(dtype)
    opts = api.make_opts(n, td, c=c_blocks, max_iters=iters, flow=flow)
    ws = api.alloc_workspace(opts, api.FSK_MODE_RADIUS)
    K = _padded(n, td)
    cd = _padded(n, td, 0.0); cd.copy_(dev(c))
    u = torch.full((n,), float("nan"), dtype=td, device="cuda")
    v = torch.full((n,), float("nan"), dtype=td, device="cuda")
    lam, cost, loss, done = api.fsk_radius_search(opts, cd, dev(l), dev(w.a.astype(dtype)),
                                                  dev(w.b.astype(dtype)), eps, delta, 0.0, 3.0, steps,
                                                  0.0, K, u, v, ws)
    assert done == steps_o == steps
    width = 3.0 / 2 ** steps
    # the bisection decisions are signs of g; a flip can only happen where |g| is at the rounding
    # level, and then the two searches end at most two final intervals apart
    assert abs(lam - lam_o) <= 2 * width
    if lam == lam_o:                                   # same decisions: the last solves are the same problem
        assert relerr(u.cpu().numpy(), u_o) <= tol and relerr(v.cpu().numpy(), v_o) <= tol
        assert abs(cost - cost_o) <= tol * abs(cost_o)
        assert abs(loss - loss_o) <= tol * np.abs(l64).max()
    assert abs(cost - delta) <= 2 * width * abs(hi_cost - lo_cost) + tol * delta
    # the loss term only rescales columns: sum_ij P_ij l_j = b^T l
    assert abs(loss - float(b64 @ l64)) <= max(tol, 1e-6) * np.abs(l64).max()


def test_radius_search_stops_on_gtol_and_validates(orc):
    n = 256
    w, c, l = _problem(orc, n, np.float32, 3)
    opts = api.make_opts(n, torch.float32, max_iters=50)
    ws = api.alloc_workspace(opts, api.FSK_MODE_RADIUS)
    K = torch.empty(n, n, device="cuda"); u = torch.empty(n, device="cuda"); v = torch.empty(n, device="cuda")
    cd, ld_, a, b = dev(c), dev(l), dev(w.a), dev(w.b)
    hi_cost = api.fsk_radius_search(opts, cd, ld_, a, b, 0.1, 0.0, 0.0, 0.0, 1, 0.0, K, u, v, ws)[1]
    lo_cost = api.fsk_radius_search(opts, cd, ld_, a, b, 0.1, 0.0, 3.0, 3.0, 1, 0.0, K, u, v, ws)[1]
    assert lo_cost < hi_cost
    delta = 0.5 * (lo_cost + hi_cost)
    gtol = 1e-3 * delta
    lam, cost, loss, done = api.fsk_radius_search(opts, cd, ld_, a, b, 0.1, delta, 0.0, 3.0, 40, gtol, K, u, v, ws)
    assert done < 40 and abs(cost - delta) <= gtol and 0.0 < lam < 3.0
    with pytest.raises(api.FskError):
        api.fsk_radius_search(opts, cd, ld_, a, b, 0.1, delta, 2.0, 1.0, 5, 0.0, K, u, v, ws)
    with pytest.raises(api.FskError):
        api.fsk_radius_search(opts, cd, ld_, a, b, 0.1, delta, 0.0, 1.0, 5, 0.0, cd, u, v, ws)
    with pytest.raises(api.FskError):
        api.fsk_radius_search(opts, cd, ld_, a, b, 0.1, delta, 0.0, 1.0, 5, 0.0, K, u, v, ws[:64])
