"""GPU parity of the synchronous iteration with w local steps between collectives (Sec. 3.1
Remark; appendix on local steps) against the oracle's per-client-view statement of it."""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import TOL, dev, relerr, run_dense, tdtype

pytestmark = pytest.mark.gpu


def run_local(K, a, b, iters, c, w, u0=None, v0=None):
    n = K.shape[0]; dt = K.dtype; td = tdtype(dt)
    pack = 16 // np.dtype(dt).itemsize
    ld = (n + pack - 1) // pack * pack
    Kd = torch.full((n, ld), float("nan"), dtype=td, device="cuda")[:, :n]
    Kd.copy_(dev(K))
    opts = api.make_opts(n, td, c=c, max_iters=iters)
    ws = torch.empty(api.fsk_local_steps_workspace_bytes(opts), dtype=torch.uint8, device="cuda")
    u = torch.ones(n, dtype=td, device="cuda") if u0 is None else dev(u0.astype(dt))
    v = torch.ones(n, dtype=td, device="cuda") if v0 is None else dev(v0.astype(dt))
    api.fsk_sinkhorn_local_steps(opts, Kd, dev(a.astype(dt)), dev(b.astype(dt)), u, v, w, ws)
    torch.cuda.synchronize()
    return u.cpu().numpy(), v.cpu().numpy()


def problem(orc, n, dtype, eps=0.2):
    wl = workloads.make(3, n=n)
    K64, _ = orc.gibbs_from_points(wl.x, wl.y, eps, True)
    return np.ascontiguousarray(K64.astype(dtype)), wl.a.astype(dtype), wl.b.astype(dtype)


@pytest.mark.parametrize("dtype,n", [(np.float32, 1024), (np.float64, 520), (np.float32, 1000)])
@pytest.mark.parametrize("c,w,iters", [(4, 1, 20), (4, 2, 21), (8, 5, 23), (2, 7, 30), (5, 3, 10)])
def test_local_steps_match_oracle(orc, dtype, n, c, w, iters):
    """Several (clients, local steps), iteration counts that end inside a round as well as at a
    collective; n = 1000 with c = 8 or 5 gives blocks of 125 / 200 entries, which do not start on
    16-byte boundaries (a pack of four columns then belongs to two clients)."""
    K, a, b = problem(orc, n, dtype)
    if n % c != 0:                   # both sides refuse blocks of unequal height (n = c m, Sec. 3.1)
        with pytest.raises(api.FskError) as e:
            run_local(K, a, b, iters, c, w)
        assert e.value.status == api.FSK_EDIV
        with pytest.raises(ValueError):
            orc.sinkhorn_local_steps(K, a, b, iters, c, w)
        return
    uo, vo = orc.sinkhorn_local_steps(K, a, b, iters, c, w)
    u, v = run_local(K, a, b, iters, c, w)
    assert relerr(u, uo) <= TOL[np.dtype(dtype)] and relerr(v, vo) <= TOL[np.dtype(dtype)]
    if w > 1 and c > 1:      # the schedule matters: Algorithm 1 is somewhere else by now
        ud, vd = orc.sinkhorn_dense(K, a, b, iters)
        assert relerr(uo, ud) > 1e-3


@pytest.mark.parametrize("dtype,n,c", [(np.float32, 2048, 8), (np.float64, 777, 7), (np.float32, 1000, 8)])
def test_one_local_step_is_algorithm_1_bit_for_bit(orc, dtype, n, c):
    """w = 1: every iteration gathers, the views are the global vectors, and the call enqueues
    the kernels of the Algorithm-1 flow on the same values."""
    K, a, b = problem(orc, n, dtype)
    u, v = run_local(K, a, b, 25, c, 1)
    up, vp, _, _ = run_dense(K, a, b, 25, flow=api.FSK_FLOW_PAPER, c=c)
    assert np.array_equal(u, up) and np.array_equal(v, vp)
    # one client has no peers: any w is the centralised run
    u1, v1 = run_local(K, a, b, 25, 1, 6)
    ut, vt, _, _ = run_dense(K, a, b, 25, flow=api.FSK_FLOW_TWO_PASS, c=1)
    assert np.array_equal(u1, ut) and np.array_equal(v1, vt)


def test_local_steps_resume_at_a_collective_and_reject_bad_arguments(orc):
    K, a, b = problem(orc, 768, np.float32)
    u, v = run_local(K, a, b, 24, 4, 3)
    ua, va = run_local(K, a, b, 9, 4, 3)
    ub, vb = run_local(K, a, b, 15, 4, 3, ua, va)
    assert np.array_equal(u, ub) and np.array_equal(v, vb)
    opts = api.make_opts(64, torch.float32, c=2, max_iters=1)
    Kd = torch.ones(64, 64, device="cuda"); x = torch.ones(64, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(api.FskError) as e:
        api.fsk_sinkhorn_local_steps(opts, Kd, x, x, x.clone(), x.clone(), 0, ws)
    assert e.value.status == api.FSK_EINVAL
    opts.damping = api.FSK_DAMP_ARITHMETIC; opts.eta = 0.5
    with pytest.raises(api.FskError) as e:
        api.fsk_sinkhorn_local_steps(opts, Kd, x, x, x.clone(), x.clone(), 2, ws)
    assert e.value.status == api.FSK_EUNSUPPORTED
    opts.damping = api.FSK_DAMP_NONE
    with pytest.raises(api.FskError) as e:
        api.fsk_sinkhorn_local_steps(opts, Kd, x, x, x.clone(), x.clone(), 2, ws[:64])
    assert e.value.status == api.FSK_EWORKSPACE


def test_local_steps_at_configuration_3_size(orc):
    """n = 32768, c = 8, w = 4 in the launch shapes a full-size run uses: 8 iterations (two
    rounds) against the oracle."""
    wl = workloads.make(3)
    K, _ = orc.gibbs_from_points_f32(wl.x, wl.y, wl.eps, True)
    uo, vo = orc.sinkhorn_local_steps(K, wl.a, wl.b, 8, 8, 4)
    u, v = run_local(K, wl.a, wl.b, 8, 8, 4)
    assert relerr(u, uo) <= 1e-4 and relerr(v, vo) <= 1e-4
