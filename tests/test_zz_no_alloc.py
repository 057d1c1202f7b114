"""The dense call on the library's built-in scratch array (for callers that cannot allocate)
against the ordinary call with a workspace: same kernels, so the results must be identical.
Two calls in a row, the second on a smaller problem, so that what the first call left in the
shared array is there when the second runs."""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev, relerr

pytestmark = pytest.mark.gpu


def _problem(orc, n, dtype, seed):
    w = workloads.make(2, n=n, seed=seed)
    K64, _ = orc.gibbs_from_points(w.x, w.y, w.eps, True)
    nd = np.float64 if dtype == torch.float64 else np.float32
    pack = 16 // np.dtype(nd).itemsize
    ld = (n + pack - 1) // pack * pack
    Kd = torch.zeros(n, ld, dtype=dtype, device="cuda")[:, :n]
    Kd.copy_(dev(K64.astype(nd)))
    return K64.astype(nd), Kd, w.a.astype(nd), w.b.astype(nd)


def _both(opts, Kd, a, b, dtype):
    n = opts.n
    u1 = torch.ones(n, dtype=dtype, device="cuda"); v1 = torch.ones(n, dtype=dtype, device="cuda")
    u2 = torch.ones(n, dtype=dtype, device="cuda"); v2 = torch.ones(n, dtype=dtype, device="cuda")
    r2 = api.fsk_sinkhorn_dense_static(opts, Kd, dev(a), dev(b), u2, v2)
    torch.cuda.synchronize()
    ws = api.alloc_workspace(opts)
    r1 = api.fsk_sinkhorn_dense(opts, Kd, dev(a), dev(b), u1, v1, ws)
    torch.cuda.synchronize()
    return (u1, v1, r1), (u2, v2, r2)


def test_static_scratch_call_equals_the_workspace_call_twice_in_a_row(orc):
    cases = [  # (n, dtype, c, flow, iterations, tol): the second of each pair is the smaller one
        (4096, torch.float32, 4, api.FSK_FLOW_FUSED, 40, 0.0),
        (1000, torch.float32, 1, api.FSK_FLOW_FUSED, 40, 0.0),
        (1537, torch.float64, 1, api.FSK_FLOW_TWO_PASS, 25, 0.0),
        (512, torch.float64, 4, api.FSK_FLOW_PAPER, 25, 0.0),
        (2048, torch.float32, 2, api.FSK_FLOW_FUSED, 400, 1e-5),      # tolerance mode: polls, restore
        (512, torch.float64, 1, api.FSK_FLOW_RESIDENT, 30, 0.0),      # its barrier counter starts at zero
    ]
    for n, dtype, c, flow, iters, tol in cases:
        print(f"case n={n} dtype={dtype} c={c} flow={flow} iters={iters} tol={tol}", flush=True)
        K, Kd, a, b = _problem(orc, n, dtype, 700 + n)
        opts = api.make_opts(n, dtype, c=c, max_iters=iters, flow=flow, tol=tol, check_every=7)
        (u1, v1, r1), (u2, v2, r2) = _both(opts, Kd, a, b, dtype)
        assert torch.equal(u1, u2) and torch.equal(v1, v2)
        assert r1[0] == r2[0] and (r1[1] == r2[1] or (np.isnan(r1[1]) and np.isnan(r2[1])))
        # and both are the method's iterates
        if tol > 0:
            uo, vo, done_o, _ = orc.sinkhorn_dense_tol(K, a, b, iters, tol, 7)
            assert abs(done_o - r2[0]) <= 7
            uo, vo = orc.sinkhorn_dense(K, a, b, r2[0])
        else:
            uo, vo = orc.sinkhorn_dense(K, a, b, iters)
        bar = 1e-10 if dtype == torch.float64 else 1e-4
        assert relerr(u2.cpu().numpy(), uo) <= bar and relerr(v2.cpu().numpy(), vo) <= bar


def test_static_scratch_call_refuses_a_problem_beyond_the_array():
    n = 46400
    opts = api.make_opts(n, torch.float32, max_iters=1, flow=api.FSK_FLOW_TWO_PASS)
    K = torch.empty(8, n, device="cuda")       # never read: the size check comes first
    x = torch.ones(n, device="cuda")
    with pytest.raises(api.FskError) as e:
        api.fsk_sinkhorn_dense_static(opts, K, x, x, x, x)
    assert e.value.status == api.FSK_EWORKSPACE
