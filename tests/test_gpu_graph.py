"""The fixed-iteration entry points only enqueue kernels on the caller's stream (no allocation,
no synchronisation, no memset nodes), so a caller can record them into a HIP graph.  Each case
records one call, then replays the graph several times with ordinary eager work and
synchronisations in between, and compares every replay bit for bit with the eager call."""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev

pytestmark = pytest.mark.gpu


def _replay_matches_eager(call, outputs, reset):
    """call(): the library call; outputs: tensors it writes; reset(): restore the start state."""
    reset(); call(); torch.cuda.synchronize()          # eager run (also the warm-up of the capture)
    want = [t.clone() for t in outputs]
    reset(); torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for rep in range(3):
        reset()                                         # eager kernels between the replays
        scratch = torch.rand(1 << 16, device="cuda").sum().item()   # unrelated eager work + a sync
        assert np.isfinite(scratch)
        g.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outputs, want):
            assert torch.equal(got, ref), f"replay {rep} differs from the eager call"


@pytest.mark.parametrize("n,td,flow,c", [
    (2048, torch.float32, api.FSK_FLOW_FUSED, 1),
    (2048, torch.float32, api.FSK_FLOW_FUSED, 8),
    (1030, torch.float32, api.FSK_FLOW_TWO_PASS, 1),
    (1024, torch.float32, api.FSK_FLOW_PAPER, 4),
    (512, torch.float64, api.FSK_FLOW_RESIDENT, 1),
])
def test_dense_call_in_a_graph(n, td, flow, c):
    w = workloads.make(2, n=n)
    nd = np.float64 if td == torch.float64 else np.float32
    opts = api.make_opts(n, td, c=c, max_iters=40, flow=flow)
    pack = 16 // np.dtype(nd).itemsize
    ld = (n + pack - 1) // pack * pack
    K = torch.empty(n, ld, dtype=td, device="cuda")[:, :n]
    api.fsk_kernel_from_points(opts, dev(w.x.astype(nd)), dev(w.y.astype(nd)), w.eps, True, K,
                               api.alloc_workspace(opts, api.FSK_MODE_SETUP))
    a, b = dev(w.a.astype(nd)), dev(w.b.astype(nd))
    u = torch.empty(n, dtype=td, device="cuda"); v = torch.empty(n, dtype=td, device="cuda")
    ws = api.alloc_workspace(opts)

    def reset():
        u.fill_(1.0); v.fill_(1.0)

    _replay_matches_eager(lambda: api.fsk_sinkhorn_dense(opts, K, a, b, u, v, ws), [u, v], reset)


@pytest.mark.parametrize("td,m,damping", [(torch.float32, 64, api.FSK_DAMP_NONE), (torch.float32, 150, api.FSK_DAMP_NONE),
                                          (torch.float64, 64, api.FSK_DAMP_NONE),
                                          (torch.float32, 70, api.FSK_DAMP_GEOMETRIC),
                                          (torch.float64, 33, api.FSK_DAMP_ARITHMETIC)])
def test_batched_call_in_a_graph(td, m, damping):
    n = 1030
    nd = np.float64 if td == torch.float64 else np.float32
    w = workloads.make(5, n=n, m=m, seed=77)
    opts = api.make_opts(n, td, m=m, max_iters=10, damping=damping, eta=0.6)
    pack = 16 // np.dtype(nd).itemsize
    ld = (n + pack - 1) // pack * pack
    K = torch.empty(n, ld, dtype=td, device="cuda")[:, :n]
    api.fsk_kernel_from_points(opts, dev(w.x.astype(nd)), dev(w.y.astype(nd)), w.eps, False, K, None)
    A, B = dev(np.ascontiguousarray(w.a.astype(nd))), dev(np.ascontiguousarray(w.b.astype(nd)))
    U = torch.empty(n, m, dtype=td, device="cuda"); V = torch.empty(n, m, dtype=td, device="cuda")
    ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)

    def reset():
        U.fill_(1.0); V.fill_(1.0)

    _replay_matches_eager(lambda: api.fsk_sinkhorn_batched(opts, K, A, B, U, V, ws), [U, V], reset)


def test_log_domain_call_in_a_graph():
    n, d = 1500, 16
    w = workloads.make(4, n=n)
    opts = api.make_opts(n, torch.float32, max_iters=12)
    x, y, a, b = dev(w.x), dev(w.y), dev(w.a), dev(w.b)
    f = torch.empty(n, device="cuda"); g = torch.empty(n, device="cuda")
    ws = api.alloc_workspace(opts, api.FSK_MODE_LOG, d)

    def reset():
        f.zero_(); g.zero_()

    _replay_matches_eager(lambda: api.fsk_sinkhorn_log_points(opts, x, y, w.eps, a, b, f, g, ws), [f, g], reset)


@pytest.mark.parametrize("which", ["local_steps", "async", "grid", "static"])
def test_other_dense_calls_in_a_graph(which):
    """The schedules built from the two-pass kernels (their device-to-device copies become memcpy
    nodes) and the dense call on the library's built-in scratch, which exists for exactly this
    caller: code under capture cannot allocate."""
    n = 1536
    w = workloads.make(3, n=n)
    opts = api.make_opts(n, torch.float32, c=4, max_iters=14)
    K = torch.empty(n, n, device="cuda")
    api.fsk_kernel_from_points(opts, dev(w.x), dev(w.y), 0.2, True, K,
                               api.alloc_workspace(opts, api.FSK_MODE_SETUP))
    a, b = dev(w.a), dev(w.b)
    u = torch.empty(n, device="cuda"); v = torch.empty(n, device="cuda")

    def reset():
        u.fill_(1.0); v.fill_(1.0)

    if which == "local_steps":
        ws = torch.empty(api.fsk_local_steps_workspace_bytes(opts), dtype=torch.uint8, device="cuda")
        call = lambda: api.fsk_sinkhorn_local_steps(opts, K, a, b, u, v, 3, ws)
    elif which == "async":
        opts.damping = api.FSK_DAMP_ARITHMETIC; opts.eta = 0.7
        ws = torch.empty(api.fsk_async_workspace_bytes(opts, 1, 2), dtype=torch.uint8, device="cuda")
        call = lambda: api.fsk_sinkhorn_async_emulated(opts, K, a, b, u, v, 1, 2, ws)
    elif which == "grid":
        ws = torch.empty(api.fsk_grid_workspace_bytes(opts, 4, 2), dtype=torch.uint8, device="cuda")
        call = lambda: api.fsk_sinkhorn_grid(opts, K, a, b, u, v, 4, 2, ws)
    else:
        call = lambda: api.fsk_sinkhorn_dense_static(opts, K, a, b, u, v)
    _replay_matches_eager(call, [u, v], reset)
