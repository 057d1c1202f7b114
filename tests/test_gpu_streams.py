"""Calls enqueued on separate streams (each with its own outputs and workspace) run side by
side without disturbing each other: the library keeps no device state of its own between or
across calls.  Every result must equal, bit for bit, what the same call gives alone."""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev

pytestmark = pytest.mark.gpu


def _dense_job(n, flow, c, iters):
    w = workloads.make(2, n=n)
    opts = api.make_opts(n, torch.float32, c=c, max_iters=iters, flow=flow)
    K = torch.empty(n, n, device="cuda")
    api.fsk_kernel_from_points(opts, dev(w.x.astype(np.float32)), dev(w.y.astype(np.float32)), w.eps, True, K,
                               api.alloc_workspace(opts, api.FSK_MODE_SETUP))
    a, b = dev(w.a.astype(np.float32)), dev(w.b.astype(np.float32))
    u = torch.empty(n, device="cuda"); v = torch.empty(n, device="cuda")
    ws = api.alloc_workspace(opts)
    reset = lambda: (u.fill_(1.0), v.fill_(1.0))
    return reset, (lambda s: api.fsk_sinkhorn_dense(opts, K, a, b, u, v, ws, stream=s)), [u, v]


def _batched_job(n, m, td, iters, damping=api.FSK_DAMP_NONE):
    nd = np.float64 if td == torch.float64 else np.float32
    w = workloads.make(5, n=n, m=m, seed=31)
    opts = api.make_opts(n, td, m=m, max_iters=iters, damping=damping, eta=0.6)
    K = torch.empty(n, n, dtype=td, device="cuda")
    api.fsk_kernel_from_points(opts, dev(w.x.astype(nd)), dev(w.y.astype(nd)), 0.2, False, K, None)
    A, B = dev(np.ascontiguousarray(w.a.astype(nd))), dev(np.ascontiguousarray(w.b.astype(nd)))
    U = torch.empty(n, m, dtype=td, device="cuda"); V = torch.empty(n, m, dtype=td, device="cuda")
    ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
    reset = lambda: (U.fill_(1.0), V.fill_(1.0))
    return reset, (lambda s: api.fsk_sinkhorn_batched(opts, K, A, B, U, V, ws, stream=s)), [U, V]


def _log_job(n, iters):
    w = workloads.make(4, n=n)
    opts = api.make_opts(n, torch.float32, max_iters=iters)
    x, y, a, b = dev(w.x), dev(w.y), dev(w.a), dev(w.b)
    f = torch.empty(n, device="cuda"); g = torch.empty(n, device="cuda")
    ws = api.alloc_workspace(opts, api.FSK_MODE_LOG, w.x.shape[1])
    reset = lambda: (f.zero_(), g.zero_())
    return reset, (lambda s: api.fsk_sinkhorn_log_points(opts, x, y, w.eps, a, b, f, g, ws, stream=s)), [f, g]


def test_calls_on_separate_streams_do_not_disturb_each_other():
    jobs = [_dense_job(2048, api.FSK_FLOW_FUSED, 8, 60), _dense_job(1024, api.FSK_FLOW_TWO_PASS, 1, 60),
            _dense_job(2048, api.FSK_FLOW_FUSED, 1, 60),          # same shape as the first: same kernels, other buffers
            _batched_job(1024, 64, torch.float32, 20), _batched_job(768, 70, torch.float64, 10),
            _batched_job(1024, 40, torch.float32, 20, api.FSK_DAMP_GEOMETRIC), _log_job(3000, 10)]
    alone = []
    for reset, call, outs in jobs:                  # each call by itself on the current stream
        reset(); call(None); torch.cuda.synchronize()
        alone.append([t.clone() for t in outs])
    streams = [torch.cuda.Stream() for _ in jobs]   # default priority
    for reset, _, _ in jobs:
        reset()
    torch.cuda.synchronize()
    for (_, call, _), s in zip(jobs, streams):      # all in flight together
        call(s)
    torch.cuda.synchronize()
    for k, ((_, _, outs), want) in enumerate(zip(jobs, alone)):
        for got, ref in zip(outs, want):
            assert torch.equal(got, ref), f"job {k} differs when run beside the others"
