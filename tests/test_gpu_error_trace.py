"""The error trace: every poll of a tolerance-mode call leaves (iteration, error) in a buffer the
caller lent (the paper plots the marginal error err_a against the iteration count, Sec. 5.4).  The
recorded errors are checked against the oracle's evaluation of the oracle's own iterates at the
same iterations."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev

pytestmark = pytest.mark.gpu


def _trace(cap):
    buf = (ctypes.c_double * (2 * cap))()
    api.fsk_set_error_trace(buf, cap)
    return buf


def _pairs(buf, count, cap):
    a = np.frombuffer(buf, dtype=np.float64).reshape(-1, 2)[:min(count, cap)]
    return a[:, 0].astype(int), a[:, 1].copy()


def test_dense_trace_matches_the_oracle_error_at_every_poll(orc):
    n, every, tol = 600, 6, 1e-7
    w = workloads.make(1, n=n)
    K64, _ = orc.gibbs_from_points(w.x, w.y, w.eps, False)
    try:
        for flow, c in ((api.FSK_FLOW_FUSED, 4), (api.FSK_FLOW_TWO_PASS, 1), (api.FSK_FLOW_RESIDENT, 1)):
            n_ = 512 if flow == api.FSK_FLOW_RESIDENT else n
            K = np.ascontiguousarray(K64[:n_, :n_]); a = np.full(n_, 1.0 / n_); b = a.copy()
            buf = _trace(64)
            opts = api.make_opts(n_, torch.float64, c=c, max_iters=200, tol=tol, check_every=every, flow=flow)
            u = torch.ones(n_, dtype=torch.float64, device="cuda"); v = torch.ones_like(u)
            done, err = api.fsk_sinkhorn_dense(opts, dev(K), dev(a), dev(b), u, v, api.alloc_workspace(opts))
            count = api.fsk_error_trace_count()
            its, errs = _pairs(buf, count, 64)
            assert count == len(its) == done // every and done % every == 0   # stopped at a poll
            assert list(its) == list(range(every, done + 1, every))
            assert errs[-1] == err and err < tol and np.all(errs[:-1] >= tol)
            assert np.all(np.diff(errs) < 0)              # the L1 marginal error of Sinkhorn never increases
            for k in (0, len(its) // 2, len(its) - 1):    # the oracle's error of its own state there
                uo, vo = orc.sinkhorn_dense(K, a, b, int(its[k]))
                e1, _ = orc.marginal_error(K, a, uo, vo)
                assert errs[k] == pytest.approx(e1, rel=1e-6)
        # a buffer that is too small: the count goes on, the buffer holds the first polls
        buf = _trace(2)
        u.fill_(1.0); v.fill_(1.0)
        opts = api.make_opts(n_, torch.float64, max_iters=40, tol=1e-300, check_every=4, flow=api.FSK_FLOW_TWO_PASS)
        done, err = api.fsk_sinkhorn_dense(opts, dev(K), dev(a), dev(b), u, v, api.alloc_workspace(opts))
        assert done == 40 and api.fsk_error_trace_count() == 10
        its, errs = _pairs(buf, 10, 2)
        assert list(its) == [4, 8]
        # a fixed-iteration call leaves the last trace alone; switching off stops the recording
        opts.tol = 0.0
        api.fsk_sinkhorn_dense(opts, dev(K), dev(a), dev(b), u, v, api.alloc_workspace(opts))
        assert api.fsk_error_trace_count() == 10
    finally:
        api.fsk_set_error_trace(None, 0)
    assert api.fsk_error_trace_count() == 0


def test_log_domain_and_multitarget_calls_trace_their_polls(orc):
    try:
        # log domain
        w = workloads.make(4, n=700)
        buf = _trace(32)
        opts = api.make_opts(700, torch.float64, max_iters=60, tol=1e-300, check_every=10)
        f = torch.zeros(700, dtype=torch.float64, device="cuda"); g = torch.zeros_like(f)
        x, y = dev(w.x.astype(np.float64)), dev(w.y.astype(np.float64))
        a, b = dev(w.a.astype(np.float64)), dev(w.b.astype(np.float64))
        done, err = api.fsk_sinkhorn_log_points(opts, x, y, 0.05, a, b, f, g,
                                                api.alloc_workspace(opts, api.FSK_MODE_LOG, w.d))
        its, errs = _pairs(buf, api.fsk_error_trace_count(), 32)
        assert list(its) == [10, 20, 30, 40, 50, 60] and errs[-1] == err
        fo, go, _, eo = orc.sinkhorn_log_points(w.x, w.y, 0.05, w.a, w.b, 30, 1e-300, 30)
        assert errs[2] == pytest.approx(eo, rel=1e-6)
        # multitarget: the maximum over the targets
        w5 = workloads.make(5, n=520, m=12, seed=9)
        K64, _ = orc.gibbs_from_points(w5.x, w5.y, w5.eps, False)
        buf = _trace(32)
        opts = api.make_opts(520, torch.float64, m=12, max_iters=25, tol=1e-300, check_every=5)
        U = torch.ones(520, 12, dtype=torch.float64, device="cuda"); V = torch.ones_like(U)
        A, B = dev(w5.a.astype(np.float64)), dev(w5.b.astype(np.float64))
        done, err = api.fsk_sinkhorn_batched_tol(opts, dev(K64), A, B, U, V,
                                                 api.alloc_workspace(opts, api.FSK_MODE_BATCHED))
        its, errs = _pairs(buf, api.fsk_error_trace_count(), 32)
        assert list(its) == [5, 10, 15, 20, 25] and errs[-1] == err
        Uo, Vo, _, eo = orc.sinkhorn_batched_tol(K64, w5.a, w5.b, 10, 1e-300, 10)
        assert errs[1] == pytest.approx(eo, rel=1e-6)
    finally:
        api.fsk_set_error_trace(None, 0)
