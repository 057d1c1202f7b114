"""Seeded random VALID problems (size, precision, flow, block count, damping, row pitch, iteration
count drawn at random) through the C ABI against the oracle, at the usual bars: 1e-4 (fp32) and
1e-10 (fp64) on the scalings (|f - f_oracle| / eps in the log domain), and random stop rules
against the oracle's.  Complements the hand-picked sizes of the other files."""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api
from gpu_util import dev, relerr

pytestmark = pytest.mark.gpu


def _pick(rng):
    dtype = np.float32 if rng.random() < 0.6 else np.float64
    return dtype, (torch.float32 if dtype == np.float32 else torch.float64), (1e-4 if dtype == np.float32 else 1e-10)


def _padded(K, td, extra_packs):
    n = K.shape[0]
    pack = 16 // K.dtype.itemsize
    ld = (n + pack - 1) // pack * pack + pack * extra_packs
    full = torch.full((n, ld), float("nan"), dtype=td, device="cuda")
    full[:, :n] = dev(K)
    return full


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_dense_problems(orc, seed):
    rng = np.random.default_rng(seed)
    for case in range(25):
        dtype, td, tol = _pick(rng)
        n = int(rng.choice([rng.integers(1, 70), rng.integers(1, 1200), rng.integers(1000, 4200),
                            rng.integers(4000, 9000)], p=[0.2, 0.4, 0.3, 0.1]))
        resident_ok = n <= (1024 if dtype == np.float32 else 512)
        flow = int(rng.choice([api.FSK_FLOW_FUSED, api.FSK_FLOW_TWO_PASS, api.FSK_FLOW_PAPER]
                              + ([api.FSK_FLOW_RESIDENT] if resident_ok else [])))
        c = int(rng.choice([k for k in range(1, min(n, 64) + 1) if n % k == 0]))
        damping = int(rng.choice([api.FSK_DAMP_NONE, api.FSK_DAMP_ARITHMETIC, api.FSK_DAMP_GEOMETRIC],
                                 p=[0.6, 0.25, 0.15]))
        eta = float(rng.uniform(0.3, 1.0))
        iters = int(rng.integers(1, 6))
        d = int(rng.integers(1, 5))
        x = rng.standard_normal((n, d)); y = rng.standard_normal((n, d)) + 0.3
        K64, _ = orc.gibbs_from_points(x, y, float(rng.uniform(0.2, 1.0)), True)
        K = np.ascontiguousarray(K64.astype(dtype))
        a = rng.uniform(0.5, 1.5, n); a = (a / a.sum()).astype(dtype)
        b = rng.uniform(0.5, 1.5, n); b = (b / b.sum()).astype(dtype)
        full = _padded(K, td, int(rng.integers(0, 3)))
        opts = api.make_opts(n, td, c=c, max_iters=iters, flow=flow, damping=damping, eta=eta)
        u = torch.ones(n, dtype=td, device="cuda"); v = torch.ones(n, dtype=td, device="cuda")
        api.fsk_sinkhorn_dense(opts, full[:, :n], dev(a), dev(b), u, v, api.alloc_workspace(opts))
        torch.cuda.synchronize()
        if damping == api.FSK_DAMP_NONE:
            uo, vo = orc.sinkhorn_dense(K, a, b, iters)
        else:
            uo, vo = orc.sinkhorn_dense_damped(K, a, b, iters, eta, damping == api.FSK_DAMP_GEOMETRIC)
        what = (seed, case, n, np.dtype(dtype).name, flow, c, damping, iters)
        assert relerr(u.cpu().numpy(), uo) <= tol and relerr(v.cpu().numpy(), vo) <= tol, what
        assert bool(torch.isnan(full[:, n:]).all()), what          # the padding columns are never written


@pytest.mark.parametrize("seed", [21, 22])
def test_random_multitarget_problems(orc, seed):
    rng = np.random.default_rng(seed)
    rng_damp = np.random.default_rng(seed + 1000)
    for case in range(20):
        dtype, td, tol = _pick(rng)
        n = int(rng.choice([rng.integers(1, 100), rng.integers(100, 1500), rng.integers(1500, 3000)]))
        m = int(rng.choice([1, rng.integers(1, 65), rng.integers(65, 300)]))
        iters = int(rng.integers(1, 5))
        x = rng.uniform(size=(n, 2)); y = rng.uniform(size=(n, 2))
        K64, _ = orc.gibbs_from_points(x, y, float(rng.uniform(0.2, 1.0)), False)
        K = np.ascontiguousarray(K64.astype(dtype))
        A = rng.exponential(size=(n, m)); A = np.ascontiguousarray((A / A.sum(0)).astype(dtype))
        B = rng.exponential(size=(n, m)); B = np.ascontiguousarray((B / B.sum(0)).astype(dtype))
        full = _padded(K, td, int(rng.integers(0, 2)))
        damping = int(rng_damp.choice([api.FSK_DAMP_NONE, api.FSK_DAMP_ARITHMETIC, api.FSK_DAMP_GEOMETRIC]))
        eta = float(rng_damp.uniform(0.2, 1.0))
        opts = api.make_opts(n, td, m=m, max_iters=iters, damping=damping, eta=eta)
        ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
        if dtype == np.float32 and damping == api.FSK_DAMP_NONE and rng.random() < 0.25:
            ws = ws[: ws.numel() - n * n * 4]                      # no room for K^T: the direct row kernel
        U = torch.ones(n, m, dtype=td, device="cuda"); V = torch.ones(n, m, dtype=td, device="cuda")
        api.fsk_sinkhorn_batched(opts, full[:, :n], dev(A), dev(B), U, V, ws)
        torch.cuda.synchronize()
        if damping == api.FSK_DAMP_NONE:
            Uo, Vo = orc.sinkhorn_batched(K, A, B, iters)
        else:
            ones = np.ones((n, m))
            Uo, Vo = orc.sinkhorn_batched_damped(K, A, B, iters, eta, damping == api.FSK_DAMP_GEOMETRIC, ones, ones)
        what = (seed, case, n, m, np.dtype(dtype).name, iters, damping, eta)
        assert relerr(U.cpu().numpy(), Uo) <= tol and relerr(V.cpu().numpy(), Vo) <= tol, what


@pytest.mark.parametrize("seed", [31, 32])
def test_random_log_domain_problems(orc, seed):
    rng = np.random.default_rng(seed)
    for case in range(20):
        dtype, td, tol = _pick(rng)
        n = int(rng.choice([rng.integers(1, 100), rng.integers(100, 1500), rng.integers(1500, 3000)]))
        d = int(rng.choice([rng.integers(1, 33), rng.integers(33, 80)], p=[0.8, 0.2]))
        iters = int(rng.integers(1, 6))
        eps = float(rng.uniform(0.01, 0.1)) * d
        x = rng.uniform(size=(n, d)).astype(np.float32); y = rng.uniform(size=(n, d)).astype(np.float32)
        a = rng.uniform(0.5, 1.5, n); a = (a / a.sum()).astype(np.float32)
        b = rng.uniform(0.5, 1.5, n); b = (b / b.sum()).astype(np.float32)
        opts = api.make_opts(n, td, max_iters=iters)
        f = torch.zeros(n, dtype=td, device="cuda"); g = torch.zeros(n, dtype=td, device="cuda")
        api.fsk_sinkhorn_log_points(opts, dev(x.astype(dtype)), dev(y.astype(dtype)), eps, dev(a.astype(dtype)),
                                    dev(b.astype(dtype)), f, g, api.alloc_workspace(opts, api.FSK_MODE_LOG, d))
        torch.cuda.synchronize()
        fo, go, _, _ = orc.sinkhorn_log_points(x, y, eps, a, b, iters)
        what = (seed, case, n, d, np.dtype(dtype).name, iters)
        assert np.max(np.abs(f.cpu().numpy() - fo)) / eps <= tol, what
        assert np.max(np.abs(g.cpu().numpy() - go)) / eps <= tol, what


@pytest.mark.parametrize("seed", [41, 42])
def test_random_tolerance_mode_problems(orc, seed):
    """Stop rules (either norm, any poll period) of the dense flows, the multitarget call and the
    log domain: stop iteration against the oracle's rule (exact in fp64, within one poll in fp32)
    and the reported error against the oracle's evaluation of the handed-back state."""
    rng = np.random.default_rng(seed)
    cap = 600
    for case in range(45):
        dtype = np.float32 if rng.random() < 0.4 else np.float64
        td = torch.float32 if dtype == np.float32 else torch.float64
        l2 = bool(rng.random() < 0.5)
        norm = api.FSK_NORM_L2 if l2 else api.FSK_NORM_L1
        ce = int(rng.integers(1, 6))
        tol = float(10 ** rng.uniform(-9, -6)) if dtype == np.float64 else float(10 ** rng.uniform(-5.3, -4))
        kind = int(rng.integers(0, 3))
        n = int(rng.choice([rng.integers(2, 100), rng.integers(100, 700)]))
        x = rng.uniform(size=(n, 2)); y = rng.uniform(size=(n, 2))
        K64, _ = orc.gibbs_from_points(x, y, float(rng.uniform(0.2, 0.6)), False)
        K = np.ascontiguousarray(K64.astype(dtype))
        Kd = _padded(K, td, 0)[:, :n]
        which = 1 if l2 else 0
        if kind == 0:      # dense flows
            flow = int(rng.choice([api.FSK_FLOW_FUSED, api.FSK_FLOW_TWO_PASS, api.FSK_FLOW_PAPER, api.FSK_FLOW_RESIDENT]))
            if flow == api.FSK_FLOW_RESIDENT and n > (512 if dtype == np.float64 else 1024):
                flow = api.FSK_FLOW_FUSED
            c = int(rng.choice([c for c in (1, 2, 4, 8) if n % c == 0]))
            a = rng.uniform(0.5, 1.5, n) ** 2; a = (a / a.sum()).astype(dtype)
            b = rng.uniform(0.5, 1.5, n) ** 2; b = (b / b.sum()).astype(dtype)
            _, _, done_o, err_o = orc.sinkhorn_dense_tol(K, a, b, cap, tol, check_every=ce, l2=l2)
            opts = api.make_opts(n, td, c=c, max_iters=cap, tol=tol, check_every=ce, flow=flow, err_norm=norm)
            u = torch.ones(n, dtype=td, device="cuda"); v = torch.ones(n, dtype=td, device="cuda")
            done, err = api.fsk_sinkhorn_dense(opts, Kd, dev(a), dev(b), u, v, api.alloc_workspace(opts))
            state = orc.marginal_error(K, a, u.cpu().numpy(), v.cpu().numpy())[which]
            what = ("dense", seed, case, n, np.dtype(dtype).name, flow, c, ce, l2, tol)
        elif kind == 1:    # multitarget
            m = int(rng.choice([1, rng.integers(2, 65), rng.integers(65, 140)]))
            A = rng.uniform(0.5, 1.5, (n, m)) ** 2; A = np.ascontiguousarray((A / A.sum(0)).astype(dtype))
            B = rng.uniform(0.5, 1.5, (n, m)) ** 2; B = np.ascontiguousarray((B / B.sum(0)).astype(dtype))
            _, _, done_o, err_o = orc.sinkhorn_batched_tol(K, A, B, cap, tol, ce, l2=l2)
            opts = api.make_opts(n, td, m=m, max_iters=cap, tol=tol, check_every=ce, err_norm=norm)
            U = torch.ones(n, m, dtype=td, device="cuda"); V = torch.ones(n, m, dtype=td, device="cuda")
            done, err = api.fsk_sinkhorn_batched_tol(opts, Kd, dev(A), dev(B), U, V,
                                                     api.alloc_workspace(opts, api.FSK_MODE_BATCHED))
            Un, Vn = U.cpu().numpy(), V.cpu().numpy()
            state = max(orc.marginal_error(K, A[:, k], Un[:, k], Vn[:, k])[which] for k in range(m))
            what = ("multitarget", seed, case, n, m, np.dtype(dtype).name, ce, l2, tol)
        else:              # log domain
            d = int(rng.integers(1, 20))
            xl = rng.uniform(size=(n, d)).astype(np.float32); yl = rng.uniform(size=(n, d)).astype(np.float32)
            eps = float(rng.uniform(0.05, 0.2)) * d
            a = rng.uniform(0.5, 1.5, n); a = (a / a.sum()).astype(np.float32)
            b = rng.uniform(0.5, 1.5, n); b = (b / b.sum()).astype(np.float32)
            _, _, done_o, err_o = orc.sinkhorn_log_points(xl, yl, eps, a, b, cap, tol=tol, check_every=ce, l2=l2)
            opts = api.make_opts(n, td, max_iters=cap, tol=tol, check_every=ce, err_norm=norm)
            f = torch.zeros(n, dtype=td, device="cuda"); g = torch.zeros(n, dtype=td, device="cuda")
            done, err = api.fsk_sinkhorn_log_points(opts, dev(xl.astype(dtype)), dev(yl.astype(dtype)), eps,
                                                    dev(a.astype(dtype)), dev(b.astype(dtype)), f, g,
                                                    api.alloc_workspace(opts, api.FSK_MODE_LOG, d))
            rows = orc.log_row_marginal_points(xl, f.double().cpu().numpy(), yl, g.double().cpu().numpy(), eps)
            state = float(np.linalg.norm(rows - a) if l2 else np.abs(rows - a).sum())
            what = ("log", seed, case, n, d, np.dtype(dtype).name, ce, l2, tol)
        if dtype == np.float64:
            assert done == done_o, what
            assert abs(err - err_o) <= 1e-3 * err_o + 1e-13 and abs(err - state) <= 1e-3 * state + 1e-13, what
        else:              # fp32 sums may cross the threshold one poll earlier or later
            assert abs(done - done_o) <= ce and abs(err - state) <= 0.2 * state + 2e-6, what
