"""GPU parity of the log-domain path (cost on the fly from point clouds) against the oracle.

Bar: |f - f_oracle| / eps and |g - g_oracle| / eps <= 1e-4 (this is the relative error of
u = exp(f/eps), v = exp(g/eps), which themselves overflow fp32), and relative error of the
row / column marginals <= 1e-4, at fixed iteration counts.  Stop iterations are compared
only up to one polling interval: the GPU evaluates exponentials in fp32.
"""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev

pytestmark = pytest.mark.gpu


def run_log(x, y, a, b, eps, iters, tol=0.0, check_every=1, f0=None, g0=None, dtype=np.float32,
            damping=api.FSK_DAMP_NONE, eta=1.0):
    n, d = x.shape
    td = torch.float64 if dtype == np.float64 else torch.float32
    opts = api.make_opts(n, td, max_iters=iters, tol=tol, check_every=check_every, damping=damping, eta=eta)
    ws = api.alloc_workspace(opts, api.FSK_MODE_LOG, d)
    f = torch.zeros(n, dtype=td, device="cuda") if f0 is None else dev(f0.astype(dtype))
    g = torch.zeros(n, dtype=td, device="cuda") if g0 is None else dev(g0.astype(dtype))
    cast = lambda t: dev(np.ascontiguousarray(t.astype(dtype)))
    done, err = api.fsk_sinkhorn_log_points(opts, cast(x), cast(y), eps, cast(a), cast(b), f, g, ws)
    torch.cuda.synchronize()
    return f.cpu().numpy().astype(np.float64), g.cpu().numpy().astype(np.float64), done, err


def check_potentials(orc, x, y, a, b, eps, f, g, fo, go, tol=1e-4):
    assert np.max(np.abs(f - fo)) / eps <= tol and np.max(np.abs(g - go)) / eps <= tol
    rows = orc.log_row_marginal_points(x, f, y, g, eps)
    rows_o = orc.log_row_marginal_points(x, fo, y, go, eps)
    assert np.max(np.abs(rows - rows_o) / rows_o) <= tol
    cols = orc.log_row_marginal_points(y, g, x, f, eps)      # column marginal: roles swapped
    assert np.max(np.abs(cols - b.astype(np.float64)) / b) <= tol   # exact after a g-update


@pytest.mark.parametrize("n", [1500, 4096])
def test_cfg4_law_fixed_iterations(orc, n):
    w = workloads.make(4, n=n)
    for iters in (1, 10, 100):
        fo, go, _, _ = orc.sinkhorn_log_points(w.x, w.y, w.eps, w.a, w.b, iters)
        f, g, done, _ = run_log(w.x, w.y, w.a, w.b, w.eps, iters)
        assert done == iters
        check_potentials(orc, w.x, w.y, w.a, w.b, w.eps, f, g, fo, go)


@pytest.mark.parametrize("n,d", [(1, 16), (2, 3), (3, 1), (65, 2), (257, 5), (513, 8), (700, 16),
                                 (300, 20), (300, 32), (400, 10), (333, 12), (300, 17), (515, 24),
                                 (300, 25)])
def test_ragged_sizes_and_dimensions(orc, n, d):
    rng = np.random.default_rng(100 * n + d)
    x = rng.uniform(size=(n, d)).astype(np.float32); y = rng.uniform(size=(n, d)).astype(np.float32)
    a = rng.uniform(0.5, 1.5, n); a = (a / a.sum()).astype(np.float32)
    b = rng.uniform(0.5, 1.5, n); b = (b / b.sum()).astype(np.float32)
    eps = 0.02 * d
    fo, go, _, _ = orc.sinkhorn_log_points(x, y, eps, a, b, 12)
    f, g, _, _ = run_log(x, y, a, b, eps, 12)
    check_potentials(orc, x, y, a, b, eps, f, g, fo, go)


@pytest.mark.parametrize("n,d,dtype,tol", [(1, 33, np.float32, 1e-4), (70, 33, np.float32, 1e-4),
                                           (300, 40, np.float32, 1e-4), (521, 64, np.float32, 1e-4),
                                           (1030, 100, np.float32, 1e-4), (300, 257, np.float32, 1e-4),
                                           (257, 50, np.float64, 1e-10), (600, 64, np.float64, 1e-10)])
def test_dimensions_above_32_take_the_generic_kernel(orc, n, d, dtype, tol):
    rng = np.random.default_rng(7000 + 10 * n + d)
    x = rng.uniform(size=(n, d)).astype(np.float32); y = rng.uniform(size=(n, d)).astype(np.float32)
    a = rng.uniform(0.5, 1.5, n); a = (a / a.sum()).astype(np.float32)
    b = rng.uniform(0.5, 1.5, n); b = (b / b.sum()).astype(np.float32)
    eps = 0.02 * d
    fo, go, _, _ = orc.sinkhorn_log_points(x, y, eps, a, b, 12)
    f, g, _, _ = run_log(x, y, a, b, eps, 12, dtype=dtype)
    check_potentials(orc, x, y, a, b, eps, f, g, fo, go, tol)


def test_dimension_outside_the_supported_range_is_refused():
    v = torch.full((8,), 0.125, device="cuda")
    opts = api.make_opts(8, torch.float32, max_iters=1)
    x = torch.zeros(8, 4097, device="cuda")
    assert api.fsk_workspace_bytes(opts, api.FSK_MODE_LOG, 4097) == 0
    with pytest.raises(api.FskError) as e:
        api.fsk_sinkhorn_log_points(opts, x, x, 0.1, v, v, v.clone(), v.clone(),
                                    torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert e.value.status == api.FSK_EUNSUPPORTED


def test_tolerance_mode_and_cap(orc):
    w = workloads.make(4, n=900)
    eps = 0.05
    fo, go, done_o, err_o = orc.sinkhorn_log_points(w.x, w.y, eps, w.a, w.b, 3000, tol=1e-5, check_every=5)
    f, g, done, err = run_log(w.x, w.y, w.a, w.b, eps, 3000, tol=1e-5, check_every=5)
    assert done % 5 == 0 and abs(done - done_o) <= 5 and err < 1e-5
    fo2, go2, _, _ = orc.sinkhorn_log_points(w.x, w.y, eps, w.a, w.b, done)
    check_potentials(orc, w.x, w.y, w.a, w.b, eps, f, g, fo2, go2)
    rows = orc.log_row_marginal_points(w.x, f, w.y, g, eps)
    assert err == pytest.approx(np.abs(rows - w.a).sum(), rel=0.05, abs=2e-7)
    # the state handed back is exactly the one after `done` iterations (the iteration whose
    # f-update revealed its error has been undone), also when every iteration is polled
    ff, gf, _, _ = run_log(w.x, w.y, w.a, w.b, eps, done)
    assert np.array_equal(f, ff) and np.array_equal(g, gf)
    f1, g1, done1, err1 = run_log(w.x, w.y, w.a, w.b, eps, 3000, tol=1e-5, check_every=1)
    assert done1 <= done and done - done1 < 5 and err1 < 1e-5
    ff, gf, _, _ = run_log(w.x, w.y, w.a, w.b, eps, done1)
    assert np.array_equal(f1, ff) and np.array_equal(g1, gf)
    f, g, done, err = run_log(w.x, w.y, w.a, w.b, eps, 9, tol=1e-30, check_every=4)
    assert done == 9 and err > 0


def test_warm_start_continues_the_run(orc):
    w = workloads.make(4, n=777)
    fo, go, _, _ = orc.sinkhorn_log_points(w.x, w.y, w.eps, w.a, w.b, 40)
    f1, g1, _, _ = run_log(w.x, w.y, w.a, w.b, w.eps, 15)
    f2, g2, _, _ = run_log(w.x, w.y, w.a, w.b, w.eps, 25, f0=f1, g0=g1)
    check_potentials(orc, w.x, w.y, w.a, w.b, w.eps, f2, g2, fo, go)
    fa, ga, _, _ = run_log(w.x, w.y, w.a, w.b, w.eps, 40)
    fb, gb, _, _ = run_log(w.x, w.y, w.a, w.b, w.eps, 40)
    assert np.array_equal(fa, fb) and np.array_equal(ga, gb)     # deterministic


def test_small_eps_where_the_dense_kernel_underflows(orc):
    rng = np.random.default_rng(7)
    n, d, eps = 600, 16, 0.002
    x = rng.uniform(size=(n, d)).astype(np.float32); y = rng.uniform(size=(n, d)).astype(np.float32)
    a = np.full(n, 1.0 / n, dtype=np.float32); b = a.copy()
    fo, go, _, _ = orc.sinkhorn_log_points(x, y, eps, a, b, 20)
    f, g, _, _ = run_log(x, y, a, b, eps, 20)
    assert np.isfinite(f).all() and np.isfinite(g).all()
    check_potentials(orc, x, y, a, b, eps, f, g, fo, go)


@pytest.mark.parametrize("n,d", [(1500, 16), (257, 5), (64, 32), (3, 2)])
def test_fp64_interface(orc, n, d):
    """FSK_F64: potentials, exponentials and sums in fp64; the bar is 1e-10."""
    rng = np.random.default_rng(7 * n + d)
    x = rng.uniform(size=(n, d)); y = rng.uniform(size=(n, d))
    a = rng.uniform(0.5, 1.5, n); a /= a.sum()
    b = rng.uniform(0.5, 1.5, n); b /= b.sum()
    eps = 0.01 * d
    for iters in (1, 25):
        fo, go, _, _ = orc.sinkhorn_log_points(x, y, eps, a, b, iters)
        f, g, done, _ = run_log(x, y, a, b, eps, iters, dtype=np.float64)
        assert done == iters
        check_potentials(orc, x, y, a, b, eps, f, g, fo, go, tol=1e-10)


def test_fp64_tolerance_mode_reaches_what_fp32_cannot(orc):
    w = workloads.make(4, n=512)
    x, y, a, b = (t.astype(np.float64) for t in (w.x, w.y, w.a, w.b))
    eps = 0.5
    fo, go, done_o, err_o = orc.sinkhorn_log_points(x, y, eps, a, b, 1000, tol=1e-11, check_every=10)
    f, g, done, err = run_log(x, y, a, b, eps, 1000, tol=1e-11, check_every=10, dtype=np.float64)
    assert done == done_o and done < 1000 and err < 1e-11
    assert np.max(np.abs(f - fo)) / eps <= 1e-10 and np.max(np.abs(g - go)) / eps <= 1e-10


@pytest.mark.parametrize("dtype,tol", [(np.float32, 1e-4), (np.float64, 1e-10)])
@pytest.mark.parametrize("damping,geometric", [(api.FSK_DAMP_ARITHMETIC, False), (api.FSK_DAMP_GEOMETRIC, True)])
def test_relaxed_updates_in_the_log_domain(orc, dtype, tol, damping, geometric):
    """Sec. 3.3 on the potentials, at an eps small enough that exp(f / eps) overflows fp64."""
    rng = np.random.default_rng(55)
    n, d = 700, 6
    x = rng.uniform(size=(n, d)).astype(np.float32); y = rng.uniform(size=(n, d)).astype(np.float32)
    a = rng.uniform(0.5, 1.5, n); a = (a / a.sum()).astype(np.float32)
    b = rng.uniform(0.5, 1.5, n); b = (b / b.sum()).astype(np.float32)
    for eps, eta in ((0.05, 0.6), (0.0005, 0.35)):
        fo, go = orc.sinkhorn_log_points_damped(x, y, eps, a, b, 15, eta, geometric)
        f, g, done, _ = run_log(x, y, a, b, eps, 15, dtype=dtype, damping=damping, eta=eta)
        assert done == 15
        assert np.max(np.abs(f - fo)) / eps <= tol and np.max(np.abs(g - go)) / eps <= tol
