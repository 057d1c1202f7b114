"""GPU parity of the dense hot path against the CPU oracle, through the C ABI.

Bars (written here, from the benchmark spec): max relative error on u, v and both marginals
<= 1e-10 in fp64 and <= 1e-4 in fp32, on the same seeded inputs.  The GPU is always fed the
kernel matrix the oracle's own setup produced (rounded to the storage type), so the comparison
isolates the iteration; the GPU setup kernels are checked separately.
"""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import TOL, dev, relerr, run_dense, tdtype

pytestmark = pytest.mark.gpu

FLOWS = [api.FSK_FLOW_FUSED, api.FSK_FLOW_TWO_PASS, api.FSK_FLOW_PAPER]


def oracle_kernel(orc, w):
    K, _ = orc.gibbs_from_points(w.x, w.y, w.eps, w.normalise_by_max)
    return np.ascontiguousarray(K.astype(w.dtype))


def check_against_oracle(orc, K, a, b, u, v, iters, tol, c=1):
    uo, vo = orc.sinkhorn_dense(K, a, b, iters)
    assert relerr(u, uo) <= tol and relerr(v, vo) <= tol
    # marginals of the GPU scalings, evaluated by the oracle, against the oracle's own
    assert relerr(orc.row_marginal(K, u, v), orc.row_marginal(K, uo, vo)) <= tol
    assert relerr(orc.col_marginal(K, u, v), b.astype(np.float64)) <= tol


@pytest.mark.parametrize("flow", FLOWS)
def test_cfg1_n512_fp64_full_run(orc, flow):
    w = workloads.make(1)
    K = oracle_kernel(orc, w)
    u, v, done, _ = run_dense(K, w.a, w.b, w.iters, flow=flow)
    assert done == 200
    check_against_oracle(orc, K, w.a, w.b, u, v, 200, TOL[w.dtype])


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("n", [1, 2, 3, 5, 67, 130, 515, 1000, 2049, 2050, 4101])
def test_ragged_sizes_all_flows(orc, n, dtype):
    """Sizes that are not multiples of the pack width, the tile or the strip, incl. n = 1."""
    rng = np.random.default_rng(1000 + n)
    x = rng.uniform(size=(n, 3)); y = rng.uniform(size=(n, 3)) + 0.2
    a = rng.uniform(0.5, 1.5, n); a /= a.sum()
    b = rng.uniform(0.5, 1.5, n); b /= b.sum()
    K64, _ = orc.gibbs_from_points(x, y, 0.5, True)
    K = np.ascontiguousarray(K64.astype(dtype)); a = a.astype(dtype); b = b.astype(dtype)
    pack = 16 // np.dtype(dtype).itemsize
    ld = (n + pack - 1) // pack * pack + 3 * pack      # padded rows, NaN in the padding
    for flow in FLOWS:
        u, v, done, _ = run_dense(K, a, b, 7, flow=flow, ld=ld)
        check_against_oracle(orc, K, a, b, u, v, 7, TOL[np.dtype(dtype)])


def test_cfg2_n8192_fp32_full_run(orc):
    w = workloads.make(2)
    K = oracle_kernel(orc, w)
    uo, vo = orc.sinkhorn_dense(K, w.a, w.b, w.iters)
    for flow in FLOWS:
        u, v, done, _ = run_dense(K, w.a, w.b, w.iters, flow=flow)
        assert done == 500
        assert relerr(u, uo) <= 1e-4 and relerr(v, vo) <= 1e-4, flow
        assert relerr(orc.col_marginal(K, u, v), w.b) <= 1e-4
        assert relerr(orc.row_marginal(K, u, v), orc.row_marginal(K, uo, vo)) <= 1e-4


@pytest.mark.parametrize("c", [2, 4, 8])
def test_blocked_equals_centralised_cfg3_law(orc, c):
    """Proposition 1 on the GPU: c row blocks give the centralised iterates, bit for bit in every
    flow.  Two-pass and Algorithm-1 flows sum every column over the same fixed row strips whatever
    c is; the fused flow cuts every block into strips whose height depends on n alone (here
    2048 / 16 = 128 rows, and 2048 / c is a multiple of it), so its partial sums are the same too."""
    w = workloads.make(3, n=2048)
    K = oracle_kernel(orc, w)
    uo, vo = orc.sinkhorn_blocked(K, w.a, w.b, 60, c, 1)
    u1, v1, _, _ = run_dense(K, w.a, w.b, 60, flow=api.FSK_FLOW_TWO_PASS, c=1)
    for flow in (api.FSK_FLOW_TWO_PASS, api.FSK_FLOW_PAPER):
        u, v, _, _ = run_dense(K, w.a, w.b, 60, flow=flow, c=c)
        assert np.array_equal(u, u1) and np.array_equal(v, v1)
    uf1, vf1, _, _ = run_dense(K, w.a, w.b, 60, flow=api.FSK_FLOW_FUSED, c=1)
    uf, vf, _, _ = run_dense(K, w.a, w.b, 60, flow=api.FSK_FLOW_FUSED, c=c)
    assert np.array_equal(uf, uf1) and np.array_equal(vf, vf1)
    for u, v in ((u1, v1), (uf, vf)):
        assert relerr(u, uo) <= 1e-4 and relerr(v, vo) <= 1e-4


@pytest.mark.parametrize("n,dtype,cs,aligned", [
    (8192, np.float32, (2, 8, 64, 256), True),      # 256 strips of 32 rows: every c | 256 is aligned
    (4096, np.float64, (2, 16), True),              # 16 strips of 256 rows
    (4096, np.float32, (32,), False),               # blocks of 128 rows are shorter than a strip
    (3000, np.float32, (3, 5), False),              # 1000 and 600 rows are not multiples of 192
    (9000, np.float64, (4, 8), False),              # 36-row strips do not divide 2250 or 1125
])
def test_fused_flow_is_bitwise_independent_of_c_when_blocks_are_whole_strips(orc, n, dtype, cs, aligned):
    """The fused flow's strips: when the block height is a multiple of the strip height that
    c = 1 gets, every c gives the same bits; otherwise the strips differ and the iterates agree
    to rounding only (and with the oracle at the usual bar either way)."""
    w = workloads.make(3, n=n)
    K = oracle_kernel(orc, w).astype(dtype)
    a, b = w.a.astype(dtype), w.b.astype(dtype)
    iters = 12
    u1, v1, _, _ = run_dense(K, a, b, iters, flow=api.FSK_FLOW_FUSED, c=1)
    uo, vo = orc.sinkhorn_dense(K, a, b, iters)
    for c in cs:
        u, v, _, _ = run_dense(K, a, b, iters, flow=api.FSK_FLOW_FUSED, c=c)
        if aligned:
            assert np.array_equal(u, u1) and np.array_equal(v, v1), c
        else:
            assert relerr(u, u1) <= 100 * np.finfo(dtype).eps and relerr(v, v1) <= 100 * np.finfo(dtype).eps
        assert relerr(u, uo) <= TOL[np.dtype(dtype)] and relerr(v, vo) <= TOL[np.dtype(dtype)]


def test_c_must_divide_n():
    opts = api.make_opts(100, torch.float32, c=3, max_iters=1)
    t = torch.ones(100, 100, device="cuda")
    vec = torch.ones(100, device="cuda")
    with pytest.raises(api.FskError) as e:
        api.fsk_sinkhorn_dense(opts, t, vec, vec, vec.clone(), vec.clone(), torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert e.value.status == api.FSK_EDIV


def test_runs_are_bitwise_reproducible_and_resumable(orc):
    w = workloads.make(2, n=1536)
    K = oracle_kernel(orc, w)
    for flow in FLOWS:
        u, v, _, _ = run_dense(K, w.a, w.b, 40, flow=flow, c=4)
        u2, v2, _, _ = run_dense(K, w.a, w.b, 40, flow=flow, c=4)
        assert np.array_equal(u, u2) and np.array_equal(v, v2)
        ua, va, _, _ = run_dense(K, w.a, w.b, 15, flow=flow, c=4)
        ub, vb, _, _ = run_dense(K, w.a, w.b, 25, flow=flow, c=4, u0=ua, v0=va)
        assert np.array_equal(u, ub) and np.array_equal(v, vb)


def test_tolerance_mode(orc):
    w = workloads.make(1, n=300)
    K = oracle_kernel(orc, w)
    uo, vo, done_o, err_o = orc.sinkhorn_dense_tol(K, w.a, w.b, 5000, 1e-9, check_every=7)
    for flow in FLOWS:
        u, v, done, err = run_dense(K, w.a, w.b, 5000, flow=flow, tol=1e-9, check_every=7)
        assert done == done_o and done % 7 == 0
        assert err < 1e-9 and err == pytest.approx(err_o, rel=1e-3)
        assert relerr(u, uo) <= 1e-10 and relerr(v, vo) <= 1e-10
        # the state handed back is exactly the state after `done` iterations: the iteration whose
        # u-update revealed the error of that state has been undone
        uf, vf, _, _ = run_dense(K, w.a, w.b, done, flow=flow)
        assert np.array_equal(u, uf) and np.array_equal(v, vf)
    # the cap binds and the last iteration is polled
    u, v, done, err = run_dense(K, w.a, w.b, 10, tol=1e-300, check_every=4)
    assert done == 10 and err > 0
    # polling every iteration, blocks, damping: same stop as the oracle's rule
    w3 = workloads.make(3, n=512)
    K3, _ = orc.gibbs_from_points_f32(w3.x, w3.y, w3.eps, True)
    uo, vo, done_o, err_o = orc.sinkhorn_dense_tol(K3, w3.a, w3.b, 3000, 1e-4, check_every=1)
    for flow, c in ((api.FSK_FLOW_FUSED, 8), (api.FSK_FLOW_PAPER, 4), (api.FSK_FLOW_TWO_PASS, 1)):
        u, v, done, err = run_dense(K3, w3.a, w3.b, 3000, flow=flow, c=c, tol=1e-4, check_every=1)
        assert abs(done - done_o) <= 1 and err < 1e-4
        uf, vf, _, _ = run_dense(K3, w3.a, w3.b, done, flow=flow, c=c)
        assert np.array_equal(u, uf) and np.array_equal(v, vf)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_damped_updates(orc, dtype):
    w = workloads.make(2, n=777)
    K64, _ = orc.gibbs_from_points(w.x, w.y, 0.3, True)
    K = np.ascontiguousarray(K64.astype(dtype)); a = w.a.astype(dtype); b = w.b.astype(dtype)
    for damping, geo in ((api.FSK_DAMP_ARITHMETIC, False), (api.FSK_DAMP_GEOMETRIC, True)):
        uo, vo = orc.sinkhorn_dense_damped(K, a, b, 30, 0.5, geo)
        for flow in FLOWS:
            u, v, _, _ = run_dense(K, a, b, 30, flow=flow, damping=damping, eta=0.5)
            assert relerr(u, uo) <= TOL[np.dtype(dtype)] and relerr(v, vo) <= TOL[np.dtype(dtype)]


def test_marginals_entry_point(orc):
    w = workloads.make(2, n=1100)
    K = oracle_kernel(orc, w)
    u, v, _, _ = run_dense(K, w.a, w.b, 12)
    opts = api.make_opts(1100, torch.float32)
    ws = api.alloc_workspace(opts)
    rm = torch.empty(1100, device="cuda"); cm = torch.empty(1100, device="cuda")
    err = api.fsk_marginals(opts, dev(K), dev(w.a), dev(u), dev(v), rm, cm, ws, want_err=True)
    torch.cuda.synchronize()
    assert relerr(rm.cpu().numpy(), orc.row_marginal(K, u, v)) <= 1e-5
    assert relerr(cm.cpu().numpy(), orc.col_marginal(K, u, v)) <= 1e-5
    assert err == pytest.approx(orc.marginal_error(K, w.a, u, v)[0], rel=1e-3, abs=1e-7)
    # the paper's own metric, ||P1 - a||_2, from the same row pass (no marginals asked for)
    e1, e2 = api.fsk_marginals(opts, dev(K), dev(w.a), dev(u), dev(v), None, None, ws, want_l2=True)
    o1, o2 = orc.marginal_error(K, w.a, u, v)
    assert e1 == err and e2 == pytest.approx(o2, rel=1e-3, abs=1e-9) and e2 <= e1
    # fp64 on a state that is not converged: both norms to rounding
    K64 = K.astype(np.float64); u64 = np.linspace(0.5, 2.0, 1100) / 1100; v64 = np.linspace(1.5, 0.3, 1100) / 1100
    opts64 = api.make_opts(1100, torch.float64)
    a64 = w.a.astype(np.float64)
    e1, e2 = api.fsk_marginals(opts64, dev(K64), dev(a64), dev(u64), dev(v64), None, None,
                               api.alloc_workspace(opts64), want_l2=True)
    o1, o2 = orc.marginal_error(K64, a64, u64, v64)
    assert e1 == pytest.approx(o1, rel=1e-12) and e2 == pytest.approx(o2, rel=1e-12)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_one_workers_share(orc, dtype):
    """The per-worker operations of Sec. 3.1 on a real slab: rows [row0, row0+rows) only."""
    n, row0, rows = 1500, 375, 375
    w = workloads.make(3, n=n)
    K64, _ = orc.gibbs_from_points(w.x, w.y, w.eps, True)
    K = np.ascontiguousarray(K64.astype(dtype)); a = w.a.astype(dtype)
    rng = np.random.default_rng(5)
    v = rng.uniform(0.5, 2.0, n).astype(dtype)
    slab = dev(K[row0:row0 + rows])
    td = tdtype(dtype)
    opts = api.make_opts(n, td)
    ws = api.alloc_workspace(opts)
    u_slab = torch.empty(rows, dtype=td, device="cuda")
    api.fsk_block_rowpass(opts, slab, row0, dev(a[row0:row0 + rows]), dev(v), u_slab)
    u_ref = a[row0:row0 + rows].astype(np.float64) / orc.row_products(K, v, row0, row0 + rows)
    tol = TOL[np.dtype(dtype)]
    assert relerr(u_slab.cpu().numpy(), u_ref) <= tol
    s = torch.empty(n, dtype=td, device="cuda")
    api.fsk_block_colpartial(opts, slab, row0, u_slab, s, ws)
    u_full = np.zeros(n); u_full[row0:row0 + rows] = u_slab.cpu().numpy()
    s_ref = orc.col_products(K, u_full, row0, row0 + rows)
    assert relerr(s.cpu().numpy(), s_ref) <= tol
    u2 = torch.empty(rows, dtype=td, device="cuda"); s2 = torch.empty(n, dtype=td, device="cuda")
    api.fsk_block_fused(opts, slab, row0, dev(a[row0:row0 + rows]), dev(v), u2, s2, ws)
    torch.cuda.synchronize()
    assert relerr(u2.cpu().numpy(), u_ref) <= tol
    u_full[row0:row0 + rows] = u2.cpu().numpy()
    assert relerr(s2.cpu().numpy(), orc.col_products(K, u_full, row0, row0 + rows)) <= tol


@pytest.mark.parametrize("cfg,n", [(1, 512), (2, 1000), (3, 1537), (5, 900)])
def test_setup_kernels_against_oracle(orc, cfg, n):
    """K = exp(-C/eps) from points (with and without the max-normalisation) and from a stored
    cost.  The GPU evaluates in fp64 and rounds once, so fp32 storage may differ from the
    oracle's rounded value by one unit in the last place at most."""
    w = workloads.make(cfg, n=n)
    td = tdtype(w.dtype)
    opts = api.make_opts(n, td)
    ws = api.alloc_workspace(opts, api.FSK_MODE_SETUP, w.d)
    K = torch.empty(n, n, dtype=td, device="cuda")
    cmax = api.fsk_kernel_from_points(opts, dev(w.x), dev(w.y), w.eps, w.normalise_by_max, K, ws,
                                      want_cmax=True)
    K64, cmax_o = orc.gibbs_from_points(w.x, w.y, w.eps, w.normalise_by_max)
    assert cmax == pytest.approx(cmax_o, rel=1e-14)
    ulp = 2.0 ** -23 if w.dtype == np.float32 else 2.0 ** -52 * (1 + cmax_o / w.eps)
    tiny = 2.0 ** -149 if w.dtype == np.float32 else 1e-300      # spacing of subnormal results
    got = K.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - K64) <= 1.01 * ulp * K64 + tiny)
    C = orc.cost_sqeuclid(w.x, w.y).astype(w.dtype)
    K2 = torch.empty(n, n, dtype=td, device="cuda")
    api.fsk_kernel_from_cost(opts, dev(C), w.eps, K2)
    ref = orc.gibbs(C.astype(np.float64), w.eps)
    assert np.all(np.abs(K2.cpu().numpy().astype(np.float64) - ref) <= 1.01 * ulp * ref + tiny)


def test_end_to_end_with_gpu_setup(orc):
    """Setup and iteration both on the GPU against the oracle end to end (cfg 2 law)."""
    w = workloads.make(2, n=2048)
    opts = api.make_opts(2048, torch.float32)
    K = torch.empty(2048, 2048, device="cuda")
    api.fsk_kernel_from_points(opts, dev(w.x), dev(w.y), w.eps, True, K,
                               api.alloc_workspace(opts, api.FSK_MODE_SETUP, w.d))
    u, v, _, _ = run_dense(None, w.a, w.b, 200, K_dev=K)
    K64, _ = orc.gibbs_from_points(w.x, w.y, w.eps, True)
    uo, vo = orc.sinkhorn_dense(K64, w.a, w.b, 200)
    assert relerr(u, uo) <= 1e-4 and relerr(v, vo) <= 1e-4


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_every_pack_count_of_the_fused_kernel(dtype):
    """The fused kernel has one variant per number of 16-byte packs a thread holds of a row (1 to
    16), each with and without masking of the last slot.  For every variant: one-step consistency
    of the second iteration on sampled rows and columns, the definition written out in NumPy fp64
    on slices of the K the GPU holds (row pitch padded with NaN columns where n is ragged)."""
    td = tdtype(dtype)
    es = np.dtype(dtype).itemsize
    pack = 16 // es
    tol = TOL[np.dtype(dtype)]
    rng = np.random.default_rng(99)
    for vpt in range(1, 17):
        for ragged in (0, 5):
            n = 512 * pack * vpt - ragged
            ld = (n + pack - 1) // pack * pack + (pack if ragged else 0)
            x = dev(rng.standard_normal((n, 3)).astype(dtype)); y = dev(rng.standard_normal((n, 3)).astype(dtype))
            a64 = rng.uniform(0.5, 1.5, n); a64 /= a64.sum()
            b64 = rng.uniform(0.5, 1.5, n); b64 /= b64.sum()
            a = dev(a64.astype(dtype)); b = dev(b64.astype(dtype))
            full = torch.full((n, ld), float("nan"), dtype=td, device="cuda")
            K = full[:, :n]
            opts = api.make_opts(n, td, max_iters=1)
            api.fsk_kernel_from_points(opts, x, y, 0.1, True, K, api.alloc_workspace(opts, api.FSK_MODE_SETUP))
            ws = api.alloc_workspace(opts)
            u = torch.ones(n, dtype=td, device="cuda"); v = torch.ones(n, dtype=td, device="cuda")
            api.fsk_sinkhorn_dense(opts, K, a, b, u, v, ws)
            v1 = v.clone()
            api.fsk_sinkhorn_dense(opts, K, a, b, u, v, ws)
            torch.cuda.synchronize()
            idx = np.unique(np.concatenate([[0, n - 1], rng.choice(n, 30, replace=False)]))
            tix = torch.from_numpy(idx).cuda()
            q = K[tix].double().cpu().numpy() @ v1.double().cpu().numpy()
            assert relerr(u[tix].cpu().numpy(), a.double().cpu().numpy()[idx] / q) <= tol, (vpt, ragged)
            r = K[:, tix].double().cpu().numpy().T @ u.double().cpu().numpy()
            assert relerr(v[tix].cpu().numpy(), b.double().cpu().numpy()[idx] / r) <= tol, (vpt, ragged)
            assert bool(torch.isfinite(u).all()) and bool(torch.isfinite(v).all())
            del full, K
