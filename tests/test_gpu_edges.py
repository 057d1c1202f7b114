"""Edge cases of the GPU entry points: zero iterations, the degenerate inputs the method has
(an underflowed kernel row, which makes the scalings non-finite), and the sizes at which the
fused kernel hands over to the two-pass kernels."""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev, relerr, run_dense

pytestmark = pytest.mark.gpu


def test_zero_iterations_leave_the_state_alone(orc):
    n, m = 300, 5
    w = workloads.make(2, n=n)
    K, _ = orc.gibbs_from_points_f32(w.x, w.y, w.eps, True)
    rng = np.random.default_rng(0)
    u0 = rng.uniform(0.5, 2.0, n).astype(np.float32); v0 = rng.uniform(0.5, 2.0, n).astype(np.float32)
    for flow in (api.FSK_FLOW_FUSED, api.FSK_FLOW_TWO_PASS, api.FSK_FLOW_PAPER, api.FSK_FLOW_RESIDENT):
        u, v, done, _ = run_dense(K, w.a, w.b, 0, flow=flow, u0=u0, v0=v0)
        assert done == 0 and np.array_equal(u, u0) and np.array_equal(v, v0)
    # log domain
    w4 = workloads.make(4, n=n)
    opts = api.make_opts(n, torch.float32, max_iters=0)
    ws = api.alloc_workspace(opts, api.FSK_MODE_LOG, w4.d)
    f = dev(u0.copy()); g = dev(v0.copy())
    done, _ = api.fsk_sinkhorn_log_points(opts, dev(w4.x), dev(w4.y), w4.eps, dev(w4.a), dev(w4.b), f, g, ws)
    torch.cuda.synchronize()
    assert done == 0 and np.array_equal(f.cpu().numpy(), u0) and np.array_equal(g.cpu().numpy(), v0)
    # multitarget
    w5 = workloads.make(5, n=n, m=m)
    opts = api.make_opts(n, torch.float32, m=m, max_iters=0)
    ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
    U0 = rng.uniform(0.5, 2.0, (n, m)).astype(np.float32)
    U = dev(U0.copy()); V = dev(U0.copy())
    pad = torch.zeros(n, 304, device="cuda"); pad[:, :n] = dev(K)
    api.fsk_sinkhorn_batched(opts, pad[:, :n], dev(w5.a), dev(w5.b), U, V, ws)
    torch.cuda.synchronize()
    assert np.array_equal(U.cpu().numpy(), U0) and np.array_equal(V.cpu().numpy(), U0)


@pytest.mark.parametrize("flow", [api.FSK_FLOW_FUSED, api.FSK_FLOW_TWO_PASS, api.FSK_FLOW_RESIDENT])
def test_underflowed_kernel_row_is_reported(orc, flow):
    """A row of K that underflowed to zero (the paper assumes K > 0) gives q_i = 0 and an
    infinite scaling: tolerance mode reports it at the first poll instead of iterating on."""
    n = 256
    w = workloads.make(2, n=n)
    K, _ = orc.gibbs_from_points_f32(w.x, w.y, w.eps, True)
    K = K.copy(); K[17, :] = 0.0
    with pytest.raises(api.FskError) as e:
        run_dense(K, w.a, w.b, 20, flow=flow, tol=1e-6, check_every=5)
    assert e.value.status == api.FSK_ENONFINITE
    # fixed-iteration mode does not poll: the non-finite values are simply there to see
    u, v, _, _ = run_dense(K, w.a, w.b, 3, flow=flow)
    assert not np.isfinite(u[17]) or not np.isfinite(v).all()
    # what the refused call leaves in u, v is the polled state itself (5 iterations, the first
    # poll), not the state advanced past it by the update that revealed the error
    opts = api.make_opts(n, torch.float32, max_iters=20, tol=1e-6, check_every=5, flow=flow)
    ud = torch.ones(n, device="cuda"); vd = torch.ones(n, device="cuda")
    with pytest.raises(api.FskError):
        api.fsk_sinkhorn_dense(opts, dev(K), dev(w.a), dev(w.b), ud, vd, api.alloc_workspace(opts))
    torch.cuda.synchronize()
    u5, v5, _, _ = run_dense(K, w.a, w.b, 5, flow=flow)
    assert np.array_equal(ud.cpu().numpy(), u5, equal_nan=True)
    assert np.array_equal(vd.cpu().numpy(), v5, equal_nan=True)


def test_above_the_fused_limit_the_call_falls_back_to_two_passes(orc):
    """n = 32772 fp32 is four columns beyond what a workgroup of the fused kernel can hold:
    FSK_FLOW_FUSED then runs the two-pass kernels, bitwise."""
    w = workloads.make(3, n=32772)
    n = w.n
    K, _ = orc.gibbs_from_points_f32(w.x, w.y, w.eps, True)
    Kd = dev(K); a = dev(w.a); b = dev(w.b)

    def run(flow, iters):
        opts = api.make_opts(n, torch.float32, max_iters=iters, flow=flow)
        ws = api.alloc_workspace(opts)
        u = torch.ones(n, device="cuda"); v = torch.ones(n, device="cuda")
        api.fsk_sinkhorn_dense(opts, Kd, a, b, u, v, ws)
        torch.cuda.synchronize()
        return u, v

    uf, vf = run(api.FSK_FLOW_FUSED, 3)
    ut, vt = run(api.FSK_FLOW_TWO_PASS, 3)
    assert torch.equal(uf, ut) and torch.equal(vf, vt)
    uo, vo = orc.sinkhorn_dense(K, w.a, w.b, 3)
    assert relerr(uf.cpu().numpy(), uo) <= 1e-4 and relerr(vf.cpu().numpy(), vo) <= 1e-4
    with pytest.raises(api.FskError) as e:          # and the per-worker fused call says so
        opts = api.make_opts(n, torch.float32, max_iters=1)
        api.fsk_block_fused(opts, Kd[:4096], 0, a[:4096], torch.ones(n, device="cuda"),
                            torch.empty(4096, device="cuda"), torch.empty(n, device="cuda"),
                            torch.empty(1 << 26, dtype=torch.uint8, device="cuda"))
    assert e.value.status == api.FSK_EUNSUPPORTED


@pytest.mark.parametrize("n,c", [(1024, 1024), (1024, 512), (1536, 384), (600, 300)])
def test_more_blocks_than_compute_units(orc, n, c):
    """c far above the number of compute units (down to one row per block): teams of workgroups
    walk several blocks each; every flow still reproduces the centralised iterates."""
    w = workloads.make(3, n=n)
    K, _ = orc.gibbs_from_points_f32(w.x, w.y, w.eps, True)
    uo, vo = orc.sinkhorn_blocked(K, w.a, w.b, 15, c, 1)
    ref = None
    for flow in (api.FSK_FLOW_FUSED, api.FSK_FLOW_TWO_PASS, api.FSK_FLOW_PAPER):
        u, v, _, _ = run_dense(K, w.a, w.b, 15, flow=flow, c=c)
        assert relerr(u, uo) <= 1e-4 and relerr(v, vo) <= 1e-4
        if flow != api.FSK_FLOW_FUSED:      # the two-pass flows are bitwise independent of c
            u1, v1, _, _ = run_dense(K, w.a, w.b, 15, flow=api.FSK_FLOW_TWO_PASS, c=1)
            assert np.array_equal(u, u1) and np.array_equal(v, v1)


def test_more_than_2_to_31_matrix_entries(orc):
    """n = 46400: K has 2.15e9 entries (8.6 GB in fp32), so every element index beyond 2^31 and
    every byte offset beyond 2^33 is exercised: the setup kernel (sampled entries against the
    oracle's cost and exponential), then two iterations of the two-pass flow and of the blocked
    Algorithm-1 flow against the oracle on the very K the GPU built."""
    n = 46400
    w = workloads.make(3, n=n)
    opts = api.make_opts(n, torch.float32, max_iters=2, flow=api.FSK_FLOW_TWO_PASS)
    Kd = torch.empty(n, n, device="cuda")
    x, y = dev(w.x), dev(w.y)
    cmax = api.fsk_kernel_from_points(opts, x, y, w.eps, True, Kd,
                                      api.alloc_workspace(opts, api.FSK_MODE_SETUP), want_cmax=True)
    K = Kd.cpu().numpy()
    rng = np.random.default_rng(46)
    rows = np.concatenate([[0, n - 1], rng.choice(n, 6, replace=False)])
    C = orc.cost_sqeuclid(w.x[rows].astype(np.float64), w.y.astype(np.float64))
    assert abs(cmax - orc.max_sqeuclid(w.x, w.y)) <= 1e-12 * cmax
    ref = np.exp(-(C / cmax) / w.eps)
    assert relerr(K[rows], ref) <= 4 * np.finfo(np.float32).eps + 20 * 2.0 ** -24

    a, b = dev(w.a), dev(w.b)
    uo, vo = orc.sinkhorn_dense(K, w.a, w.b, 2)
    for flow, c in ((api.FSK_FLOW_TWO_PASS, 1), (api.FSK_FLOW_PAPER, 8)):
        o = api.make_opts(n, torch.float32, c=c, max_iters=2, flow=flow)
        u = torch.ones(n, device="cuda"); v = torch.ones(n, device="cuda")
        api.fsk_sinkhorn_dense(o, Kd, a, b, u, v, api.alloc_workspace(o))
        torch.cuda.synchronize()
        assert relerr(u.cpu().numpy(), uo) <= 1e-4 and relerr(v.cpu().numpy(), vo) <= 1e-4


@pytest.mark.parametrize("td", [torch.float32, torch.float64])
def test_batched_call_refuses_a_row_pitch_beyond_its_32_bit_offsets(td):
    """The multitarget kernels address K by 32-bit offsets from a per-chunk base: a pitch above
    2^22 elements is refused before anything is launched; the widest accepted pitch runs (three
    chunks of the contraction range, so the main loop's loads see the largest offsets)."""
    n, m = 96, 4
    A = torch.full((n, m), 1.0 / n, dtype=td, device="cuda"); B = A.clone()
    for ld, ok in (((1 << 22), True), ((1 << 22) + 4, False)):
        store = torch.ones(n * ld, dtype=td, device="cuda")
        K = store.as_strided((n, n), (ld, 1))
        U = torch.ones(n, m, dtype=td, device="cuda"); V = torch.ones(n, m, dtype=td, device="cuda")
        opts = api.make_opts(n, td, m=m, max_iters=2)
        ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
        if ok:
            api.fsk_sinkhorn_batched(opts, K, A, B, U, V, ws)
            torch.cuda.synchronize()
            # K = 1, a = b = 1/n: u = 1/(n n), then v = (1/n) / (n u) = 1
            assert torch.allclose(U, torch.full_like(U, 1.0 / (n * n)), rtol=1e-6)
            assert torch.allclose(V, torch.ones_like(V), rtol=1e-6)
        else:
            with pytest.raises(api.FskError) as e:
                api.fsk_sinkhorn_batched(opts, K, A, B, U, V, ws)
            assert e.value.status == api.FSK_EUNSUPPORTED
        del store, K
