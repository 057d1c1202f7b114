"""GPU parity of the multitarget (batched) path against the oracle: n x m scalings sharing K,
the two products done as matrix products on the matrix cores.  Bar: max relative error on U, V
and the column marginals <= 1e-4 (fp32)."""
import numpy as np
import pytest
import torch

from paper_2502_07021_amd import api, workloads
from gpu_util import dev, relerr, run_dense

pytestmark = pytest.mark.gpu


def run_batched(K, A, B, iters, ld=None, small_workspace=False, dtype=np.float32, U0=None, V0=None):
    n, m = A.shape
    td = torch.float64 if dtype == np.float64 else torch.float32
    opts = api.make_opts(n, td, m=m, max_iters=iters)
    ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
    if small_workspace:      # no room for the transposed copy of K: the direct row kernel runs
        ws = ws[: ws.numel() - n * n * 4]
    if ld is None:
        ld = (n + 3) // 4 * 4
    full = torch.full((n, ld), float("nan"), dtype=td, device="cuda")
    full[:, :n] = dev(np.ascontiguousarray(K.astype(dtype)))
    U = torch.ones(n, m, dtype=td, device="cuda") if U0 is None else dev(U0)
    V = torch.ones(n, m, dtype=td, device="cuda") if V0 is None else dev(V0)
    api.fsk_sinkhorn_batched(opts, full[:, :n], dev(np.ascontiguousarray(A.astype(dtype))),
                             dev(np.ascontiguousarray(B.astype(dtype))), U, V, ws)
    torch.cuda.synchronize()
    return U.cpu().numpy(), V.cpu().numpy()


def problem(orc, n, m, seed, eps=0.05):
    w = workloads.make(5, n=n, m=m, seed=seed)
    K64, _ = orc.gibbs_from_points(w.x, w.y, eps, False)
    return np.ascontiguousarray(K64.astype(np.float32)), w.a, w.b


@pytest.mark.parametrize("n,m", [(1, 1), (5, 3), (64, 64), (65, 33), (100, 1), (257, 64), (1000, 40),
                                 (1030, 64), (2048, 64)])
def test_batched_matches_oracle(orc, n, m):
    K, A, B = problem(orc, n, m, 500 + n + m)
    Uo, Vo = orc.sinkhorn_batched(K, A, B, 9)
    U, V = run_batched(K, A, B, 9, ld=(n + 3) // 4 * 4 + 8)
    assert relerr(U, Uo) <= 1e-4 and relerr(V, Vo) <= 1e-4
    # column marginals of every plan, evaluated by the oracle on the GPU's scalings
    for k in range(0, m, max(1, m // 4)):
        cm = orc.col_marginal(K, U[:, k], V[:, k])
        assert relerr(cm, B[:, k]) <= 1e-4


@pytest.mark.parametrize("n,m", [(65, 33), (1030, 64)])
def test_batched_without_room_for_the_transposed_kernel(orc, n, m):
    K, A, B = problem(orc, n, m, 900 + n)
    Uo, Vo = orc.sinkhorn_batched(K, A, B, 9)
    U, V = run_batched(K, A, B, 9, small_workspace=True)
    assert relerr(U, Uo) <= 1e-4 and relerr(V, Vo) <= 1e-4


@pytest.mark.parametrize("dtype,small", [(np.float32, False), (np.float32, True), (np.float64, False)])
def test_a_split_run_gives_the_bits_of_the_run_in_one_call(orc, dtype, small):
    """Which kernel forms K V rests on (n, m, workspace), never on the iteration count: 9
    iterations == 8 + 1 == 1 + 8, bit for bit, with and without room for the transposed copy."""
    K, A, B = problem(orc, 1030, 64, 77)
    U, V = run_batched(K, A, B, 9, small_workspace=small, dtype=dtype)
    for first in (8, 1):
        Ua, Va = run_batched(K, A, B, first, small_workspace=small, dtype=dtype)
        Ub, Vb = run_batched(K, A, B, 9 - first, small_workspace=small, dtype=dtype, U0=Ua, V0=Va)
        assert np.array_equal(U, Ub) and np.array_equal(V, Vb)


def test_cfg5_law_full_iteration_count(orc):
    """Configuration 5 at reduced n: Dirichlet(1) marginals (entries down to 1e-9), eps = 0.05,
    300 iterations, m = 64."""
    K, A, B = problem(orc, 1536, 64, 20250207 * 10 + 5)
    Uo, Vo = orc.sinkhorn_batched(K, A, B, 300)
    U, V = run_batched(K, A, B, 300)
    assert relerr(U, Uo) <= 1e-4 and relerr(V, Vo) <= 1e-4


def test_batched_column_equals_single_histogram_run(orc):
    """Sec. 5.3.2: column k of the stacked run is the run on (a_k, b_k) alone."""
    K, A, B = problem(orc, 700, 8, 77)
    U, V = run_batched(K, A, B, 25)
    for k in (0, 3, 7):
        u, v, _, _ = run_dense(K, A[:, k].copy(), B[:, k].copy(), 25)
        assert relerr(U[:, k], u) <= 2e-5 and relerr(V[:, k], v) <= 2e-5


@pytest.mark.parametrize("n,m,small", [(300, 65, False), (513, 130, False), (1000, 200, False),
                                         (257, 67, True), (400, 500, False), (200, 5000, False)])
def test_more_than_64_histograms_go_in_column_groups(orc, n, m, small):
    """The paper stacks hundreds of targets: columns beyond 64 are served in groups of 64, each
    column still an independent run."""
    K, A, B = problem(orc, n, m, 1300 + n + m)
    Uo, Vo = orc.sinkhorn_batched(K, A, B, 7)
    U, V = run_batched(K, A, B, 7, small_workspace=small)
    assert relerr(U, Uo) <= 1e-4 and relerr(V, Vo) <= 1e-4
    for k in (0, 63, 64, m - 1):
        cm = orc.col_marginal(K, U[:, k], V[:, k])
        assert relerr(cm, B[:, k]) <= 1e-4


@pytest.mark.parametrize("n,m", [(1, 1), (2, 2), (5, 3), (64, 64), (65, 33), (100, 1), (257, 64),
                                 (1000, 40), (1030, 64), (515, 130), (300, 200)])
def test_batched_fp64_matches_oracle(orc, n, m):
    """FSK_F64: the same products on the fp64 matrix instruction; the bar is 1e-10."""
    w = workloads.make(5, n=n, m=m, seed=2100 + n + m)
    K, _ = orc.gibbs_from_points(w.x, w.y, 0.05, False)
    A = w.a.astype(np.float64); B = w.b.astype(np.float64)
    Uo, Vo = orc.sinkhorn_batched(K, A, B, 9)
    U, V = run_batched(K, A, B, 9, ld=(n + 1) // 2 * 2 + 6, dtype=np.float64)
    assert relerr(U, Uo) <= 1e-10 and relerr(V, Vo) <= 1e-10
    for k in (0, m // 2, m - 1):
        cm = orc.col_marginal(K, U[:, k], V[:, k])
        assert relerr(cm, B[:, k]) <= 1e-10


def test_batched_fp64_needs_the_full_workspace():
    n, m = 300, 8
    opts = api.make_opts(n, torch.float64, m=m, max_iters=2)
    ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
    K = torch.ones(n, n, dtype=torch.float64, device="cuda")
    X = torch.ones(n, m, dtype=torch.float64, device="cuda")
    with pytest.raises(api.FskError) as e:
        api.fsk_sinkhorn_batched(opts, K, X, X, X.clone(), X.clone(), ws[: ws.numel() // 2])
    assert e.value.status == api.FSK_EWORKSPACE


def _run_tol(K, A, B, max_iters, tol, check_every, dtype):
    n, m = A.shape
    td = torch.float64 if dtype == np.float64 else torch.float32
    opts = api.make_opts(n, td, m=m, max_iters=max_iters, tol=tol, check_every=check_every)
    ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
    pack = 16 // np.dtype(dtype).itemsize
    full = torch.full((n, (n + pack - 1) // pack * pack), float("nan"), dtype=td, device="cuda")
    full[:, :n] = dev(np.ascontiguousarray(K.astype(dtype)))
    Kd = full[:, :n]
    U = torch.ones(n, m, dtype=td, device="cuda"); V = torch.ones(n, m, dtype=td, device="cuda")
    done, err = api.fsk_sinkhorn_batched_tol(opts, Kd, dev(np.ascontiguousarray(A.astype(dtype))),
                                             dev(np.ascontiguousarray(B.astype(dtype))), U, V, ws)
    return U.cpu().numpy(), V.cpu().numpy(), done, err


@pytest.mark.parametrize("dtype,n,m,tol,check_every", [
    (np.float64, 300, 70, 1e-9, 1), (np.float64, 515, 5, 1e-9, 7),
    (np.float32, 1030, 64, 2e-5, 1), (np.float32, 400, 150, 2e-5, 4),
])
def test_batched_tolerance_mode(orc, dtype, n, m, tol, check_every):
    """Stop rule over all targets at once (Sec. 5.3.2): the polled state, its iteration count
    and its error against the oracle's; the handed-back state is the fixed-count run's."""
    rng = np.random.default_rng(4000 + n + m)
    x = rng.uniform(size=(n, 2)); y = rng.uniform(size=(n, 2))
    K64, _ = orc.gibbs_from_points(x, y, 0.3, False)
    K = np.ascontiguousarray(K64.astype(dtype))
    A = rng.uniform(0.5, 1.5, (n, m)) ** 3; A = np.ascontiguousarray((A / A.sum(0)).astype(dtype))   # targets of
    B = rng.uniform(0.5, 1.5, (n, m)) ** 3; B = np.ascontiguousarray((B / B.sum(0)).astype(dtype))   # unequal speed
    Uo, Vo, done_o, err_o = orc.sinkhorn_batched_tol(K, A, B, 400, tol, check_every)
    U, V, done, err = _run_tol(K, A, B, 400, tol, check_every, dtype)
    assert done_o < 400 and err < tol
    if dtype == np.float64:
        assert done == done_o and err == pytest.approx(err_o, rel=1e-5)
        assert relerr(U, Uo) <= 1e-10 and relerr(V, Vo) <= 1e-10
    else:  # fp32 sums may cross the threshold one poll earlier or later
        assert abs(done - done_o) <= check_every
    assert done % check_every == 0
    Uf, Vf = run_batched(K, A, B, done, dtype=dtype)         # same state as the fixed-count run
    assert np.array_equal(U, Uf) and np.array_equal(V, Vf)
    # the error it reports is the error of the state it hands back (oracle's evaluation, fp64)
    errs = [orc.marginal_error(K, A[:, k], U[:, k], V[:, k])[0] for k in range(0, m, max(1, m // 8))]
    assert max(errs) <= err * (1 + 1e-3) + (1e-6 if dtype == np.float32 else 1e-13)


def test_batched_tolerance_cap_fixed_mode_and_workspace(orc):
    K, A, B = problem(orc, 257, 33, 77)
    U, V, done, err = _run_tol(K, A, B, 6, 1e-30, 4, np.float32)           # cap: last iteration polled
    assert done == 6 and err > 1e-30
    Uf, Vf = run_batched(K, A, B, 6)
    assert np.array_equal(U, Uf) and np.array_equal(V, Vf)
    U, V, done, err = _run_tol(K, A, B, 5, 0.0, 1, np.float32)             # tol <= 0: fixed count
    assert done == 5 and np.isnan(err)
    opts = api.make_opts(257, torch.float32, m=33, max_iters=5, tol=1e-6, check_every=1)
    small = api.alloc_workspace(api.make_opts(257, torch.float32, m=33, max_iters=5), api.FSK_MODE_BATCHED)
    Kd = torch.zeros(257, 260, device="cuda")[:, :257]; Kd.copy_(dev(K))
    Ad = dev(A.astype(np.float32)); Bd = dev(B.astype(np.float32))
    X = torch.ones(257, 33, device="cuda")
    with pytest.raises(api.FskError) as e:                                  # no room for the copy of U
        api.fsk_sinkhorn_batched_tol(opts, Kd, Ad, Bd, X.clone(), X.clone(), small)
    assert e.value.status == api.FSK_EWORKSPACE


def _run_damped(K, A, B, iters, eta, geometric, dtype, tol=0.0, check_every=1, small_workspace=False):
    n, m = A.shape
    td = torch.float64 if dtype == np.float64 else torch.float32
    damping = api.FSK_DAMP_GEOMETRIC if geometric else api.FSK_DAMP_ARITHMETIC
    opts = api.make_opts(n, td, m=m, max_iters=iters, damping=damping, eta=eta, tol=tol, check_every=check_every)
    ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
    if small_workspace:
        ws = ws[: ws.numel() - 256]
    pack = 16 // np.dtype(dtype).itemsize
    full = torch.full((n, (n + pack - 1) // pack * pack), float("nan"), dtype=td, device="cuda")
    full[:, :n] = dev(np.ascontiguousarray(K.astype(dtype)))
    U = torch.ones(n, m, dtype=td, device="cuda"); V = torch.ones(n, m, dtype=td, device="cuda")
    Ad = dev(np.ascontiguousarray(A.astype(dtype))); Bd = dev(np.ascontiguousarray(B.astype(dtype)))
    if tol > 0:
        done, err = api.fsk_sinkhorn_batched_tol(opts, full[:, :n], Ad, Bd, U, V, ws)
    else:
        api.fsk_sinkhorn_batched(opts, full[:, :n], Ad, Bd, U, V, ws)
        done, err = iters, float("nan")
    torch.cuda.synchronize()
    return U.cpu().numpy(), V.cpu().numpy(), done, err


@pytest.mark.parametrize("dtype,n,m,eta,geometric", [
    (np.float64, 300, 70, 0.6, False), (np.float64, 515, 5, 0.35, True), (np.float64, 64, 64, 1.0, False),
    (np.float32, 1030, 64, 0.5, False), (np.float32, 400, 150, 0.7, True), (np.float32, 5, 3, 0.25, True),
])
def test_batched_relaxed_updates(orc, dtype, n, m, eta, geometric):
    """Relaxed updates (Sec. 3.3) on every target of the multitarget iteration, both means."""
    K, A, B = problem(orc, n, m, 6100 + n + m, eps=0.1)
    K = np.ascontiguousarray(K.astype(dtype)); A = A.astype(dtype); B = B.astype(dtype)
    ones = np.ones((n, m))
    Uo, Vo = orc.sinkhorn_batched_damped(K, A, B, 12, eta, geometric, ones, ones)
    U, V, _, _ = _run_damped(K, A, B, 12, eta, geometric, dtype)
    bar = 1e-10 if dtype == np.float64 else 1e-4
    assert relerr(U, Uo) <= bar and relerr(V, Vo) <= bar
    if eta == 1.0:                                             # eta = 1 is the plain iteration
        Up, Vp = run_batched(K, A, B, 12, dtype=dtype)
        assert np.array_equal(U, Up) and np.array_equal(V, Vp)


@pytest.mark.parametrize("dtype,geometric", [(np.float64, False), (np.float32, True)])
def test_batched_relaxed_updates_with_the_stop_rule(orc, dtype, geometric):
    """Damped run with a tolerance: the error polled is that of the damped state (its undamped
    next U against it), and the state handed back is the fixed-count damped run's."""
    n, m, eta, ce = 300, 40, 0.6, 3
    tol = 1e-8 if dtype == np.float64 else 3e-5
    rng = np.random.default_rng(93)
    x = rng.uniform(size=(n, 2)); y = rng.uniform(size=(n, 2))
    K64, _ = orc.gibbs_from_points(x, y, 0.3, False)
    K = np.ascontiguousarray(K64.astype(dtype))
    A = rng.uniform(0.5, 1.5, (n, m)) ** 3; A = np.ascontiguousarray((A / A.sum(0)).astype(dtype))
    B = rng.uniform(0.5, 1.5, (n, m)) ** 3; B = np.ascontiguousarray((B / B.sum(0)).astype(dtype))
    U, V, done, err = _run_damped(K, A, B, 600, eta, geometric, dtype, tol=tol, check_every=ce)
    assert 0 < done < 600 and done % ce == 0 and err < tol
    Uf, Vf, _, _ = _run_damped(K, A, B, done, eta, geometric, dtype)
    assert np.array_equal(U, Uf) and np.array_equal(V, Vf)
    ones = np.ones((n, m))
    worst = lambda UU, VV: max(orc.marginal_error(K, A[:, k], UU[:, k], VV[:, k])[0] for k in range(m))
    Uo, Vo = orc.sinkhorn_batched_damped(K, A, B, done, eta, geometric, ones, ones)
    assert worst(Uo, Vo) == pytest.approx(err, rel=1e-6 if dtype == np.float64 else 0.2)
    if dtype == np.float64:                                    # the poll before it had not converged
        Up, Vp = orc.sinkhorn_batched_damped(K, A, B, done - ce, eta, geometric, ones, ones)
        assert worst(Up, Vp) >= tol and relerr(U, Uo) <= 1e-10


def test_batched_relaxed_updates_need_the_scratch_matrix(orc):
    K, A, B = problem(orc, 100, 8, 5)
    with pytest.raises(api.FskError) as e:
        _run_damped(K, A, B, 3, 0.5, False, np.float32, small_workspace=True)
    assert e.value.status == api.FSK_EWORKSPACE
