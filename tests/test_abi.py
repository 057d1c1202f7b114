"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before touching the GPU (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def api():
    from paper_2502_07021_amd import api as _api
    if not os.path.exists(_api.LIB_PATH):
        from paper_2502_07021_amd import build
        build.build_library()
    return _api


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fsk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fsk_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(api):
    names = declared_functions()
    assert len(names) >= 12
    L = api.lib()
    for name in names:
        assert hasattr(L, name), f"{name} declared in fsk.h but not exported"
    assert set(names) == set(api.EXPORTS)      # the binding covers the same set


def test_opts_struct_layout_matches_header(api):
    # int32 x4, double, int32 x4, double  -> 8-byte aligned, 48 bytes
    assert ctypes.sizeof(api.fsk_opts) == 56 and api.fsk_opts.err_norm.offset == 48
    assert api.fsk_opts.tol.offset == 16 and api.fsk_opts.check_every.offset == 24
    assert api.fsk_opts.eta.offset == 40


def test_dp_struct_layout_and_host_accountant(api, orc):
    # double x4, uint64 x2 -> 48 bytes
    assert ctypes.sizeof(api.fsk_dp) == 48 and api.fsk_dp.seed.offset == 32
    # the accountant runs on the host: same bound as the oracle's, and bad arguments are refused
    orders = [1.25, 1.5, 2.0, 3.0, 5.0, 8.0, 16.0, 32.0, 64.0]
    for S, sigma, T in ((4.0, 50.0, 2000), (1.0, 1.0, 10), (20.0, 0.5, 2)):
        eps, p = api.fsk_rdp_epsilon(S, sigma, T, 1e-5, orders)
        eps_o, p_o = orc.rdp_epsilon(S, sigma, T, 1e-5, orders)
        assert p == p_o and eps == pytest.approx(eps_o, rel=1e-14)
    for bad in ((0.0, 1.0, 5, 1e-5, orders), (1.0, 0.0, 5, 1e-5, orders), (1.0, 1.0, -1, 1e-5, orders),
                (1.0, 1.0, 5, 1.0, orders), (1.0, 1.0, 5, 1e-5, [0.5, 1.0])):
        with pytest.raises(api.FskError):
            api.fsk_rdp_epsilon(*bad)


def test_version_and_error_string(api):
    assert api.fsk_version() >= 100
    assert isinstance(api.lib().fsk_last_error(), bytes)


@pytest.mark.parametrize("field,value,status", [
    ("n", 0, -1), ("m", 0, -1), ("c", 0, -1), ("max_iters", -1, -1), ("dtype", 7, -1),
    ("flow", 9, -1), ("damping", 5, -1), ("c", 3, -3),
])
def test_bad_options_are_rejected_on_the_host(api, field, value, status):
    import torch
    opts = api.make_opts(64, torch.float32, max_iters=1)
    setattr(opts, field, value)
    dummy = ctypes.c_void_p(256)     # never dereferenced: validation fails first
    rc = api.lib().fsk_sinkhorn_dense(ctypes.byref(opts), dummy, ctypes.c_int64(64), dummy, dummy,
                                      dummy, dummy, dummy, ctypes.c_size_t(1 << 30), None, None, None)
    assert rc == status
    assert api.lib().fsk_last_error() != b""
    assert api.fsk_workspace_bytes(opts) == 0


def test_bad_pointers_and_alignment_are_rejected_on_the_host(api):
    import torch
    L = api.lib()
    opts = api.make_opts(64, torch.float32, max_iters=1)
    ok = ctypes.c_void_p(4096)
    args = lambda K, ld, u: (ctypes.byref(opts), K, ctypes.c_int64(ld), ok, ok, u, ok, ok,
                             ctypes.c_size_t(1 << 30), None, None, None)
    assert L.fsk_sinkhorn_dense(*args(None, 64, ok)) == api.FSK_EINVAL
    assert L.fsk_sinkhorn_dense(*args(ctypes.c_void_p(4100), 64, ok)) == api.FSK_EALIGN
    assert L.fsk_sinkhorn_dense(*args(ok, 66, ok)) == api.FSK_EALIGN       # pitch not 16 B
    assert L.fsk_sinkhorn_dense(*args(ok, 32, ok)) == api.FSK_EINVAL       # ld < n
    assert L.fsk_sinkhorn_dense(*args(ok, 64, ctypes.c_void_p(4100))) == api.FSK_EALIGN
    opts.damping = api.FSK_DAMP_ARITHMETIC; opts.eta = 0.0
    assert L.fsk_sinkhorn_dense(*args(ok, 64, ok)) == api.FSK_EINVAL
    opts.damping = 0; opts.tol = 1e-3; opts.check_every = 0
    assert L.fsk_sinkhorn_dense(*args(ok, 64, ok)) == api.FSK_EINVAL
    # workspace too small
    opts.tol = 0.0
    small = (ctypes.byref(opts), ok, ctypes.c_int64(64), ok, ok, ok, ok, ok, ctypes.c_size_t(16),
             None, None, None)
    assert L.fsk_sinkhorn_dense(*small) == api.FSK_EWORKSPACE
    assert b"workspace" in L.fsk_last_error()


def test_multitarget_calls_refuse_what_they_do_not_carry(api):
    """Options a call would otherwise ignore are refused on the host, before any launch."""
    import torch
    L = api.lib()
    ok = ctypes.c_void_p(4096)
    big = ctypes.c_size_t(1 << 40)
    opts = api.make_opts(64, torch.float32, m=8, max_iters=3, damping=api.FSK_DAMP_ARITHMETIC, eta=0.5)
    done, err = ctypes.c_int32(0), ctypes.c_double(0.0)
    fixed = lambda: L.fsk_sinkhorn_batched(ctypes.byref(opts), ok, ctypes.c_int64(64), ok, ok, ok, ok, ok, big, None)
    tolc = lambda: L.fsk_sinkhorn_batched_tol(ctypes.byref(opts), ok, ctypes.c_int64(64), ok, ok, ok, ok, ok, big,
                                              ctypes.byref(done), ctypes.byref(err), None)
    dp = api.fsk_dp(1.0, 1.0, 0.1, 0.1, 7, 0)
    noisy = lambda: L.fsk_sinkhorn_batched_dp(ctypes.byref(opts), ok, ctypes.c_int64(64), ok, ok, ok, ok,
                                              ctypes.byref(dp), ok, big, None)
    assert noisy() == api.FSK_EUNSUPPORTED and b"undamped" in L.fsk_last_error()
    # a damped multitarget run keeps every half-step in a scratch matrix: more workspace, or a refusal
    undamped = api.make_opts(64, torch.float32, m=8, max_iters=3)
    need = api.fsk_workspace_bytes(opts, api.FSK_MODE_BATCHED)
    assert need >= api.fsk_workspace_bytes(undamped, api.FSK_MODE_BATCHED) + 64 * 8 * 4
    short = lambda: L.fsk_sinkhorn_batched(ctypes.byref(opts), ok, ctypes.c_int64(64), ok, ok, ok, ok, ok,
                                           ctypes.c_size_t(need - 16), None)
    assert short() == api.FSK_EWORKSPACE and b"damped" in L.fsk_last_error()
    opts.damping = api.FSK_DAMP_NONE; opts.tol = 1e-6
    assert fixed() == api.FSK_EUNSUPPORTED and b"fsk_sinkhorn_batched_tol" in L.fsk_last_error()
    opts.c = 2
    assert tolc() == api.FSK_EUNSUPPORTED
    # tolerance mode asks for more workspace than the fixed-count mode (the copy of U)
    opts.c = 1
    with_tol = api.fsk_workspace_bytes(opts, api.FSK_MODE_BATCHED)
    opts.tol = 0.0
    assert with_tol >= api.fsk_workspace_bytes(opts, api.FSK_MODE_BATCHED) + 64 * 8 * 4


def test_last_error_is_per_thread(api):
    """fsk_last_error() reports the calling thread's last failure, not another thread's."""
    import threading
    import torch
    L = api.lib()
    ok = ctypes.c_void_p(4096)
    seen = {}
    gate = threading.Barrier(2)

    def worker(name, n):
        opts = api.make_opts(64, torch.float32, max_iters=1)
        opts.n = n                                            # 0 / negative: refused with the value in the text
        st = L.fsk_sinkhorn_dense(ctypes.byref(opts), ok, ctypes.c_int64(64), ok, ok, ok, ok, ok,
                                  ctypes.c_size_t(1 << 30), None, None, None)
        gate.wait()                                           # both calls have failed before either reads
        seen[name] = (st, bytes(L.fsk_last_error()))

    ts = [threading.Thread(target=worker, args=("first", 0)), threading.Thread(target=worker, args=("second", -7))]
    [t.start() for t in ts]; [t.join() for t in ts]
    assert seen["first"][0] == api.FSK_EINVAL and seen["second"][0] == api.FSK_EINVAL
    assert seen["first"][1] != seen["second"][1]
    assert b"-7" in seen["second"][1] and b"-7" not in seen["first"][1]


def test_static_scratch_call_refuses_what_does_not_fit(api):
    """The entry point for callers that cannot allocate rejects, on the host, a problem whose
    scratch exceeds the built-in array (and bad arguments like its sibling)."""
    import torch
    L = api.lib()
    ok = ctypes.c_void_p(4096)
    opts = api.make_opts(46400, torch.float32, max_iters=1, flow=api.FSK_FLOW_TWO_PASS)
    assert api.fsk_workspace_bytes(opts) > api.FSK_STATIC_SCRATCH_BYTES
    rc = L.fsk_sinkhorn_dense_static(ctypes.byref(opts), ok, ctypes.c_int64(46400), ok, ok, ok, ok,
                                     None, None, None)
    assert rc == api.FSK_EWORKSPACE and b"built-in" in L.fsk_last_error()
    opts = api.make_opts(64, torch.float32, max_iters=1)
    assert L.fsk_sinkhorn_dense_static(ctypes.byref(opts), None, ctypes.c_int64(64), ok, ok, ok, ok,
                                       None, None, None) == api.FSK_EINVAL
    text = open(os.path.join(ROOT, "include", "fsk.h")).read()
    assert int(re.search(r"FSK_STATIC_SCRATCH_BYTES \((\d+)u \* 1024u \* 1024u\)", text).group(1)) * 1024 * 1024 \
        == api.FSK_STATIC_SCRATCH_BYTES
