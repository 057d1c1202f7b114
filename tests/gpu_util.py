"""Helpers for the GPU parity tests: move seeded inputs to the device, call the C ABI through
the binding, bring results back.  No arithmetic of the method lives here."""
import numpy as np
import torch

from paper_2502_07021_amd import api

TOL = {np.dtype(np.float32): 1e-4, np.dtype(np.float64): 1e-10}   # max relative error bar


def tdtype(np_dtype):
    return torch.float64 if np.dtype(np_dtype) == np.float64 else torch.float32


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def relerr(got, ref):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref) / np.abs(ref)))


def gauge_free(got, ref):
    """Error of a positive scaling vector that a uniform rescaling cannot hide or cause: the
    scalings of the iteration are unique up to (u/s, s v) (appendix on convergence, uniqueness up
    to rescaling), so d = log(got/ref) is split into its mean (the drift along that direction) and
    max |d - mean|.  Returns (max |d - mean d|, largest |mean d|); an n x m matrix of scalings has
    one such direction per column (target)."""
    d = np.log(np.asarray(got, dtype=np.float64) / np.asarray(ref, dtype=np.float64))
    mean = d.mean(axis=0, keepdims=True)
    return float(np.max(np.abs(d - mean))), float(np.max(np.abs(mean)))


def say(capsys, msg):
    """A progress line that reaches the terminal although pytest captures output: the long
    oracle runs print one after every chunk."""
    with capsys.disabled():
        print(msg, flush=True)


def run_dense(K_host, a, b, iters, flow=api.FSK_FLOW_FUSED, c=1, u0=None, v0=None, tol=0.0,
              check_every=1, damping=api.FSK_DAMP_NONE, eta=1.0, ld=None, K_dev=None,
              err_norm=api.FSK_NORM_L1):
    """Runs fsk_sinkhorn_dense; returns (u, v, iters_done, err) with u, v as NumPy arrays."""
    n = K_host.shape[0] if K_dev is None else K_dev.shape[0]
    dt = K_host.dtype if K_dev is None else (np.float64 if K_dev.dtype == torch.float64 else np.float32)
    td = tdtype(dt)
    pack = 16 // np.dtype(dt).itemsize
    if K_dev is None and ld is None and n % pack != 0:
        ld = (n + pack - 1) // pack * pack     # the ABI wants 16-byte row pitch
    if K_dev is None:
        if ld is None:
            K_dev = dev(K_host)
        else:                       # padded rows: garbage (NaN) in the padding columns
            full = torch.full((n, ld), float("nan"), dtype=td, device="cuda")
            full[:, :n] = dev(K_host)
            K_dev = full[:, :n]
    opts = api.make_opts(n, td, c=c, max_iters=iters, tol=tol, check_every=check_every, flow=flow,
                         damping=damping, eta=eta, err_norm=err_norm)
    ws = api.alloc_workspace(opts, api.FSK_MODE_DENSE)
    u = torch.ones(n, dtype=td, device="cuda") if u0 is None else dev(np.asarray(u0, dtype=dt))
    v = torch.ones(n, dtype=td, device="cuda") if v0 is None else dev(np.asarray(v0, dtype=dt))
    done, err = api.fsk_sinkhorn_dense(opts, K_dev, dev(a.astype(dt)), dev(b.astype(dt)), u, v, ws)
    torch.cuda.synchronize()
    return u.cpu().numpy(), v.cpu().numpy(), done, err
