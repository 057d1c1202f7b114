"""ctypes binding of libfsk's C ABI (see ``include/fsk.h``).

Argument marshalling only: every function here has the name of the C entry point it calls,
takes torch tensors that live on the GPU (torch is used for device memory and streams, nothing
else), turns them into raw pointers / leading dimensions and returns what the C call returns.
No step of the method runs in Python, and there is no CPU fallback: if ``libfsk.so`` has not
been built, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfsk.so")

FSK_OK = 0
FSK_EINVAL, FSK_EALIGN, FSK_EDIV, FSK_EWORKSPACE, FSK_ENONFINITE, FSK_EHIP, FSK_EUNSUPPORTED = \
    -1, -2, -3, -4, -5, -6, -7
FSK_F32, FSK_F64 = 0, 1
FSK_FLOW_FUSED, FSK_FLOW_TWO_PASS, FSK_FLOW_PAPER, FSK_FLOW_RESIDENT = 0, 1, 2, 3
FSK_DAMP_NONE, FSK_DAMP_ARITHMETIC, FSK_DAMP_GEOMETRIC = 0, 1, 2
FSK_NORM_L1, FSK_NORM_L2 = 0, 1
FSK_MODE_DENSE, FSK_MODE_LOG, FSK_MODE_BATCHED, FSK_MODE_SETUP, FSK_MODE_PLAN = 0, 1, 2, 3, 4
FSK_MODE_RADIUS = 5

EXPORTS = (
    "fsk_version", "fsk_last_error", "fsk_workspace_bytes", "fsk_kernel_from_cost",
    "fsk_kernel_from_points", "fsk_sinkhorn_dense", "fsk_marginals", "fsk_block_rowpass",
    "fsk_block_colpartial", "fsk_block_fused", "fsk_sinkhorn_log_points", "fsk_sinkhorn_batched",
    "fsk_sinkhorn_batched_tol",
    "fsk_dense_profile", "fsk_bench_copy", "fsk_bench_read", "fsk_async_workspace_bytes",
    "fsk_sinkhorn_async_emulated", "fsk_plan_objective", "fsk_kernel_from_cost_lambda",
    "fsk_radius_search", "fsk_grid_workspace_bytes", "fsk_sinkhorn_grid", "fsk_dp_release",
    "fsk_sinkhorn_batched_dp", "fsk_rdp_epsilon", "fsk_set_barrier_poll_limit",
    "fsk_sinkhorn_dense_static", "fsk_local_steps_workspace_bytes", "fsk_sinkhorn_local_steps",
    "fsk_set_error_trace", "fsk_error_trace_count",
)
FSK_STATIC_SCRATCH_BYTES = 34 * 1024 * 1024


class fsk_opts(ctypes.Structure):
    _fields_ = [
        ("n", ctypes.c_int32), ("m", ctypes.c_int32), ("c", ctypes.c_int32),
        ("max_iters", ctypes.c_int32), ("tol", ctypes.c_double), ("check_every", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("flow", ctypes.c_int32), ("damping", ctypes.c_int32),
        ("eta", ctypes.c_double), ("err_norm", ctypes.c_int32),
    ]


class FskError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"fsk status {status}: {message}")
        self.status = status
        self.message = message


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2502_07021_amd.build` (needs hipcc)")
        L = ctypes.CDLL(LIB_PATH)
        L.fsk_last_error.restype = ctypes.c_char_p
        L.fsk_workspace_bytes.restype = ctypes.c_size_t
        L.fsk_workspace_bytes.argtypes = [ctypes.POINTER(fsk_opts), ctypes.c_int, ctypes.c_int]
        L.fsk_async_workspace_bytes.restype = ctypes.c_size_t
        L.fsk_async_workspace_bytes.argtypes = [ctypes.POINTER(fsk_opts), ctypes.c_int32, ctypes.c_int32]
        L.fsk_local_steps_workspace_bytes.restype = ctypes.c_size_t
        L.fsk_local_steps_workspace_bytes.argtypes = [ctypes.POINTER(fsk_opts)]
        L.fsk_grid_workspace_bytes.restype = ctypes.c_size_t
        L.fsk_grid_workspace_bytes.argtypes = [ctypes.POINTER(fsk_opts), ctypes.c_int32, ctypes.c_int32]
        _lib = L
    return _lib


def _check(status: int) -> int:
    if status != FSK_OK:
        raise FskError(status, lib().fsk_last_error().decode())
    return status


def make_opts(n: int, dtype: torch.dtype = torch.float32, m: int = 1, c: int = 1,
              max_iters: int = 0, tol: float = 0.0, check_every: int = 1,
              flow: int = FSK_FLOW_FUSED, damping: int = FSK_DAMP_NONE, eta: float = 1.0,
              err_norm: int = FSK_NORM_L1) -> fsk_opts:
    return fsk_opts(n=n, m=m, c=c, max_iters=max_iters, tol=tol, check_every=check_every,
                    dtype=FSK_F64 if dtype == torch.float64 else FSK_F32, flow=flow,
                    damping=damping, eta=eta, err_norm=err_norm)


def _p(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(None)
    if not t.is_cuda:
        raise ValueError("fsk takes device tensors")
    return ctypes.c_void_p(t.data_ptr())


def _ld(t: torch.Tensor) -> ctypes.c_int64:
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("matrix must be 2-D with unit column stride")
    return ctypes.c_int64(t.stride(0))


def _vec(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    if t is not None and not t.is_contiguous():
        raise ValueError("vectors and n x m state matrices must be contiguous")
    return _p(t)


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ws(workspace: Optional[torch.Tensor]):
    if workspace is None:
        return ctypes.c_void_p(None), ctypes.c_size_t(0)
    return _p(workspace), ctypes.c_size_t(workspace.numel() * workspace.element_size())


def fsk_version() -> int:
    return int(lib().fsk_version())


def fsk_workspace_bytes(opts: fsk_opts, mode: int = FSK_MODE_DENSE, d: int = 0) -> int:
    return int(lib().fsk_workspace_bytes(ctypes.byref(opts), mode, d))


def alloc_workspace(opts: fsk_opts, mode: int = FSK_MODE_DENSE, d: int = 0,
                    device="cuda") -> torch.Tensor:
    """Device scratch of the size the library asks for (torch owns the memory)."""
    nbytes = fsk_workspace_bytes(opts, mode, d)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def fsk_kernel_from_cost(opts, C, eps, K, stream=None) -> int:
    return _check(lib().fsk_kernel_from_cost(ctypes.byref(opts), _p(C), _ld(C), ctypes.c_double(eps),
                                             _p(K), _ld(K), _stream(stream)))


def fsk_kernel_from_points(opts, x, y, eps, normalise_by_max, K, workspace=None, want_cmax=False,
                           stream=None):
    """Returns max_ij C_ij if ``want_cmax`` (synchronises), else None."""
    wp, wn = _ws(workspace)
    cmax = ctypes.c_double(0.0)
    _check(lib().fsk_kernel_from_points(
        ctypes.byref(opts), _vec(x), _vec(y), ctypes.c_int(x.shape[1]), ctypes.c_double(eps),
        ctypes.c_int(1 if normalise_by_max else 0), _p(K), _ld(K), wp, wn,
        ctypes.byref(cmax) if want_cmax else None, _stream(stream)))
    return float(cmax.value) if want_cmax else None


def fsk_sinkhorn_dense(opts, K, a, b, u, v, workspace, stream=None):
    """Returns (iters_done, err); err is NaN in fixed-iteration mode."""
    wp, wn = _ws(workspace)
    done, err = ctypes.c_int32(0), ctypes.c_double(float("nan"))
    _check(lib().fsk_sinkhorn_dense(ctypes.byref(opts), _p(K), _ld(K), _vec(a), _vec(b), _vec(u),
                                    _vec(v), wp, wn, ctypes.byref(done), ctypes.byref(err),
                                    _stream(stream)))
    return int(done.value), float(err.value)


def fsk_sinkhorn_dense_static(opts, K, a, b, u, v, stream=None):
    """fsk_sinkhorn_dense on the library's built-in scratch array.  Returns (iters_done, err)."""
    done, err = ctypes.c_int32(0), ctypes.c_double(float("nan"))
    _check(lib().fsk_sinkhorn_dense_static(ctypes.byref(opts), _p(K), _ld(K), _vec(a), _vec(b), _vec(u),
                                           _vec(v), ctypes.byref(done), ctypes.byref(err),
                                           _stream(stream)))
    return int(done.value), float(err.value)


def fsk_dense_profile(opts, K, a, b, u, v, workspace, reps, stream=None):
    """Returns (stream_ms, other_ms, stream_launches) averaged per iteration over ``reps``."""
    wp, wn = _ws(workspace)
    t_stream, t_other, launches = ctypes.c_double(0.0), ctypes.c_double(0.0), ctypes.c_int32(0)
    _check(lib().fsk_dense_profile(ctypes.byref(opts), _p(K), _ld(K), _vec(a), _vec(b), _vec(u),
                                   _vec(v), wp, wn, ctypes.c_int(reps), ctypes.byref(t_stream),
                                   ctypes.byref(t_other), ctypes.byref(launches), _stream(stream)))
    return float(t_stream.value), float(t_other.value), int(launches.value)


def fsk_plan_objective(opts, K, C, eps, u, v, l, workspace, stream=None):
    """Returns [<P,C>, sum P(log P - 1), Eq. 1 objective, sum P, sum_ij P_ij l_j] (synchronises)."""
    wp, wn = _ws(workspace)
    out = (ctypes.c_double * 5)()
    _check(lib().fsk_plan_objective(ctypes.byref(opts), _p(K), _ld(K), _p(C), _ld(C),
                                    ctypes.c_double(eps), _vec(u), _vec(v), _vec(l), out, wp, wn,
                                    _stream(stream)))
    return [float(x) for x in out]


def fsk_kernel_from_cost_lambda(opts, c, lam, l, eps, K, stream=None) -> int:
    return _check(lib().fsk_kernel_from_cost_lambda(
        ctypes.byref(opts), _p(c), _ld(c), ctypes.c_double(lam), _vec(l), ctypes.c_double(eps),
        _p(K), _ld(K), _stream(stream)))


def fsk_radius_search(opts, c, l, a, b, eps, delta, lambda_lo, lambda_hi, max_steps, gtol, K, u, v,
                      workspace, stream=None):
    """Returns (lambda, <P,c>, sum_ij P_ij l_j, solves); K, u, v hold the last solve (synchronises)."""
    wp, wn = _ws(workspace)
    out = (ctypes.c_double * 4)()
    _check(lib().fsk_radius_search(
        ctypes.byref(opts), _p(c), _ld(c), _vec(l), _vec(a), _vec(b), ctypes.c_double(eps),
        ctypes.c_double(delta), ctypes.c_double(lambda_lo), ctypes.c_double(lambda_hi),
        ctypes.c_int32(max_steps), ctypes.c_double(gtol), _p(K), _ld(K), _vec(u), _vec(v), wp, wn, out,
        _stream(stream)))
    return float(out[0]), float(out[1]), float(out[2]), int(out[3])


def fsk_async_workspace_bytes(opts, tau: int, sync_every: int) -> int:
    return int(lib().fsk_async_workspace_bytes(ctypes.byref(opts), tau, sync_every))


def fsk_sinkhorn_async_emulated(opts, K, a, b, u, v, tau, sync_every, workspace, stream=None) -> int:
    wp, wn = _ws(workspace)
    return _check(lib().fsk_sinkhorn_async_emulated(
        ctypes.byref(opts), _p(K), _ld(K), _vec(a), _vec(b), _vec(u), _vec(v), ctypes.c_int32(tau),
        ctypes.c_int32(sync_every), wp, wn, _stream(stream)))


def fsk_local_steps_workspace_bytes(opts) -> int:
    return int(lib().fsk_local_steps_workspace_bytes(ctypes.byref(opts)))


def fsk_sinkhorn_local_steps(opts, K, a, b, u, v, w, workspace, stream=None) -> int:
    wp, wn = _ws(workspace)
    return _check(lib().fsk_sinkhorn_local_steps(
        ctypes.byref(opts), _p(K), _ld(K), _vec(a), _vec(b), _vec(u), _vec(v), ctypes.c_int32(w),
        wp, wn, _stream(stream)))


class fsk_dp(ctypes.Structure):
    _fields_ = [("clip_u", ctypes.c_double), ("clip_v", ctypes.c_double),
                ("sigma_u", ctypes.c_double), ("sigma_v", ctypes.c_double),
                ("seed", ctypes.c_uint64), ("release0", ctypes.c_uint64)]


def fsk_dp_release(opts, X, clip, sigma, seed, release, stream=None) -> int:
    return _check(lib().fsk_dp_release(ctypes.byref(opts), _vec(X), ctypes.c_double(clip),
                                       ctypes.c_double(sigma), ctypes.c_uint64(seed),
                                       ctypes.c_uint64(release), _stream(stream)))


def fsk_sinkhorn_batched_dp(opts, K, A, B, U, V, dp: "fsk_dp", workspace, stream=None) -> int:
    wp, wn = _ws(workspace)
    return _check(lib().fsk_sinkhorn_batched_dp(ctypes.byref(opts), _p(K), _ld(K), _vec(A), _vec(B),
                                                _vec(U), _vec(V), ctypes.byref(dp), wp, wn,
                                                _stream(stream)))


def fsk_rdp_epsilon(clip, sigma, releases, delta, orders):
    """(eps, minimising order) of the Renyi-DP accountant (host only)."""
    arr = (ctypes.c_double * len(orders))(*[float(x) for x in orders])
    eps, order = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().fsk_rdp_epsilon(ctypes.c_double(clip), ctypes.c_double(sigma), ctypes.c_int64(releases),
                                 ctypes.c_double(delta), arr, ctypes.c_int32(len(orders)),
                                 ctypes.byref(eps), ctypes.byref(order)))
    return float(eps.value), float(order.value)


def fsk_set_error_trace(buf, capacity: int) -> None:
    """buf: a ctypes array of 2*capacity doubles owned by the caller (None switches the trace off)."""
    lib().fsk_set_error_trace(buf, ctypes.c_int32(capacity))


def fsk_error_trace_count() -> int:
    return int(lib().fsk_error_trace_count())


def fsk_set_barrier_poll_limit(polls: int) -> None:
    lib().fsk_set_barrier_poll_limit(ctypes.c_uint32(polls))


def fsk_grid_workspace_bytes(opts, p_r: int, p_c: int) -> int:
    return int(lib().fsk_grid_workspace_bytes(ctypes.byref(opts), p_r, p_c))


def fsk_sinkhorn_grid(opts, K, a, b, u, v, p_r, p_c, workspace, stream=None) -> int:
    wp, wn = _ws(workspace)
    return _check(lib().fsk_sinkhorn_grid(
        ctypes.byref(opts), _p(K), _ld(K), _vec(a), _vec(b), _vec(u), _vec(v), ctypes.c_int32(p_r),
        ctypes.c_int32(p_c), wp, wn, _stream(stream)))


def fsk_marginals(opts, K, a, u, v, row_marginal, col_marginal, workspace, want_err=False,
                  stream=None, want_l2=False):
    """Returns None, ||P1 - a||_1 (want_err), or the pair (l1, l2) (want_l2)."""
    wp, wn = _ws(workspace)
    err = ctypes.c_double(float("nan"))
    err2 = ctypes.c_double(float("nan"))
    _check(lib().fsk_marginals(ctypes.byref(opts), _p(K), _ld(K), _vec(a), _vec(u), _vec(v),
                               _vec(row_marginal), _vec(col_marginal), wp, wn,
                               ctypes.byref(err) if (want_err or want_l2) else None,
                               ctypes.byref(err2) if want_l2 else None, _stream(stream)))
    if want_l2:
        return float(err.value), float(err2.value)
    return float(err.value) if want_err else None


def fsk_block_rowpass(opts, K_slab, row0, a_slab, v_full, u_slab, stream=None) -> int:
    return _check(lib().fsk_block_rowpass(ctypes.byref(opts), _p(K_slab), _ld(K_slab),
                                          ctypes.c_int32(row0), ctypes.c_int32(K_slab.shape[0]),
                                          _vec(a_slab), _vec(v_full), _vec(u_slab), _stream(stream)))


def fsk_block_colpartial(opts, K_slab, row0, u_slab, s_partial, workspace, stream=None) -> int:
    wp, wn = _ws(workspace)
    return _check(lib().fsk_block_colpartial(ctypes.byref(opts), _p(K_slab), _ld(K_slab),
                                             ctypes.c_int32(row0), ctypes.c_int32(K_slab.shape[0]),
                                             _vec(u_slab), _vec(s_partial), wp, wn, _stream(stream)))


def fsk_block_fused(opts, K_slab, row0, a_slab, v_full, u_slab, s_partial, workspace,
                    stream=None) -> int:
    wp, wn = _ws(workspace)
    return _check(lib().fsk_block_fused(ctypes.byref(opts), _p(K_slab), _ld(K_slab),
                                        ctypes.c_int32(row0), ctypes.c_int32(K_slab.shape[0]),
                                        _vec(a_slab), _vec(v_full), _vec(u_slab), _vec(s_partial),
                                        wp, wn, _stream(stream)))


def fsk_sinkhorn_log_points(opts, x, y, eps, a, b, f, g, workspace, stream=None):
    """Returns (iters_done, err)."""
    wp, wn = _ws(workspace)
    done, err = ctypes.c_int32(0), ctypes.c_double(float("nan"))
    _check(lib().fsk_sinkhorn_log_points(ctypes.byref(opts), _vec(x), _vec(y),
                                         ctypes.c_int(x.shape[1]), ctypes.c_double(eps), _vec(a),
                                         _vec(b), _vec(f), _vec(g), wp, wn, ctypes.byref(done),
                                         ctypes.byref(err), _stream(stream)))
    return int(done.value), float(err.value)


def fsk_sinkhorn_batched(opts, K, A, B, U, V, workspace, stream=None) -> int:
    wp, wn = _ws(workspace)
    return _check(lib().fsk_sinkhorn_batched(ctypes.byref(opts), _p(K), _ld(K), _vec(A), _vec(B),
                                             _vec(U), _vec(V), wp, wn, _stream(stream)))


def fsk_sinkhorn_batched_tol(opts, K, A, B, U, V, workspace, stream=None):
    """Returns (iters_done, err); err is NaN in fixed-iteration mode."""
    wp, wn = _ws(workspace)
    done, err = ctypes.c_int32(0), ctypes.c_double(float("nan"))
    _check(lib().fsk_sinkhorn_batched_tol(ctypes.byref(opts), _p(K), _ld(K), _vec(A), _vec(B), _vec(U),
                                          _vec(V), wp, wn, ctypes.byref(done), ctypes.byref(err),
                                          _stream(stream)))
    return int(done.value), float(err.value)


def fsk_bench_copy(dst, src, stream=None) -> int:
    nbytes = src.numel() * src.element_size()
    return _check(lib().fsk_bench_copy(_p(dst), _p(src), ctypes.c_size_t(nbytes), _stream(stream)))


def fsk_bench_read(src, sink, stream=None) -> int:
    nbytes = src.numel() * src.element_size()
    return _check(lib().fsk_bench_read(_p(src), ctypes.c_size_t(nbytes), _p(sink), _stream(stream)))
