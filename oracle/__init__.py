"""CPU oracle for the Sinkhorn hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``sinkhorn_oracle.c`` (plain fp64 C written from the
paper's definitions).  Only ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the GPU library never does and
shares no code with it.

Every function takes and returns NumPy arrays.  Vectors are promoted to fp64.
``K`` may be a float32 or float64 C-contiguous matrix; its entries are promoted
to fp64 one by one inside the C loops, so a 4 GiB fp32 kernel is never copied.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sinkhorn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math: the summation order is part of it)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
               "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized() -> str:
    """The same source with gcc's address and undefined-behaviour sanitizers (host code only): an
    out-of-bounds read, an overflowing index or a misaligned access inside the oracle then aborts
    the process instead of passing silently.  Used by tests/test_oracle_sanitized.py, which runs
    the pins against it in a child process (FSK_ORACLE_LIB selects the library to load)."""
    lib = os.path.join(_HERE, "liboracle_san.so")
    if not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
               "-shared", "-fPIC", _SRC, "-o", lib, "-lm"]
        subprocess.run(cmd, check=True)
    return lib


def _load():
    global _lib
    if _lib is None:
        path = os.environ.get("FSK_ORACLE_LIB")     # a build of the same source (the sanitized one)
        if not path:
            build()
            path = _LIB
        L = ctypes.CDLL(path)
        L.orc_max.restype = ctypes.c_double
        L.orc_max_sqeuclid.restype = ctypes.c_double
        L.orc_lse.restype = ctypes.c_double
        L.orc_dp_normal.restype = ctypes.c_double
        L.orc_rdp_epsilon.restype = ctypes.c_double
        for name in ("orc_num_threads", "orc_sinkhorn_dense", "orc_sinkhorn_dense_tol", "orc_sinkhorn_batched_tol", "orc_sinkhorn_batched_damped",
                     "orc_sinkhorn_blocked", "orc_sinkhorn_dense_damped", "orc_sinkhorn_batched",
                     "orc_sinkhorn_async_emulated", "orc_sinkhorn_local_steps", "orc_sinkhorn_grid", "orc_sinkhorn_batched_dp",
                     "orc_sinkhorn_log_points", "orc_sinkhorn_log_cost", "orc_sinkhorn_log_points_damped"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


_P = ctypes.c_void_p
_I64 = ctypes.c_int64
_INT = ctypes.c_int
_DBL = ctypes.c_double


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float64)


def _ptr(x: np.ndarray):
    return _P(x.ctypes.data)


def _kargs(K: np.ndarray):
    if K.dtype not in (np.float32, np.float64) or K.ndim != 2 or not K.flags.c_contiguous:
        raise ValueError("K must be a C-contiguous float32/float64 matrix")
    # (pointer, storage flag, number of columns, leading dimension)
    return _ptr(K), _INT(1 if K.dtype == np.float32 else 0), _I64(K.shape[1]), _I64(K.shape[1])


def _square(K: np.ndarray):
    if K.shape[0] != K.shape[1]:
        raise ValueError("K must be square")
    return _kargs(K)


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_threads(t: int) -> None:
    _load().orc_set_threads(_INT(t))


# ---------------------------------------------------------------- setup ----

def cost_sqeuclid(x, y) -> np.ndarray:
    """C_ij = ||x_i - y_j||^2 (Sec. 5.6)."""
    x, y = _f64(x), _f64(y)
    C = np.empty((x.shape[0], y.shape[0]), dtype=np.float64)
    _load().orc_cost_sqeuclid(_ptr(x), _ptr(y), _I64(x.shape[0]), _I64(y.shape[0]),
                              _INT(x.shape[1]), _ptr(C))
    return C


def gibbs(C, eps: float) -> np.ndarray:
    """K = exp(-C/eps) (Sec. 1)."""
    C = _f64(C)
    K = np.empty_like(C)
    _load().orc_gibbs(_ptr(C), _I64(C.size), _DBL(eps), _ptr(K))
    return K


def gibbs_from_points(x, y, eps: float, normalise_by_max: bool) -> tuple[np.ndarray, float]:
    """fp64 K from two point clouds, with the optional C / max(C) step.  Returns (K, max C)."""
    C = cost_sqeuclid(x, y)
    cmax = float(_load().orc_max(_ptr(C), _I64(C.size)))
    if normalise_by_max:
        _load().orc_divide_inplace(_ptr(C), _I64(C.size), _DBL(cmax))
    return gibbs(C, eps), cmax


def max_sqeuclid(x, y) -> float:
    """max_ij ||x_i - y_j||^2 without forming the cost matrix (large n)."""
    x, y = _f64(x), _f64(y)
    return float(_load().orc_max_sqeuclid(_ptr(x), _ptr(y), _I64(x.shape[0]), _I64(y.shape[0]),
                                          _INT(x.shape[1])))


def gibbs_from_points_f32(x, y, eps: float, normalise_by_max: bool) -> tuple[np.ndarray, float]:
    """Same values rounded to fp32 storage, without any n x n fp64 temporary (large n)."""
    x, y = _f64(x), _f64(y)
    L = _load()
    nx, ny, d = x.shape[0], y.shape[0], x.shape[1]
    cmax = float(L.orc_max_sqeuclid(_ptr(x), _ptr(y), _I64(nx), _I64(ny), _INT(d)))
    K = np.empty((nx, ny), dtype=np.float32)
    L.orc_gibbs_from_points_f32(_ptr(x), _ptr(y), _I64(nx), _I64(ny), _INT(d),
                                _DBL(cmax if normalise_by_max else 1.0), _DBL(eps), _ptr(K))
    return K, cmax


# ------------------------------------------------------ kernel products ----

def row_products(K, v, r0: int = 0, r1: int | None = None) -> np.ndarray:
    """q_i = sum_j K_ij v_j for rows [r0, r1); returns the slice only."""
    kp, kf, n, ld = _kargs(K)
    r1 = K.shape[0] if r1 is None else r1
    v = _f64(v)
    q = np.zeros(K.shape[0], dtype=np.float64)
    _load().orc_row_products(kp, kf, n, ld, _I64(r0), _I64(r1), _ptr(v), _ptr(q))
    return q[r0:r1]


def col_products(K, u, r0: int = 0, r1: int | None = None, c0: int = 0, c1: int | None = None) -> np.ndarray:
    """r_j = sum_{i in [r0,r1)} K_ij u_i for columns [c0, c1); returns the slice only."""
    kp, kf, n, ld = _kargs(K)
    r1 = K.shape[0] if r1 is None else r1
    c1 = K.shape[1] if c1 is None else c1
    u = _f64(u)
    r = np.zeros(K.shape[1], dtype=np.float64)
    _load().orc_col_products(kp, kf, n, ld, _I64(r0), _I64(r1), _I64(c0), _I64(c1), _ptr(u), _ptr(r))
    return r[c0:c1]


# ------------------------------------------------------------ iterations ---

def _init(n, init, m=None):
    shape = (n,) if m is None else (n, m)
    return np.ones(shape, dtype=np.float64) if init is None else _f64(init).copy()


def sinkhorn_dense(K, a, b, iters: int, u0=None, v0=None):
    """`iters` iterations of Algorithm 1's loop body (u then v), from u = v = 1 or a warm start."""
    kp, kf, n, ld = _square(K)
    a, b = _f64(a), _f64(b)
    u, v = _init(K.shape[0], u0), _init(K.shape[0], v0)
    rc = _load().orc_sinkhorn_dense(kp, kf, n, ld, _ptr(a), _ptr(b), _ptr(u), _ptr(v), _INT(iters))
    assert rc == 0
    return u, v


def sinkhorn_dense_tol(K, a, b, max_iters: int, tol: float, check_every: int = 1, u0=None, v0=None,
                       l2: bool = False):
    """Tolerance mode; returns (u, v, iterations done, last evaluated error): the 1-norm of
    P1 - a, or with l2 its 2-norm (the paper's own metric)."""
    kp, kf, n, ld = _square(K)
    a, b = _f64(a), _f64(b)
    u, v = _init(K.shape[0], u0), _init(K.shape[0], v0)
    err = _DBL(0.0)
    done = _load().orc_sinkhorn_dense_tol(kp, kf, n, ld, _ptr(a), _ptr(b), _ptr(u), _ptr(v),
                                          _INT(max_iters), _DBL(tol), _INT(check_every),
                                          ctypes.byref(err), _INT(1 if l2 else 0))
    return u, v, int(done), float(err.value)


def sinkhorn_blocked(K, a, b, iters: int, c: int, flow: int, u0=None, v0=None):
    """Row-partitioned iteration with c contiguous blocks; flow 0 = Algorithm 1 as printed
    (column slab for the transpose action), flow 1 = row slab only, partial sums added in
    block order."""
    kp, kf, n, ld = _square(K)
    a, b = _f64(a), _f64(b)
    u, v = _init(K.shape[0], u0), _init(K.shape[0], v0)
    rc = _load().orc_sinkhorn_blocked(kp, kf, n, ld, _ptr(a), _ptr(b), _ptr(u), _ptr(v),
                                      _INT(iters), _INT(c), _INT(flow))
    if rc == -2:
        raise ValueError("c must divide n")
    assert rc == 0
    return u, v


def sinkhorn_grid(K, a, b, iters: int, p_r: int, p_c: int, u0=None, v0=None):
    """Iteration on a p_r x p_c block grid: block products reduced along block rows (for K v)
    and block columns (for K^T u) in block order."""
    kp, kf, n, ld = _square(K)
    a, b = _f64(a), _f64(b)
    u, v = _init(K.shape[0], u0), _init(K.shape[0], v0)
    rc = _load().orc_sinkhorn_grid(kp, kf, n, ld, _ptr(a), _ptr(b), _ptr(u), _ptr(v), _INT(iters),
                                   _INT(p_r), _INT(p_c))
    if rc == -2:
        raise ValueError("p_r and p_c must divide n")
    assert rc == 0
    return u, v


def sinkhorn_dense_damped(K, a, b, iters: int, eta: float, geometric: bool, u0=None, v0=None):
    """Relaxed updates of Sec. 3.3 (arithmetic) or its Remark (geometric)."""
    kp, kf, n, ld = _square(K)
    a, b = _f64(a), _f64(b)
    u, v = _init(K.shape[0], u0), _init(K.shape[0], v0)
    rc = _load().orc_sinkhorn_dense_damped(kp, kf, n, ld, _ptr(a), _ptr(b), _ptr(u), _ptr(v),
                                           _INT(iters), _DBL(eta), _INT(1 if geometric else 0))
    assert rc == 0
    return u, v


def sinkhorn_async_emulated(K, a, b, iters: int, c: int, eta: float, tau: int, w: int = 1,
                            u0=None, v0=None):
    """Bounded-delay emulation of Algorithm 3: remote slices are `tau` iterations old (and only
    refreshed every `w` iterations), a client's own slice is always current."""
    kp, kf, n, ld = _square(K)
    a, b = _f64(a), _f64(b)
    u, v = _init(K.shape[0], u0), _init(K.shape[0], v0)
    rc = _load().orc_sinkhorn_async_emulated(kp, kf, n, ld, _ptr(a), _ptr(b), _ptr(u), _ptr(v),
                                             _INT(iters), _INT(c), _DBL(eta), _INT(tau), _INT(w))
    if rc == -2:
        raise ValueError("need c | n, tau >= 0, w >= 1")
    assert rc == 0
    return u, v


def sinkhorn_local_steps(K, a, b, iters: int, c: int, w: int, u0=None, v0=None):
    """Synchronous federated iteration whose collectives run only every `w` iterations: between
    them every client works on its own views (own slices current, peers' slices as of the last
    collective).  w = 1 is Algorithm 1."""
    kp, kf, n, ld = _square(K)
    a, b = _f64(a), _f64(b)
    u, v = _init(K.shape[0], u0), _init(K.shape[0], v0)
    rc = _load().orc_sinkhorn_local_steps(kp, kf, n, ld, _ptr(a), _ptr(b), _ptr(u), _ptr(v),
                                          _INT(iters), _INT(c), _INT(w))
    if rc == -2:
        raise ValueError("need c | n and w >= 1")
    assert rc == 0
    return u, v


def sinkhorn_batched(K, A, B, iters: int, U0=None, V0=None):
    """Multitarget form (Sec. 5.3.2): A, B are n x m, one histogram pair per column."""
    kp, kf, n, ld = _square(K)
    A, B = _f64(A), _f64(B)
    m = A.shape[1]
    U, V = _init(K.shape[0], U0, m), _init(K.shape[0], V0, m)
    rc = _load().orc_sinkhorn_batched(kp, kf, n, ld, _INT(m), _ptr(A), _ptr(B), _ptr(U), _ptr(V),
                                      _INT(iters))
    assert rc == 0
    return U, V


def sinkhorn_batched_damped(K, A, B, iters: int, eta: float, geometric: bool, U0=None, V0=None):
    """Multitarget form with the relaxed updates of Sec. 3.3 on every target."""
    kp, kf, n, ld = _square(K)
    A, B = _f64(A), _f64(B)
    m = A.shape[1]
    U, V = _init(K.shape[0], U0, m), _init(K.shape[0], V0, m)
    rc = _load().orc_sinkhorn_batched_damped(kp, kf, n, ld, _INT(m), _ptr(A), _ptr(B), _ptr(U), _ptr(V),
                                             _INT(iters), _DBL(eta), _INT(1 if geometric else 0))
    assert rc == 0
    return U, V


def sinkhorn_batched_tol(K, A, B, max_iters: int, tol: float, check_every: int = 1, U0=None, V0=None,
                         l2: bool = False):
    """Multitarget form until every column's row-marginal error (1-norm; 2-norm with l2) is below tol at a poll.
    Returns (U, V, iterations done, max over columns of the error at the last poll)."""
    kp, kf, n, ld = _square(K)
    A, B = _f64(A), _f64(B)
    m = A.shape[1]
    U, V = _init(K.shape[0], U0, m), _init(K.shape[0], V0, m)
    err = ctypes.c_double(float("inf"))
    done = _load().orc_sinkhorn_batched_tol(kp, kf, n, ld, _INT(m), _ptr(A), _ptr(B), _ptr(U), _ptr(V),
                                            _INT(max_iters), _DBL(tol), _INT(check_every), ctypes.byref(err),
                                            _INT(1 if l2 else 0))
    assert done >= 0
    return U, V, int(done), float(err.value)


# ---------------------------------------------------------- privacy layer ---

_U64 = ctypes.c_uint64


def philox4x32_10(ctr, key) -> np.ndarray:
    """One Philox4x32-10 block: counter (4 x uint32), key (2 x uint32) -> 4 x uint32."""
    c = (ctypes.c_uint32 * 4)(*[int(x) for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) for x in key])
    out = (ctypes.c_uint32 * 4)()
    _load().orc_philox4x32_10(c, k, out)
    return np.array(list(out), dtype=np.uint32)


def dp_normals(seed: int, release: int, first: int, count: int) -> np.ndarray:
    """Standard normal numbers first .. first+count-1 of a release."""
    out = np.empty(count, dtype=np.float64)
    _load().orc_dp_normals(_U64(seed), _U64(release), _U64(first), _I64(count), _ptr(out))
    return out


def dp_release(X, S: float, sigma: float, seed: int, release: int) -> np.ndarray:
    """Clip the rows of log X to l2 norm S, add sigma * N(0, 1), exponentiate; returns a new array."""
    X = _f64(X).copy()
    if X.ndim == 1:
        X = X[:, None]
    n, m = X.shape
    _load().orc_dp_release(_ptr(X), _I64(n), _INT(m), _DBL(S), _DBL(sigma), _U64(seed), _U64(release))
    return X


def sinkhorn_batched_dp(K, A, B, iters: int, S_u, S_v, sigma_u, sigma_v, seed: int, release0: int = 0,
                        U0=None, V0=None):
    """Multitarget iteration with a clipped, noised release after every update."""
    kp, kf, n, ld = _square(K)
    A, B = _f64(A), _f64(B)
    m = A.shape[1]
    U, V = _init(K.shape[0], U0, m), _init(K.shape[0], V0, m)
    rc = _load().orc_sinkhorn_batched_dp(kp, kf, n, ld, _INT(m), _ptr(A), _ptr(B), _ptr(U), _ptr(V),
                                         _INT(iters), _DBL(S_u), _DBL(S_v), _DBL(sigma_u), _DBL(sigma_v),
                                         _U64(seed), _U64(release0))
    assert rc == 0
    return U, V


def rdp_epsilon(S: float, sigma: float, releases: int, delta: float, orders):
    """(eps, minimising order) of the Renyi-DP accountant for `releases` clipped Gaussian releases."""
    orders = _f64(orders)
    best = _DBL(0.0)
    eps = _load().orc_rdp_epsilon(_DBL(S), _DBL(sigma), _I64(releases), _DBL(delta), _ptr(orders),
                                  _INT(orders.size), ctypes.byref(best))
    return float(eps), float(best.value)


def row_marginal(K, u, v) -> np.ndarray:
    kp, kf, n, ld = _square(K)
    u, v = _f64(u), _f64(v)
    out = np.empty(K.shape[0], dtype=np.float64)
    _load().orc_row_marginal(kp, kf, n, ld, _ptr(u), _ptr(v), _ptr(out))
    return out


def col_marginal(K, u, v) -> np.ndarray:
    kp, kf, n, ld = _square(K)
    u, v = _f64(u), _f64(v)
    out = np.empty(K.shape[1], dtype=np.float64)
    _load().orc_col_marginal(kp, kf, n, ld, _ptr(u), _ptr(v), _ptr(out))
    return out


def plan_objective(K, C, eps: float, u, v, l=None) -> np.ndarray:
    """[<P,C>, sum P(log P - 1), Eq. 1 objective, sum P, sum_ij P_ij l_j] at P = diag(u) K diag(v)."""
    kp, kf, n, ld = _square(K)
    C, u, v = _f64(C), _f64(u), _f64(v)
    out = np.zeros(5, dtype=np.float64)
    lp = _P(None)
    if l is not None:
        l = _f64(l)
        lp = _ptr(l)
    _load().orc_plan_objective(kp, kf, _ptr(C), n, ld, _DBL(eps), _ptr(u), _ptr(v), lp, _ptr(out))
    return out


def gibbs_lambda(c, lam: float, l, eps: float, as_f32: bool = False) -> np.ndarray:
    """K_ij = exp(-(lam c_ij - l_j)/eps), the kernel of the robust-risk example."""
    c = _f64(c)
    n = c.shape[0]
    K = np.empty((n, n), dtype=np.float64)
    lp = _P(None)
    if l is not None:
        l = _f64(l)
        lp = _ptr(l)
    _load().orc_gibbs_lambda(_ptr(c), ctypes.c_int64(n), _DBL(lam), lp, _DBL(eps), int(as_f32), _ptr(K))
    return K


def radius_search(c, l, a, b, eps: float, delta: float, lo: float, hi: float, max_steps: int,
                  gtol: float, iters: int, as_f32: bool = False):
    """Bisection on lambda until <P(lambda), c> = delta.  Returns (lambda, <P,c>, sum P_ij l_j,
    solves, u, v, K) with u, v, K as of the last solve."""
    c, a, b = _f64(c), _f64(a), _f64(b)
    n = c.shape[0]
    K = np.empty((n, n), dtype=np.float64)
    u = np.empty(n, dtype=np.float64)
    v = np.empty(n, dtype=np.float64)
    out = np.zeros(4, dtype=np.float64)
    lp = _P(None)
    if l is not None:
        l = _f64(l)
        lp = _ptr(l)
    _load().orc_radius_search(_ptr(c), lp, _ptr(a), _ptr(b), ctypes.c_int64(n), _DBL(eps), _DBL(delta),
                              _DBL(lo), _DBL(hi), int(max_steps), _DBL(gtol), int(iters), int(as_f32),
                              _ptr(K), _ptr(u), _ptr(v), _ptr(out))
    return float(out[0]), float(out[1]), float(out[2]), int(out[3]), u, v, K


def marginal_error(K, a, u, v) -> tuple[float, float]:
    """(||P1 - a||_1, ||P1 - a||_2) for P = diag(u) K diag(v)."""
    kp, kf, n, ld = _square(K)
    a, u, v = _f64(a), _f64(u), _f64(v)
    e1, e2 = _DBL(0.0), _DBL(0.0)
    _load().orc_marginal_error(kp, kf, n, ld, _ptr(a), _ptr(u), _ptr(v), ctypes.byref(e1),
                               ctypes.byref(e2))
    return float(e1.value), float(e2.value)


# ------------------------------------------------------------ log domain ---

def lse(z) -> float:
    z = _f64(z)
    return float(_load().orc_lse(_ptr(z), _I64(z.size)))


def log_update_points(p, w, q, h, eps: float, rows=None) -> np.ndarray:
    """out_t = eps log w_i - eps LSE_j((h_j - ||p_i - q_j||^2)/eps), i = rows[t] (all rows if None)."""
    p, w, q, h = _f64(p), _f64(w), _f64(q), _f64(h)
    if rows is None:
        rp, nr = _P(None), p.shape[0]
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rp, nr = _ptr(rows), rows.size
    out = np.empty(nr, dtype=np.float64)
    _load().orc_log_update_points(_ptr(p), _ptr(w), _ptr(q), _ptr(h), _I64(q.shape[0]),
                                  _INT(p.shape[1]), _DBL(eps), rp, _I64(nr), _ptr(out))
    return out


def log_row_marginal_points(x, f, y, g, eps: float, rows=None) -> np.ndarray:
    x, f, y, g = _f64(x), _f64(f), _f64(y), _f64(g)
    if rows is None:
        rp, nr = _P(None), x.shape[0]
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rp, nr = _ptr(rows), rows.size
    out = np.empty(nr, dtype=np.float64)
    _load().orc_log_row_marginal_points(_ptr(x), _ptr(f), _ptr(y), _ptr(g), _I64(y.shape[0]),
                                        _INT(x.shape[1]), _DBL(eps), rp, _I64(nr), _ptr(out))
    return out


def sinkhorn_log_points(x, y, eps: float, a, b, max_iters: int, tol: float = 0.0,
                        check_every: int = 1, f0=None, g0=None, l2: bool = False):
    """Log-domain iteration with the cost evaluated on the fly; returns (f, g, iters, err)."""
    x, y, a, b = _f64(x), _f64(y), _f64(a), _f64(b)
    n = x.shape[0]
    f = np.zeros(n) if f0 is None else _f64(f0).copy()
    g = np.zeros(n) if g0 is None else _f64(g0).copy()
    err = _DBL(0.0)
    done = _load().orc_sinkhorn_log_points(_ptr(x), _ptr(y), _I64(n), _INT(x.shape[1]), _DBL(eps),
                                           _ptr(a), _ptr(b), _ptr(f), _ptr(g), _INT(max_iters),
                                           _DBL(tol), _INT(check_every), ctypes.byref(err),
                                           _INT(1 if l2 else 0))
    return f, g, int(done), float(err.value)


def sinkhorn_log_points_damped(x, y, eps: float, a, b, iters: int, eta: float, geometric: bool,
                               f0=None, g0=None):
    """Log-domain iteration with the relaxed updates of Sec. 3.3; returns (f, g)."""
    x, y, a, b = _f64(x), _f64(y), _f64(a), _f64(b)
    n = x.shape[0]
    f = np.zeros(n) if f0 is None else _f64(f0).copy()
    g = np.zeros(n) if g0 is None else _f64(g0).copy()
    rc = _load().orc_sinkhorn_log_points_damped(_ptr(x), _ptr(y), _I64(n), _INT(x.shape[1]), _DBL(eps),
                                                _ptr(a), _ptr(b), _ptr(f), _ptr(g), _INT(iters), _DBL(eta),
                                                _INT(1 if geometric else 0))
    assert rc == 0
    return f, g


def sinkhorn_log_cost(C, eps: float, a, b, iters: int, f0=None, g0=None):
    """Log-domain iteration on an explicit cost matrix (small n)."""
    C, a, b = _f64(C), _f64(a), _f64(b)
    n = C.shape[0]
    f = np.zeros(n) if f0 is None else _f64(f0).copy()
    g = np.zeros(n) if g0 is None else _f64(g0).copy()
    rc = _load().orc_sinkhorn_log_cost(_ptr(C), _I64(n), _DBL(eps), _ptr(a), _ptr(b), _ptr(f),
                                       _ptr(g), _INT(iters))
    assert rc == 0
    return f, g
