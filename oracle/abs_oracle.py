"""TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Python face of the plain CPU oracle in ``abs_oracle.c`` (same directory): it
compiles that file with gcc, loads it with ctypes and sequences its calls in
the order of the ABS-SGD paper's Algorithm 1.  Only ``tests/``, the smoke check
and the benchmark's CPU-baseline leg may import this module; it shares nothing
with the HIP library and does not import it.

Notation follows Algorithm 1: N workers, reference batch size M_r, per-worker
accumulated gradient G_t^i and batch size M_t^i, averaged delayed gradient
Gbar_{t-1}, learning rate gamma.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "abs_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_c_i64 = ctypes.c_int64
_c_dbl = ctypes.c_double
_c_flt = ctypes.c_float
_vp = ctypes.c_void_p


def build_oracle(force=False):
    """Compile abs_oracle.c -> liboracle.so (plain gcc, no fast-math, no
    contraction, OpenMP only for the loop over parameters)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
           "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           _SRC, "-o", _LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build_oracle())
        _lib.oracle_max_threads.restype = ctypes.c_int
        _lib.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib.oracle_zero.argtypes = [_vp, _c_i64]
        _lib.oracle_accumulate_f32.argtypes = [_vp, _vp, _c_i64, _c_i64]
        _lib.oracle_accumulate_bf16.argtypes = [_vp, _vp, _c_i64, _c_i64]
        _lib.oracle_sync_update.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_int, _c_i64,
                                            _c_dbl, _c_dbl, _c_dbl]
        _lib.oracle_sync_update.restype = ctypes.c_int
        _lib.oracle_sync_update_dc.argtypes = [_vp, _vp, _vp, _vp, _vp, ctypes.c_int, _c_i64,
                                               _c_dbl, _c_dbl, _c_dbl, _c_dbl]
        _lib.oracle_sync_update_dc.restype = ctypes.c_int
        _lib.oracle32_sync_update_dc.argtypes = [_vp, _vp, _vp, _vp, _vp, ctypes.c_int, _c_i64,
                                                 _c_flt, _c_flt, _c_flt, _c_flt]
        _lib.oracle32_sync_update_dc.restype = ctypes.c_int
        _lib.oracle_sync_update_dcm.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_int, _c_i64] + [ctypes.c_double] * 5
        _lib.oracle_sync_update_dcm.restype = ctypes.c_int
        _lib.oracle32_sync_update_dcm.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_int, _c_i64] + [ctypes.c_float] * 5
        _lib.oracle32_sync_update_dcm.restype = ctypes.c_int
        _lib.oracle_sync_update_adam.argtypes = [_vp, _vp, _vp, _vp, _vp, ctypes.c_int, _c_i64,
                                                 _c_dbl, _c_dbl, _c_dbl, _c_dbl, _c_dbl, _c_i64]
        _lib.oracle_sync_update_adam.restype = ctypes.c_int
        _lib.oracle32_sync_update_adam.argtypes = [_vp, _vp, _vp, _vp, _vp, ctypes.c_int, _c_i64,
                                                   _c_flt, _c_flt, _c_flt, _c_flt, _c_flt, _c_i64]
        _lib.oracle32_sync_update_adam.restype = ctypes.c_int
        _lib.oracle_sync_update_lars.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_int, ctypes.c_int, _vp,
                                                 _c_dbl, _c_dbl, _c_dbl, _c_dbl]
        _lib.oracle_sync_update_lars.restype = ctypes.c_int
        _lib.oracle32_accumulate_f32.argtypes = [_vp, _vp, _c_i64, _c_i64, ctypes.c_int]
        _lib.oracle32_accumulate_bf16.argtypes = [_vp, _vp, _c_i64, _c_i64, ctypes.c_int]
        _lib.oracle32_sync_update.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_int, _c_i64,
                                              _c_flt, _c_flt, _c_flt]
        _lib.oracle32_sync_update.restype = ctypes.c_int
    return _lib


def max_threads():
    return int(lib().oracle_max_threads())


def set_threads(n):
    lib().oracle_set_threads(int(n))


def _ptr(a):
    return a.ctypes.data


def _check(a, dtype):
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"] or a.ndim != 1:
        raise TypeError(f"expected 1-D contiguous {dtype}, got {a.dtype} {a.shape}")


def _grad_kind(g):
    if g.dtype == np.float32:
        return "f32"
    if g.dtype == np.uint16:
        return "bf16"  # bfloat16 bit patterns
    raise TypeError(f"gradient must be float32 or uint16 (bf16 bits), got {g.dtype}")


# ---- double family ---------------------------------------------------------

def zero(G):
    """Algorithm 1, Step 2 initialisation: G_t^i = 0."""
    _check(G, np.float64)
    lib().oracle_zero(_ptr(G), G.size)


def accumulate(G, g, M_r):
    """Algorithm 1, Step 2 inner loop: G += M_r * g for one reference batch with
    mean gradient g.  The caller keeps M_t^i += M_r."""
    _check(G, np.float64)
    kind = _grad_kind(g)
    if g.size != G.size:
        raise ValueError("size mismatch")
    if kind == "f32":
        lib().oracle_accumulate_f32(_ptr(G), _ptr(g), G.size, int(M_r))
    else:
        lib().oracle_accumulate_bf16(_ptr(G), _ptr(g), G.size, int(M_r))


def sync_update(x, v, G_list, M_list, gamma, mu, wd):
    """Algorithm 1, Step 1 (weighted average of the delayed accumulators) and
    the parameter update (momentum + weight decay around the paper's plain
    step).  Returns True when something was applied, False when sum(M) == 0."""
    _check(x, np.float64)
    _check(v, np.float64)
    N = len(G_list)
    for G in G_list:
        _check(G, np.float64)
        if G.size != x.size:
            raise ValueError("size mismatch")
    ptrs = (ctypes.c_void_p * N)(*[_ptr(G) for G in G_list])
    M = np.ascontiguousarray(np.asarray(M_list, dtype=np.int64))
    rc = lib().oracle_sync_update(_ptr(x), _ptr(v), ptrs, _ptr(M), N, x.size,
                                  float(gamma), float(mu), float(wd))
    return rc == 0


def sync_update_dc(x, x_prev, v, G_list, M_list, gamma, mu, wd, lam):
    """sync_update with the delayed gradient compensation of Algorithm 1:
    Gtilde = Gbar + lam * Gbar (.) Gbar (.) (x_t - x_{t-1}); x_prev holds x_{t-1}
    on entry and x_t on return."""
    _check(x, np.float64)
    _check(x_prev, np.float64)
    _check(v, np.float64)
    N = len(G_list)
    for G in G_list:
        _check(G, np.float64)
        if G.size != x.size:
            raise ValueError("size mismatch")
    if x_prev.size != x.size:
        raise ValueError("size mismatch")
    ptrs = (ctypes.c_void_p * N)(*[_ptr(G) for G in G_list])
    M = np.ascontiguousarray(np.asarray(M_list, dtype=np.int64))
    rc = lib().oracle_sync_update_dc(_ptr(x), _ptr(x_prev), _ptr(v), ptrs, _ptr(M), N, x.size,
                                     float(gamma), float(mu), float(wd), float(lam))
    return rc == 0


def sync_update_dcm(x, v, G_list, M_list, gamma, mu, wd, lam, gamma_prev):
    """The compensated update with x_t - x_{t-1} = -gamma_prev * v_t taken from the
    momentum instead of a stored x_{t-1}; gamma_prev = 0 when the previous
    iteration applied no update."""
    _check(x, np.float64)
    _check(v, np.float64)
    N = len(G_list)
    for G in G_list:
        _check(G, np.float64)
        if G.size != x.size:
            raise ValueError("size mismatch")
    ptrs = (ctypes.c_void_p * N)(*[_ptr(G) for G in G_list])
    M = np.ascontiguousarray(np.asarray(M_list, dtype=np.int64))
    rc = lib().oracle_sync_update_dcm(_ptr(x), _ptr(v), ptrs, _ptr(M), N, x.size, float(gamma),
                                      float(mu), float(wd), float(lam), float(gamma_prev))
    return rc == 0


def sync_update_adam(x, m, v, G_list, M_list, gamma, beta1, beta2, eps, wd, step):
    """Adam driven by the delayed weighted average (the paper's stated next step);
    step = 1, 2, ... counts the updates actually applied."""
    for a in (x, m, v):
        _check(a, np.float64)
    N = len(G_list)
    for G in G_list:
        _check(G, np.float64)
        if G.size != x.size:
            raise ValueError("size mismatch")
    ptrs = (ctypes.c_void_p * N)(*[_ptr(G) for G in G_list])
    M = np.ascontiguousarray(np.asarray(M_list, dtype=np.int64))
    rc = lib().oracle_sync_update_adam(_ptr(x), _ptr(m), _ptr(v), ptrs, _ptr(M), N, x.size, float(gamma),
                                       float(beta1), float(beta2), float(eps), float(wd), int(step))
    return rc == 0


def sync_update_lars(x, v, G_list, M_list, sizes, gamma, mu, wd, eta):
    """Layer-wise adaptive rate scaling driven by the delayed weighted average;
    sizes: elements of each consecutive layer of the flat vector.  Double only:
    there is no fixed-order fp32 restatement of the norm reductions."""
    _check(x, np.float64)
    _check(v, np.float64)
    N = len(G_list)
    for G in G_list:
        _check(G, np.float64)
        if G.size != x.size:
            raise ValueError("size mismatch")
    sz = np.ascontiguousarray(np.asarray(sizes, dtype=np.int64))
    if int(sz.sum()) != x.size or (sz < 0).any():
        raise ValueError("sizes must be non-negative and sum to the vector length")
    ptrs = (ctypes.c_void_p * N)(*[_ptr(G) for G in G_list])
    M = np.ascontiguousarray(np.asarray(M_list, dtype=np.int64))
    rc = lib().oracle_sync_update_lars(_ptr(x), _ptr(v), ptrs, _ptr(M), N, sz.size, _ptr(sz), float(gamma),
                                       float(mu), float(wd), float(eta))
    return rc == 0


# ---- fp32 family with the fixed operation order ------------------------------

def accumulate32(G, g, M_r, first):
    _check(G, np.float32)
    kind = _grad_kind(g)
    if g.size != G.size:
        raise ValueError("size mismatch")
    fn = lib().oracle32_accumulate_f32 if kind == "f32" else lib().oracle32_accumulate_bf16
    fn(_ptr(G), _ptr(g), G.size, int(M_r), 1 if first else 0)


def sync_update32(x, v, G_list, M_list, gamma, mu, wd):
    _check(x, np.float32)
    _check(v, np.float32)
    N = len(G_list)
    for G in G_list:
        _check(G, np.float32)
        if G.size != x.size:
            raise ValueError("size mismatch")
    ptrs = (ctypes.c_void_p * N)(*[_ptr(G) for G in G_list])
    M = np.ascontiguousarray(np.asarray(M_list, dtype=np.int64))
    rc = lib().oracle32_sync_update(_ptr(x), _ptr(v), ptrs, _ptr(M), N, x.size,
                                    float(np.float32(gamma)), float(np.float32(mu)),
                                    float(np.float32(wd)))
    return rc == 0


def sync_update32_dc(x, x_prev, v, G_list, M_list, gamma, mu, wd, lam):
    _check(x, np.float32)
    _check(x_prev, np.float32)
    _check(v, np.float32)
    N = len(G_list)
    for G in G_list:
        _check(G, np.float32)
        if G.size != x.size:
            raise ValueError("size mismatch")
    ptrs = (ctypes.c_void_p * N)(*[_ptr(G) for G in G_list])
    M = np.ascontiguousarray(np.asarray(M_list, dtype=np.int64))
    f = lambda t: float(np.float32(t))
    rc = lib().oracle32_sync_update_dc(_ptr(x), _ptr(x_prev), _ptr(v), ptrs, _ptr(M), N, x.size,
                                       f(gamma), f(mu), f(wd), f(lam))
    return rc == 0


def sync_update32_dcm(x, v, G_list, M_list, gamma, mu, wd, lam, gamma_prev):
    _check(x, np.float32)
    _check(v, np.float32)
    N = len(G_list)
    for G in G_list:
        _check(G, np.float32)
        if G.size != x.size:
            raise ValueError("size mismatch")
    ptrs = (ctypes.c_void_p * N)(*[_ptr(G) for G in G_list])
    M = np.ascontiguousarray(np.asarray(M_list, dtype=np.int64))
    f = lambda t: float(np.float32(t))
    rc = lib().oracle32_sync_update_dcm(_ptr(x), _ptr(v), ptrs, _ptr(M), N, x.size, f(gamma), f(mu),
                                        f(wd), f(lam), f(gamma_prev))
    return rc == 0


def sync_update32_adam(x, m, v, G_list, M_list, gamma, beta1, beta2, eps, wd, step):
    for a in (x, m, v):
        _check(a, np.float32)
    N = len(G_list)
    for G in G_list:
        _check(G, np.float32)
        if G.size != x.size:
            raise ValueError("size mismatch")
    ptrs = (ctypes.c_void_p * N)(*[_ptr(G) for G in G_list])
    M = np.ascontiguousarray(np.asarray(M_list, dtype=np.int64))
    f = lambda t: float(np.float32(t))
    rc = lib().oracle32_sync_update_adam(_ptr(x), _ptr(m), _ptr(v), ptrs, _ptr(M), N, x.size, f(gamma),
                                         f(beta1), f(beta2), f(eps), f(wd), int(step))
    return rc == 0


# ---- Algorithm 1, whole loop --------------------------------------------------

def run(x0, N, T, M_r, gamma, mu, wd, batches, precision="f64", record=None, lam=None, adam=None,
        lars=None, lam_from_momentum=False):
    """Run T iterations of Algorithm 1 on the flat parameter vector x0.

    batches(t, i) -> list of mean-gradient vectors (float32 or bf16 bits), one
    per reference batch worker i processed in iteration t (its length is the
    adaptive part: it is whatever the caller's schedule says).

    Each iteration, in the paper's order: Step 2 builds the generation-t
    accumulators from zero; Step 1 averages generation t-1 and the update is
    applied to x_t; then t advances.  Step 1 and Step 2 touch disjoint data, so
    running them one after the other here equals running them in parallel.
    The last generation is accumulated and never applied (the loop returns x_T).

    precision "f64": the definition in double.  "f32": the fixed-order fp32
    restatement.  lam: compensation coefficient lambda; None leaves the
    compensation line of Algorithm 1 out (then no x_{t-1} is kept).
    lam_from_momentum: form x_t - x_{t-1} as -gamma_{t-1} * v_t instead of from a
    stored x_{t-1}.
    adam: (beta1, beta2, eps) switches the update rule to Adam (mu is unused,
    the returned "v" is then the pair (m, v)).
    lars: (sizes, eta) switches it to LARS over those layers (double only).
    Returns (x_T, v_T, M_history[T][N]).  record(t, x, v) is called after each
    iteration when given.
    """
    if precision == "f64":
        ft, upd_fn = np.float64, sync_update
    elif precision == "f32":
        ft, upd_fn = np.float32, sync_update32
    else:
        raise ValueError(precision)
    P = x0.size
    x = np.array(x0, dtype=ft)
    x_prev = x.copy()                  # no update applied yet: x_t - x_{t-1} = 0
    v = np.zeros(P, dtype=ft)
    G = [[np.zeros(P, dtype=ft) for _ in range(N)] for _ in range(2)]
    M = [[0] * N for _ in range(2)]   # G_{-1} = 0; its batch sizes are 0
    cur, prev = 0, 1
    history = []
    gamma_prev = 0.0                   # step size of the previous applied update
    if adam is not None:
        m1 = np.zeros(P, dtype=ft)
        applied = 0
    for t in range(T):
        # Step 2: accumulate generation t (at x_t)
        for i in range(N):
            # initialisation G_t^i = 0, M_t^i = 0.  The double family zeroes the
            # accumulator; the fp32 family's first reference batch overwrites it
            # instead (`first`), so whatever the buffer still holds is never read.
            if precision == "f64":
                zero(G[cur][i])
            M[cur][i] = 0
            for g in batches(t, i):
                if precision == "f64":
                    accumulate(G[cur][i], g, M_r)
                else:
                    accumulate32(G[cur][i], g, M_r, first=(M[cur][i] == 0))
                M[cur][i] += M_r
        # Step 1 + update: apply generation t-1 to x_t
        if lars is not None:
            if precision != "f64":
                raise ValueError("LARS has no fixed-order fp32 restatement")
            sync_update_lars(x, v, G[prev], M[prev], lars[0], gamma, mu, wd, lars[1])
        elif adam is not None:
            fn = sync_update_adam if precision == "f64" else sync_update32_adam
            if fn(x, m1, v, G[prev], M[prev], gamma, adam[0], adam[1], adam[2], wd, applied + 1):
                applied += 1
        elif lam is None:
            upd_fn(x, v, G[prev], M[prev], gamma, mu, wd)
        elif lam_from_momentum:
            fn = sync_update_dcm if precision == "f64" else sync_update32_dcm
            gamma_prev = gamma if fn(x, v, G[prev], M[prev], gamma, mu, wd, lam, gamma_prev) else 0.0
        elif precision == "f64":
            sync_update_dc(x, x_prev, v, G[prev], M[prev], gamma, mu, wd, lam)
        else:
            sync_update32_dc(x, x_prev, v, G[prev], M[prev], gamma, mu, wd, lam)
        history.append(list(M[cur]))
        if record is not None:
            record(t, x, v)
        cur, prev = prev, cur
    if adam is not None:
        return x, (m1, v), history
    return x, v, history
