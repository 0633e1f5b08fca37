"""CPU checker for the scheduling round: test infrastructure only.

Thin numpy/ctypes front end of oracle.c.  Only the tests, the smoke check and
the benchmark's CPU-baseline leg may import this package; the GPU library and
its Python binding never do.
"""
import ctypes as C
import os

import numpy as np

from .build import LIB, LIB_SAN, build

INFEASIBLE = np.int32(-2147483648)
_lib = None

_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")


def lib():
    global _lib
    if _lib is None:
        sanitized = os.environ.get("ORACLE_SANITIZED") == "1"
        path = LIB_SAN if sanitized else LIB
        if not os.path.exists(path):
            build(sanitize=sanitized)
        _lib = C.CDLL(path)
        _lib.orc_score_pairs.restype = C.c_int
        _lib.orc_score_pairs.argtypes = [_f32p, C.c_int, _f32p, C.c_int, C.c_int, C.c_int,
                                         _f32p, _f32p, _f32p, _f32p, _f32p, _f32p, C.c_float,
                                         C.c_int, C.c_float, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        _lib.orc_max_weight_matching.restype = C.c_int
        _lib.orc_max_weight_matching.argtypes = [_i32p, C.c_int, C.c_int, C.c_int64, _i32p, _i64p,
                                                 _i64p, C.POINTER(C.c_int64)]
        _lib.orc_brute_force.restype = C.c_int
        _lib.orc_brute_force.argtypes = [_i32p, C.c_int, C.c_int, C.c_int64, _i32p,
                                         C.POINTER(C.c_int64)]
        _lib.orc_check_certificate.restype = C.c_int
        _lib.orc_check_certificate.argtypes = [_i32p, C.c_int, C.c_int, C.c_int64, _i32p, _i64p,
                                               _i64p, C.c_int64, C.POINTER(C.c_int64),
                                               C.POINTER(C.c_int64)]
        _lib.orc_threads.restype = C.c_int
    return _lib


def threads():
    return int(lib().orc_threads())


def score_pairs(x_on, x_off, params, scale, mem_feature=0, mem_limit=1.0, wide=True, nthreads=0, sm=None,
                slow_limit=None):
    """Scores and quantised weights for every (online, offline) pair.

    sm = (online feature, offline feature): the SM share depends on the pair,
    sm(u, v) = min(1 - x_u[online feature], x_v[offline feature]), and is a third input of the
    predictor; params["W1"] then has 2F + 1 columns.
    slow_limit: the predictor has a second output unit, params["W3slow"], params["b3slow"], on the
    same hidden layers: the predicted slowdown of the pair's online workload (paper: Section
    "Lessons and future direction", the threshold on the online workloads' degradation); pairs
    predicted above slow_limit are infeasible.  It is the scorer run once more with that unit's
    output weights, then a comparison.
    Returns (sigma float32 [n,m], W int32 [n,m]); masked pairs hold INFEASIBLE in W."""
    if slow_limit is not None:
        main = {k: v for k, v in params.items() if k not in ("W3slow", "b3slow")}
        unit = dict(main, W3=params["W3slow"], b3=params["b3slow"])
        sigma, w = score_pairs(x_on, x_off, main, scale, mem_feature, mem_limit, wide, nthreads, sm)
        slow = score_pairs(x_on, x_off, unit, scale, mem_feature, mem_limit, wide, nthreads, sm)[0]
        w[slow > np.float32(slow_limit)] = INFEASIBLE
        return sigma, w
    x_on = np.ascontiguousarray(x_on, np.float32)
    x_off = np.ascontiguousarray(x_off, np.float32)
    n, F = x_on.shape
    m = x_off.shape[0]
    assert x_off.shape[1] == F
    p = {k: np.ascontiguousarray(v, np.float32) for k, v in params.items()}
    H = p["b1"].shape[0]
    sm_on, sm_off = (-1, -1) if sm is None else (int(sm[0]), int(sm[1]))
    assert p["W1"].shape == (H, 2 * F + (sm is not None)) and p["W2"].shape == (H, H) and p["W3"].shape == (H,)
    sigma = np.empty((n, m), np.float32)
    w = np.empty((n, m), np.int32)
    rc = lib().orc_score_pairs(x_on, n, x_off, m, F, H, p["W1"], p["b1"], p["W2"], p["b2"],
                               p["W3"], p["b3"], float(scale), int(mem_feature), float(mem_limit),
                               sm_on, sm_off, 1 if wide else 0, int(nthreads), sigma.ctypes.data, w.ctypes.data)
    if rc != 0:
        raise ValueError("orc_score_pairs: bad arguments")
    return sigma, w


def score_pairs_typed(x_on, x_off, params_by_type, type_on, scale, mem_feature=0, mem_limit=1.0, wide=True):
    """One predictor per GPU type (paper: Section "Matching-based scheduling", an MLP per GPU
    type): row i of the result is row i of score_pairs under params_by_type[type_on[i]]."""
    x_on = np.ascontiguousarray(x_on, np.float32)
    type_on = np.asarray(type_on)
    n, m = x_on.shape[0], np.asarray(x_off).shape[0]
    sigma = np.empty((n, m), np.float32)
    w = np.empty((n, m), np.int32)
    for t, params in enumerate(params_by_type):
        rows = np.nonzero(type_on == t)[0]
        if len(rows):
            sigma[rows], w[rows] = score_pairs(x_on[rows], x_off, params, scale, mem_feature, mem_limit, wide)
    if ((type_on < 0) | (type_on >= len(params_by_type))).any():
        raise ValueError("score_pairs_typed: type out of range")
    return sigma, w


def max_weight_matching(W):
    """Exact optimum: returns (total, row2col, u, v)."""
    W = np.ascontiguousarray(W, np.int32)
    n, m = W.shape
    r2c = np.empty(n, np.int32)
    u = np.empty(n, np.int64)
    v = np.empty(m, np.int64)
    tot = C.c_int64(0)
    rc = lib().orc_max_weight_matching(W, n, m, m, r2c, u, v, C.byref(tot))
    if rc != 0:
        raise ValueError("orc_max_weight_matching: needs n <= m")
    return int(tot.value), r2c, u, v


def brute_force(W):
    """Optimum by exhaustive enumeration (n <= m <= 10): returns (total, row2col)."""
    W = np.ascontiguousarray(W, np.int32)
    n, m = W.shape
    r2c = np.empty(max(n, 1), np.int32)
    tot = C.c_int64(0)
    rc = lib().orc_brute_force(W, n, m, m, r2c, C.byref(tot))
    if rc != 0:
        raise ValueError("orc_brute_force: needs n, m <= 10")
    return int(tot.value), r2c[:n]


def check_certificate(W, row2col, u, v, K=1):
    """Returns (code, primal, dual); code 0 = the matching is proved optimal."""
    W = np.ascontiguousarray(W, np.int32)
    n, m = W.shape
    P, D = C.c_int64(0), C.c_int64(0)
    rc = lib().orc_check_certificate(W, n, m, m, np.ascontiguousarray(row2col, np.int32),
                                     np.ascontiguousarray(u, np.int64),
                                     np.ascontiguousarray(v, np.int64), int(K),
                                     C.byref(P), C.byref(D))
    return int(rc), int(P.value), int(D.value)
