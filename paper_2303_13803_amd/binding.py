"""Thin ctypes binding over libmuxmatch.so: argument marshalling only.

Every step of the scheduling round runs inside the library's HIP kernels;
torch is used here for device buffers and the stream handle, nothing else.
There is no CPU fallback: if the shared library is missing, importing this
module raises.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmuxmatch.so")

INFEASIBLE = -2147483648
OK, ERR_ARG, ERR_SHAPE, ERR_HIP, ERR_NOT_CONVERGED, ERR_CERT, ERR_RANGE = 0, -1, -2, -3, -4, -5, -6
FALLBACK_TEAMS, FALLBACK_SEARCHES = 1, 2

EXPORTS = ["mf_create", "mf_destroy", "mf_score_pairs", "mf_solve_assignment",
           "mf_check_certificate", "mf_check_certificate_noalloc", "mf_schedule_round", "mf_schedule_round_update", "mf_score_pairs_typed",
           "mf_schedule_round_typed", "mf_set_option", "mf_last_timings", "mf_measure_ceilings",
           "mf_strerror", "mf_last_hip_error"]

TIMING_NAMES = ["projections_ms", "pair_scoring_ms", "bulk_bid_ms", "bulk_bid_launches",
                "prepare_ms", "duals_ms", "certificate_ms", "auction_ms", "bulk_bid_bytes",
                "pairs_evaluated_fraction"]


class Predictor(C.Structure):
    _fields_ = [("F", C.c_int32), ("H", C.c_int32), ("scale", C.c_float),
                ("mem_feature", C.c_int32), ("mem_limit", C.c_float),
                ("d_W1", C.c_void_p), ("d_b1", C.c_void_p), ("d_W2", C.c_void_p),
                ("d_b2", C.c_void_p), ("d_W3", C.c_void_p), ("d_b3", C.c_void_p),
                ("d_W1sm", C.c_void_p), ("sm_on_feature", C.c_int32), ("sm_off_feature", C.c_int32),
                ("d_W3_slow", C.c_void_p), ("d_b3_slow", C.c_void_p), ("slow_limit", C.c_float)]


class Result(C.Structure):
    _fields_ = [("primal", C.c_int64), ("dual", C.c_int64), ("K", C.c_int64),
                ("min_reduced_cost", C.c_int64), ("rounds", C.c_int64), ("bids", C.c_int64),
                ("bytes_scanned", C.c_int64), ("chain_bids", C.c_int64), ("chain_depth", C.c_int64),
                ("chain_retries", C.c_int64), ("team_bids", C.c_int64), ("path_steps", C.c_int64),
                ("path_scans", C.c_int64),
                ("matched", C.c_int32), ("phases", C.c_int32),
                ("cert_ok", C.c_int32), ("status", C.c_int32), ("ms_solve", C.c_float),
                ("ms_certify", C.c_float), ("fallbacks", C.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class Certificate(C.Structure):
    _fields_ = [("primal", C.c_int64), ("dual", C.c_int64), ("K", C.c_int64), ("min_reduced_cost", C.c_int64),
                ("matched", C.c_int32), ("flags", C.c_int32), ("cert_ok", C.c_int32), ("reserved", C.c_int32)]


NOALLOC_MAX_COLS = 65536


def load_library():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2303_13803_amd/build.py` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    lib.mf_create.argtypes = [C.POINTER(vp), i32, vp, i32, i32]
    lib.mf_destroy.argtypes = [vp]
    lib.mf_score_pairs.argtypes = [vp, C.POINTER(Predictor), vp, i32, vp, i32, vp, i64, vp]
    lib.mf_solve_assignment.argtypes = [vp, vp, i32, i32, i64, vp, vp, vp, C.POINTER(Result)]
    lib.mf_check_certificate.argtypes = [vp, vp, i32, i32, i64, vp, vp, vp, i64, C.POINTER(Result)]
    lib.mf_check_certificate_noalloc.argtypes = [vp, vp, i32, i32, i64, vp, vp, vp, i64, vp]
    lib.mf_schedule_round.argtypes = [vp, C.POINTER(Predictor), vp, i32, vp, i32, vp, i64, vp, vp, vp,
                                      C.POINTER(Result)]
    lib.mf_schedule_round_update.argtypes = [vp, C.POINTER(Predictor), vp, i32, vp, i32, vp, i32, vp, i32, vp, i64,
                                             vp, vp, vp, C.POINTER(Result)]
    lib.mf_score_pairs_typed.argtypes = [vp, C.POINTER(Predictor), i32, vp, vp, i32, vp, i32, vp, i64, vp]
    lib.mf_schedule_round_typed.argtypes = [vp, C.POINTER(Predictor), i32, vp, vp, i32, vp, i32, vp, i64, vp, vp, vp,
                                            C.POINTER(Result)]
    lib.mf_measure_ceilings.argtypes = [vp, vp, i64, C.POINTER(C.c_float * 8)]
    lib.mf_set_option.argtypes = [vp, C.c_char_p, i64]
    lib.mf_last_timings.argtypes = [vp, C.POINTER(C.c_float * 16)]
    lib.mf_strerror.argtypes = [i32]
    lib.mf_strerror.restype = C.c_char_p
    lib.mf_last_hip_error.argtypes = [vp]
    lib.mf_last_hip_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("mf_strerror", "mf_last_hip_error"):
            getattr(lib, name).restype = i32
    return lib


_lib = load_library()


class MuxmatchError(RuntimeError):
    def __init__(self, code, detail=""):
        self.code = code
        super().__init__(f"muxmatch error {code}: {_lib.mf_strerror(code).decode()} {detail}".strip())


def _ptr(t, dtype):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"expected a contiguous device tensor of {dtype}")
    return t.data_ptr()


class Context:
    """Owns the library's scratch for problems up to max_n x max_m on one device."""

    def __init__(self, max_n, max_m, device=0, stream=None):
        self.device = int(device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        handle = C.c_void_p()
        rc = _lib.mf_create(C.byref(handle), self.device, C.c_void_p(self.stream.cuda_stream),
                            int(max_n), int(max_m))
        if rc != OK:
            raise MuxmatchError(rc)
        self._h = handle
        self._keep = None

    def close(self):
        if getattr(self, "_h", None):
            _lib.mf_destroy(self._h)
            self._h = None

    __del__ = close

    def _check(self, rc, allow=()):
        if rc != OK and rc not in allow:
            detail = _lib.mf_last_hip_error(self._h).decode() if rc == ERR_HIP else ""
            raise MuxmatchError(rc, detail)
        return rc

    def predictor(self, params, scale, mem_feature=0, mem_limit=1.0, sm=None, slow_limit=None):
        """params: dict of float32 device tensors W1 [H,2F], b1, W2 [H,H], b2, W3 [H], b3 [1];
        with sm = (online feature, offline feature) also W1sm [H], the weights of the
        pair-dependent SM input; with slow_limit also W3slow [H], b3slow [1], the second output
        unit that predicts the online workload's slowdown (pairs above slow_limit are infeasible)."""
        H = params["b1"].numel()
        F = params["W1"].shape[1] // 2
        p = Predictor(F, H, float(scale), int(mem_feature), float(mem_limit),
                      *[_ptr(params[k], torch.float32) for k in ("W1", "b1", "W2", "b2", "W3", "b3")],
                      _ptr(params["W1sm"], torch.float32) if sm is not None else None,
                      0 if sm is None else int(sm[0]), 0 if sm is None else int(sm[1]),
                      _ptr(params["W3slow"], torch.float32) if slow_limit is not None else None,
                      _ptr(params["b3slow"], torch.float32) if slow_limit is not None else None,
                      0.0 if slow_limit is None else float(slow_limit))
        p._keep = params
        return p

    def set_option(self, name, value):
        self._check(_lib.mf_set_option(self._h, name.encode(), int(value)))

    def score_pairs(self, pred, x_on, x_off, W, sigma=None):
        n, m = x_on.shape[0], x_off.shape[0]
        self._check(_lib.mf_score_pairs(self._h, C.byref(pred), _ptr(x_on, torch.float32), n,
                                        _ptr(x_off, torch.float32), m, _ptr(W, torch.int32),
                                        W.stride(0), _ptr(sigma, torch.float32)))

    def solve_assignment(self, W, n, m, row2col, u, v, allow_cert_failure=False):
        res = Result()
        rc = _lib.mf_solve_assignment(self._h, _ptr(W, torch.int32), n, m, W.stride(0),
                                      _ptr(row2col, torch.int32), _ptr(u, torch.int64),
                                      _ptr(v, torch.int64), C.byref(res))
        self._check(rc, allow=(ERR_CERT,) if allow_cert_failure else ())
        return res

    def check_certificate(self, W, n, m, row2col, u, v, K):
        res = Result()
        self._check(_lib.mf_check_certificate(self._h, _ptr(W, torch.int32), n, m, W.stride(0),
                                              _ptr(row2col, torch.int32), _ptr(u, torch.int64),
                                              _ptr(v, torch.int64), int(K), C.byref(res)))
        return res

    def schedule_round(self, pred, x_on, x_off, W, row2col, u, v):
        n, m = x_on.shape[0], x_off.shape[0]
        res = Result()
        self._check(_lib.mf_schedule_round(self._h, C.byref(pred), _ptr(x_on, torch.float32), n,
                                           _ptr(x_off, torch.float32), m, _ptr(W, torch.int32),
                                           W.stride(0), _ptr(row2col, torch.int32),
                                           _ptr(u, torch.int64), _ptr(v, torch.int64), C.byref(res)))
        return res

    def schedule_round_update(self, pred, x_on, x_off, changed_on, changed_off, W, row2col, u, v):
        n, m = x_on.shape[0], x_off.shape[0]
        res = Result()
        self._check(_lib.mf_schedule_round_update(
            self._h, C.byref(pred), _ptr(x_on, torch.float32), n, _ptr(x_off, torch.float32), m,
            _ptr(changed_on, torch.int32) if changed_on is not None and changed_on.numel() else None,
            0 if changed_on is None else changed_on.numel(),
            _ptr(changed_off, torch.int32) if changed_off is not None and changed_off.numel() else None,
            0 if changed_off is None else changed_off.numel(),
            _ptr(W, torch.int32), W.stride(0), _ptr(row2col, torch.int32), _ptr(u, torch.int64),
            _ptr(v, torch.int64), C.byref(res)))
        return res

    def score_pairs_typed(self, preds, type_on, x_on, x_off, W, sigma=None):
        """preds: list of predictors, one per GPU type; type_on: int32 device tensor [n]."""
        n, m = x_on.shape[0], x_off.shape[0]
        arr = (Predictor * len(preds))(*preds)
        self._check(_lib.mf_score_pairs_typed(self._h, arr, len(preds), _ptr(type_on, torch.int32),
                                              _ptr(x_on, torch.float32), n, _ptr(x_off, torch.float32), m,
                                              _ptr(W, torch.int32), W.stride(0), _ptr(sigma, torch.float32)))

    def schedule_round_typed(self, preds, type_on, x_on, x_off, W, row2col, u, v):
        n, m = x_on.shape[0], x_off.shape[0]
        arr = (Predictor * len(preds))(*preds)
        res = Result()
        self._check(_lib.mf_schedule_round_typed(
            self._h, arr, len(preds), _ptr(type_on, torch.int32), _ptr(x_on, torch.float32), n,
            _ptr(x_off, torch.float32), m, _ptr(W, torch.int32), W.stride(0), _ptr(row2col, torch.int32),
            _ptr(u, torch.int64), _ptr(v, torch.int64), C.byref(res)))
        return res

    def measure_ceilings(self, buffer=None):
        """Measured fp32 and fp16 MFMA rates (TFLOP/s) and, with a device tensor, streaming read rate (GB/s)."""
        arr = (C.c_float * 8)()
        nbytes = 0 if buffer is None else buffer.numel() * buffer.element_size()
        self._check(_lib.mf_measure_ceilings(self._h, None if buffer is None else buffer.data_ptr(), nbytes,
                                             C.byref(arr)))
        return {"mfma_f32_tflops": float(arr[0]), "read_gbps": float(arr[2]), "mfma_f16_tflops": float(arr[4])}

    def last_timings(self):
        arr = (C.c_float * 16)()
        self._check(_lib.mf_last_timings(self._h, C.byref(arr)))
        return {name: float(arr[i]) for i, name in enumerate(TIMING_NAMES)}


def check_certificate_noalloc(W, n, m, row2col, u, v, K, out, stream=None):
    """mf_check_certificate_noalloc on the current device: `out` is a uint8 device tensor of
    ctypes.sizeof(Certificate) bytes that receives the result once `stream` gets there
    (read it with read_certificate after synchronising).  Returns the call's status code."""
    if not out.is_cuda or out.dtype != torch.uint8 or out.numel() < C.sizeof(Certificate) or not out.is_contiguous():
        raise TypeError("out: a contiguous uint8 device tensor of at least sizeof(Certificate) bytes")
    s = stream if stream is not None else torch.cuda.current_stream()
    return _lib.mf_check_certificate_noalloc(C.c_void_p(s.cuda_stream), _ptr(W, torch.int32), int(n), int(m),
                                             W.stride(0), _ptr(row2col, torch.int32), _ptr(u, torch.int64),
                                             _ptr(v, torch.int64), int(K), out.data_ptr())


def read_certificate(out):
    """The Certificate a finished mf_check_certificate_noalloc left in `out` (copies it to the host)."""
    return Certificate.from_buffer_copy(out.cpu().numpy().tobytes()[:C.sizeof(Certificate)])


def strerror(code):
    return _lib.mf_strerror(int(code)).decode()


def raw_library():
    return _lib
