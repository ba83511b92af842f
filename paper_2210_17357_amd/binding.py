"""ctypes binding of liblgreco.so: argument marshalling only.  Function names and argument
order follow include/lgreco.h.  Device buffers are torch CUDA(ROCm) tensors (PyTorch is used
for device memory and streams only); host tables are numpy arrays.

The library is loaded on first use and a missing library is an error: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblgreco.so")

OK, EINVAL, ENOSPACE, EINFEASIBLE, EHIP, EUNSUPPORTED = 0, -1, -2, -3, -4, -5
QUANT, TOPK, LOWRANK = 0, 1, 2
CALL_PROFILE, CALL_SOLVE, CALL_COMPRESS, CALL_RECEIVE = 0, 1, 2, 3

EXPORTS = ("lgreco_create", "lgreco_destroy", "lgreco_sizes", "lgreco_profile", "lgreco_profile_solve", "lgreco_profile_solve_compress",
           "lgreco_candidate_range", "lgreco_emax",
           "lgreco_solve", "lgreco_solve_static", "lgreco_solve_weighted", "lgreco_payload_layout", "lgreco_compress", "lgreco_decompress", "lgreco_accumulate", "lgreco_set_timing", "lgreco_set_timing_stride",
           "lgreco_get_timing", "lgreco_get_timing_of", "lgreco_get_timing_totals", "lgreco_strerror", "lgreco_last_hip_error", "lgreco_last_solve_groups",
           "lgreco_set_ef_zero_on_entry", "lgreco_late_handovers")


class Layer(C.Structure):
    _fields_ = [("offset", C.c_int64), ("numel", C.c_int64), ("rows", C.c_int32), ("cols", C.c_int32)]


class Cand(C.Structure):
    _fields_ = [("family", C.c_int32), ("reserved", C.c_int32), ("param", C.c_double)]


class Config(C.Structure):
    _fields_ = [("bucket", C.c_int32), ("stochastic", C.c_int32), ("seed", C.c_uint64),
                ("power_iters", C.c_int32), ("r_max", C.c_int32), ("reuse_thresholds", C.c_int32),
                ("dp_groups", C.c_int32), ("strict_budget", C.c_int32),
                ("keep_ef_on_failure", C.c_int32)]


class LgrecoError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("lgreco status %d: %s" % (status, text))
        self.status = status


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("liblgreco.so is not built: run `python -m paper_2210_17357_amd.build` "
                               "(there is no CPU fallback)")
        # PyTorch ships its own HIP runtime; load it first so that this library binds to the
        # same runtime instance (two runtimes in one process do not share the device).
        import torch  # noqa: F401
        l = C.CDLL(LIB_PATH)
        vp, i32, i64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
        l.lgreco_create.argtypes = [C.POINTER(vp), C.POINTER(Config), i64, i32, i32]
        l.lgreco_destroy.argtypes = [vp]
        l.lgreco_sizes.argtypes = [vp, i32, vp, i32, i32, vp]
        l.lgreco_profile.argtypes = [vp, vp, vp, vp, i32, vp, i32, vp, vp, vp, vp]
        l.lgreco_profile_solve.argtypes = [vp, vp, vp, vp, i32, vp, i32, vp, i32, i32, vp, vp, C.POINTER(dbl), vp,
                                           C.POINTER(i64), C.POINTER(dbl), vp]
        l.lgreco_profile_solve_compress.argtypes = [vp, vp, vp, vp, i32, vp, i32, vp, i32, i32, vp, vp,
                                                    C.POINTER(dbl), vp, C.POINTER(i64), C.POINTER(dbl), vp, i64, vp,
                                                    vp]
        l.lgreco_candidate_range.argtypes = [i32, dbl, i32, vp, i32, C.POINTER(i32), C.POINTER(i32)]
        l.lgreco_emax.argtypes = [vp, i32, i32, i32, C.POINTER(dbl)]
        l.lgreco_solve.argtypes = [vp, vp, vp, i32, i32, dbl, i32, vp, C.POINTER(i64), C.POINTER(dbl), vp]
        l.lgreco_solve_weighted.argtypes = [vp, vp, vp, vp, i32, i32, dbl, i32, vp, C.POINTER(i64),
                                            C.POINTER(i64), C.POINTER(dbl), vp]
        l.lgreco_solve_static.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp]
        l.lgreco_payload_layout.argtypes = [vp, i32, vp, i32, vp, i32, vp]
        l.lgreco_compress.argtypes = [vp, vp, vp, vp, i32, vp, i32, vp, vp, vp, vp, vp]
        l.lgreco_decompress.argtypes = [vp, vp, vp, vp, i32, vp, i32, vp, vp, i32, vp]
        l.lgreco_accumulate.argtypes = [vp, vp, vp, i64, i32, vp]
        l.lgreco_set_timing.argtypes = [vp, i32]
        l.lgreco_set_timing_stride.argtypes = [vp, i32]
        l.lgreco_get_timing.argtypes = [vp, vp, vp, i32]
        l.lgreco_get_timing_of.argtypes = [vp, i32, vp, vp, i32]
        l.lgreco_get_timing_totals.argtypes = [vp, i32, vp, vp, vp, i32]
        l.lgreco_strerror.argtypes = [C.c_int]
        l.lgreco_strerror.restype = C.c_char_p
        l.lgreco_last_solve_groups.argtypes = [vp]
        l.lgreco_set_ef_zero_on_entry.argtypes = [vp, C.c_int32]
        l.lgreco_late_handovers.argtypes = [vp]
        l.lgreco_late_handovers.restype = C.c_int64
        l.lgreco_last_hip_error.argtypes = [vp]
        l.lgreco_last_hip_error.restype = C.c_char_p
        for name in EXPORTS:
            if getattr(l, name).restype is C.c_int:
                pass
        _lib = l
    return _lib


def strerror(status: int) -> str:
    return lib().lgreco_strerror(status).decode()


def layer_table(offsets, numels, rows, cols):
    n = len(numels)
    arr = (Layer * n)()
    for i in range(n):
        arr[i] = Layer(int(offsets[i]), int(numels[i]), int(rows[i]), int(cols[i]))
    return arr


def cand_table(cands: Sequence[Tuple[int, float]]):
    arr = (Cand * len(cands))()
    for i, (f, p) in enumerate(cands):
        arr[i] = Cand(int(f), 0, float(p))
    return arr


def _dptr(t) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


def _stream(stream=None) -> int:
    """The HIP stream handle to pass on: the one given, else torch's current stream."""
    if stream is not None:
        return int(stream)
    import torch
    return torch.cuda.current_stream().cuda_stream


def _np(a) -> int:
    return a.ctypes.data


def sizes(layers, cands, bucket: int = 128) -> np.ndarray:
    out = np.zeros((len(layers), len(cands)), np.int64)
    st = lib().lgreco_sizes(C.addressof(layers), len(layers), C.addressof(cands), len(cands), bucket, _np(out))
    if st != OK:
        raise LgrecoError(st, strerror(st))
    return out


def candidate_range(family: int, default_param: float, r_max: int = 0):
    """[(family, parameter)] of the paper's range rule and the index of the default in it."""
    cap = 128
    arr = (Cand * cap)()
    n, d = C.c_int32(), C.c_int32()
    st = lib().lgreco_candidate_range(int(family), float(default_param), int(r_max), C.addressof(arr), cap,
                                      C.byref(n), C.byref(d))
    if st != OK:
        raise LgrecoError(st, strerror(st))
    return [(arr[i].family, arr[i].param) for i in range(n.value)], d.value


def emax(errors: np.ndarray, default_cand: int) -> float:
    errors = np.ascontiguousarray(errors, np.float64)
    v = C.c_double()
    st = lib().lgreco_emax(_np(errors), errors.shape[0], errors.shape[1], default_cand, C.byref(v))
    if st != OK:
        raise LgrecoError(st, strerror(st))
    return v.value


def payload_layout(layers, cands, choice: np.ndarray, bucket: int = 128) -> np.ndarray:
    choice = np.ascontiguousarray(choice, np.int32)
    out = np.zeros(len(layers) + 1, np.int64)
    st = lib().lgreco_payload_layout(C.addressof(layers), len(layers), C.addressof(cands), len(cands),
                                     _np(choice), bucket, _np(out))
    if st != OK:
        raise LgrecoError(st, strerror(st))
    return out


def solve_static(d_errors, d_sizes, default_cand: int, n_bins: int, d_choice, d_result, stream=None) -> int:
    """lgreco_solve_static: device tables in, device choice [L] (int32) and result [4] (int64) out;
    nothing is allocated, nothing waits.  Returns the status (OK = queued)."""
    L, P = d_errors.shape
    return lib().lgreco_solve_static(_dptr(d_errors), _dptr(d_sizes), int(L), int(P), int(default_cand),
                                     int(n_bins), _dptr(d_choice), _dptr(d_result), _stream(stream))


class Handle:
    """lgreco_handle_t with the entry points as methods."""

    def __init__(self, max_elems: int, max_layers: int, max_cands: int, bucket: int = 128,
                 stochastic: bool = False, seed: int = 0, power_iters: int = 1, r_max: int = 64,
                 reuse_thresholds: bool = False, dp_groups: int = 0, strict_budget: bool = False,
                 keep_ef_on_failure: bool = False):
        self._h = C.c_void_p()
        self.cfg = Config(bucket, int(stochastic), seed, power_iters, r_max, int(bool(reuse_thresholds)),
                          int(dp_groups), int(bool(strict_budget)), int(bool(keep_ef_on_failure)))
        st = lib().lgreco_create(C.byref(self._h), C.byref(self.cfg), max_elems, max_layers, max_cands)
        if st != OK:
            raise LgrecoError(st, strerror(st))

    def close(self):
        if self._h:
            lib().lgreco_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int, allow=()):
        if st != OK and st not in allow:
            text = strerror(st)
            if st == EHIP:
                text += " (" + lib().lgreco_last_hip_error(self._h).decode() + ")"
            raise LgrecoError(st, text)
        return st

    # Every GPU entry point takes `stream`: a HIP stream handle (int); default: torch's current stream.

    def profile(self, d_grads, d_ef, layers, cands, d_q0=None, want_sizes: bool = True, stream=None):
        L, P = len(layers), len(cands)
        errors = np.zeros((L, P), np.float64)
        szs = np.zeros((L, P), np.int64) if want_sizes else None
        st = lib().lgreco_profile(self._h, _dptr(d_grads), _dptr(d_ef), C.addressof(layers), L,
                                  C.addressof(cands), P, _dptr(d_q0), _np(errors),
                                  _np(szs) if want_sizes else None, _stream(stream))
        self._check(st)
        return errors, szs

    def profile_solve(self, d_grads, d_ef, layers, cands, default_cand: int, n_bins: int, d_q0=None,
                      stream=None):
        """profile + emax + solve in one call: (status, errors, sizes, e_max, choice, total_size,
        total_error); status is OK or EINFEASIBLE."""
        L, P = len(layers), len(cands)
        errors = np.zeros((L, P), np.float64)
        szs = np.zeros((L, P), np.int64)
        choice = np.zeros(L, np.int32)
        e_max, tsize, terr = C.c_double(), C.c_int64(), C.c_double()
        st = lib().lgreco_profile_solve(self._h, _dptr(d_grads), _dptr(d_ef), C.addressof(layers), L,
                                        C.addressof(cands), P, _dptr(d_q0), int(default_cand), int(n_bins),
                                        _np(errors), _np(szs), C.byref(e_max), _np(choice), C.byref(tsize),
                                        C.byref(terr), _stream(stream))
        self._check(st, allow=(EINFEASIBLE,))
        return st, errors, szs, e_max.value, choice, tsize.value, terr.value

    def profile_solve_compress(self, d_grads, d_ef, layers, cands, default_cand: int, n_bins: int, d_payload,
                               d_q=None, stream=None):
        """The whole path as one call: (status, errors, sizes, e_max, choice, total_size,
        total_error, offsets); the compression kernels are queued when it returns."""
        L, P = len(layers), len(cands)
        errors = np.zeros((L, P), np.float64)
        szs = np.zeros((L, P), np.int64)
        choice = np.zeros(L, np.int32)
        offsets = np.zeros(L + 1, np.int64)
        e_max, tsize, terr = C.c_double(), C.c_int64(), C.c_double()
        st = lib().lgreco_profile_solve_compress(
            self._h, _dptr(d_grads), _dptr(d_ef), C.addressof(layers), L, C.addressof(cands), P, _dptr(d_q),
            int(default_cand), int(n_bins), _np(errors), _np(szs), C.byref(e_max), _np(choice), C.byref(tsize),
            C.byref(terr), _dptr(d_payload), int(d_payload.numel() * d_payload.element_size()), _np(offsets),
            _stream(stream))
        self._check(st, allow=(EINFEASIBLE,))
        return st, errors, szs, e_max.value, choice, tsize.value, terr.value, offsets

    def solve(self, errors: np.ndarray, szs: np.ndarray, e_max: float, n_bins: int, stream=None):
        errors = np.ascontiguousarray(errors, np.float64)
        szs = np.ascontiguousarray(szs, np.int64)
        L, P = errors.shape
        choice = np.zeros(L, np.int32)
        tsize, terr = C.c_int64(), C.c_double()
        st = lib().lgreco_solve(self._h, _np(errors), _np(szs), L, P, float(e_max), int(n_bins),
                                _np(choice), C.byref(tsize), C.byref(terr), _stream(stream))
        self._check(st, allow=(EINFEASIBLE,))
        return st, choice, tsize.value, terr.value

    def solve_weighted(self, errors: np.ndarray, szs: np.ndarray, weights: np.ndarray, e_max: float,
                       n_bins: int, stream=None):
        errors = np.ascontiguousarray(errors, np.float64)
        szs = np.ascontiguousarray(szs, np.int64)
        weights = np.ascontiguousarray(weights, np.int64)
        L, P = errors.shape
        choice = np.zeros(L, np.int32)
        tsize, tcost, terr = C.c_int64(), C.c_int64(), C.c_double()
        st = lib().lgreco_solve_weighted(self._h, _np(errors), _np(szs), _np(weights), L, P, float(e_max),
                                         int(n_bins), _np(choice), C.byref(tsize), C.byref(tcost),
                                         C.byref(terr), _stream(stream))
        self._check(st, allow=(EINFEASIBLE,))
        return st, choice, tsize.value, tcost.value, terr.value

    def compress(self, d_grads, d_ef, layers, cands, choice: np.ndarray, d_payload, offsets: np.ndarray,
                 d_q=None, stream=None):
        choice = np.ascontiguousarray(choice, np.int32)
        offsets = np.ascontiguousarray(offsets, np.int64)
        st = lib().lgreco_compress(self._h, _dptr(d_grads), _dptr(d_ef), C.addressof(layers), len(layers),
                                   C.addressof(cands), len(cands), _np(choice), _dptr(d_q),
                                   _dptr(d_payload), _np(offsets), _stream(stream))
        self._check(st)

    def decompress(self, d_payload, offsets: np.ndarray, layers, cands, choice: np.ndarray, d_out,
                   accumulate: bool = False, stream=None):
        choice = np.ascontiguousarray(choice, np.int32)
        offsets = np.ascontiguousarray(offsets, np.int64)
        st = lib().lgreco_decompress(self._h, _dptr(d_payload), _np(offsets), C.addressof(layers), len(layers),
                                     C.addressof(cands), len(cands), _np(choice), _dptr(d_out),
                                     int(bool(accumulate)), _stream(stream))
        self._check(st)

    def accumulate(self, d_acc, d_grads, reset: bool = False, stream=None):
        if d_acc.numel() != d_grads.numel():
            raise ValueError("buffers differ in size")
        self._check(lib().lgreco_accumulate(self._h, _dptr(d_acc), _dptr(d_grads), int(d_grads.numel()),
                                            int(bool(reset)), _stream(stream)))

    def set_ef_zero_on_entry(self, on: bool):
        """Promise that the error-feedback buffer of profile_solve_compress holds zeros on entry (the
        profile then skips reading it); results are unchanged."""
        self._check(lib().lgreco_set_ef_zero_on_entry(self._h, int(bool(on))))

    def late_handovers(self) -> int:
        """Solves whose result block was still incomplete in host memory when its sequence number had
        arrived (caught by the block's check words)."""
        return int(lib().lgreco_late_handovers(self._h))

    def last_solve_groups(self) -> int:
        """0: sequential sweep; G: G layer groups; 1000 + G: groups with ties resolved; -G: sequential
        after the tie resolution gave up."""
        return int(lib().lgreco_last_solve_groups(self._h))

    def set_timing(self, level):
        """0 / False: off; 1 / True: main kernels; 2: every section."""
        self._check(lib().lgreco_set_timing(self._h, int(level)))

    def set_timing_stride(self, every: int):
        self._check(lib().lgreco_set_timing_stride(self._h, int(every)))

    def get_timing(self, call=None):
        """Sections of the last call, or of the last call of one kind (CALL_PROFILE, CALL_SOLVE,
        CALL_COMPRESS, CALL_RECEIVE); waits for the brackets it reads."""
        cap = 32
        names = (C.c_char_p * cap)()
        ms = (C.c_float * cap)()
        if call is None:
            n = lib().lgreco_get_timing(self._h, names, ms, cap)
        else:
            n = lib().lgreco_get_timing_of(self._h, int(call), names, ms, cap)
        if n < 0:
            self._check(n)
        return [(names[i].decode(), float(ms[i])) for i in range(min(n, cap))]

    def get_timing_totals(self, call):
        """(name, total milliseconds, calls) of every section of one kind of call since set_timing."""
        cap = 48
        names = (C.c_char_p * cap)()
        ms = (C.c_double * cap)()
        cnt = (C.c_int64 * cap)()
        n = lib().lgreco_get_timing_totals(self._h, int(call), names, ms, cnt, cap)
        if n < 0:
            self._check(n)
        return [(names[i].decode(), float(ms[i]), int(cnt[i])) for i in range(min(n, cap))]
