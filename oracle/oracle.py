"""ctypes front end of the CPU oracle (test infrastructure, see g10_oracle.cpp).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It knows nothing about the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

DIRECT, PREFIX = 0, 1
BY_BENEFIT, BY_RATIO = 0, 1        # ranking key
BAND, CLIPPED = 0, 1               # what counts as the benefit
FITS, RESIDUAL, TRUNCATED = 0, 1, 2

RECORD = np.dtype([("cand", "<u4"), ("tensor", "<u4"), ("evict_after", "<u4"),
                   ("absent_first", "<u4"), ("absent_last", "<u4"), ("next_use", "<u4"),
                   ("dest", "<u4"), ("wraps", "<u4"), ("size", "<u8"), ("t_out", "<u8"),
                   ("t_in", "<u8"), ("benefit_lo", "<u8"), ("benefit_hi", "<u8")])
assert RECORD.itemsize == 72


class _Trace(C.Structure):
    _fields_ = [("K", C.c_uint32), ("N", C.c_uint32), ("P", C.c_uint64),
                ("dur_ns", C.c_void_p), ("size_bytes", C.c_void_p), ("is_global", C.c_void_p),
                ("use_kernel", C.c_void_p), ("use_tensor", C.c_void_p), ("no_wrap", C.c_uint32)]


class _Params(C.Structure):
    _fields_ = [("gpu_cap", C.c_uint64), ("host_cap", C.c_uint64),
                ("bw_out", C.c_uint64 * 2), ("bw_in", C.c_uint64 * 2),
                ("rank", C.c_uint32), ("area", C.c_uint32)]


class _Summary(C.Structure):
    _fields_ = [("status", C.c_int32), ("n_migrations", C.c_uint64), ("n_iterations", C.c_uint64),
                ("n_null", C.c_uint64), ("n_cand_evals", C.c_uint64), ("peak_before", C.c_uint64),
                ("peak_after", C.c_uint64), ("overtime_before", C.c_uint64),
                ("overtime_after", C.c_uint64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.g10o_vitality.argtypes = [C.POINTER(_Trace), C.c_int, C.POINTER(C.c_void_p)]
        _lib.g10o_counts.argtypes = [C.c_void_p, C.POINTER(C.c_uint64)]
        _lib.g10o_counts.restype = None
        _lib.g10o_copy.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        _lib.g10o_plan.argtypes = [C.c_void_p, C.POINTER(_Params), C.c_int, C.c_uint64,
                                   C.POINTER(_Summary)]
        _lib.g10o_windows.argtypes = [C.c_void_p, C.POINTER(_Params), C.c_int, C.c_int] + [C.c_void_p] * 5
        _lib.g10o_prefetch.argtypes = [C.c_void_p, C.c_int]
        _lib.g10o_replay.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        _lib.g10o_free.argtypes = [C.c_void_p]
        _lib.g10o_free.restype = None
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


class OracleError(Exception):
    def __init__(self, code):
        super().__init__(f"oracle error {code}")
        self.code = code


class Vitality:
    """Result of the vitality analysis; also the handle planning runs on."""

    def __init__(self, trace, mode: int = DIRECT, no_wrap: bool = False):
        self._h = C.c_void_p()
        self.mode = mode
        a = [np.ascontiguousarray(trace.dur_ns, np.uint64),
             np.ascontiguousarray(trace.size_bytes, np.uint64),
             np.ascontiguousarray(trace.is_global, np.uint8),
             np.ascontiguousarray(trace.use_kernel, np.uint32),
             np.ascontiguousarray(trace.use_tensor, np.uint32)]
        K, N, P = a[0].shape[0], a[1].shape[0], a[3].shape[0]
        t = _Trace(K, N, P, _ptr(a[0]), _ptr(a[1]), _ptr(a[2]), _ptr(a[3]), _ptr(a[4]), int(no_wrap))
        rc = lib().g10o_vitality(C.byref(t), mode, C.byref(self._h))
        if rc:
            self._h = None
            raise OracleError(rc)
        self.K, self.N = K, N
        cnt = self._counts()
        self.n_uses, self.C, self.peak, self.T = cnt[0], cnt[1], cnt[2], cnt[3]
        self.use_off = self._get(0, N + 1, np.uint64)
        self.use_k = self._get(1, self.n_uses, np.uint32)
        self.birth = self._get(2, N, np.uint32)
        self.death = self._get(3, N, np.uint32)
        self.per_tensor = self._get(4, self.C, np.uint32)
        self.per_L = self._get(5, self.C, np.uint32)
        self.per_R = self._get(6, self.C, np.uint32)
        self.start = self._get(7, K + 1, np.uint64)
        self.pressure = self._get(8, K, np.uint64)

    def _counts(self):
        out = (C.c_uint64 * 8)()
        lib().g10o_counts(self._h, out)
        return [int(x) for x in out]

    def _get(self, which, n, dtype):
        a = np.zeros(n, dtype)
        if n:
            lib().g10o_copy(self._h, which, _ptr(a))
        return a

    @staticmethod
    def _params(gpu_cap, host_cap, bw_out, bw_in, rank=0, area=0):
        p = _Params()
        p.rank, p.area = int(rank), int(area)
        p.gpu_cap, p.host_cap = int(gpu_cap), int(host_cap)
        p.bw_out[0], p.bw_out[1] = int(bw_out[0]), int(bw_out[1])
        p.bw_in[0], p.bw_in[1] = int(bw_in[0]), int(bw_in[1])
        return p

    def windows(self, dest, gpu_cap, host_cap, bw_out, bw_in, mode=None):
        """Per period: (valid, a, b, tau_o, tau_i) for one destination."""
        p = self._params(gpu_cap, host_cap, bw_out, bw_in)
        n = self.C
        valid = np.zeros(n, np.uint8)
        a, b = np.zeros(n, np.uint32), np.zeros(n, np.uint32)
        to, ti = np.zeros(n, np.uint64), np.zeros(n, np.uint64)
        rc = lib().g10o_windows(self._h, C.byref(p), self.mode if mode is None else mode, dest,
                                _ptr(valid), _ptr(a), _ptr(b), _ptr(to), _ptr(ti))
        if rc:
            raise OracleError(rc)
        return valid, a, b, to, ti

    def plan(self, gpu_cap, host_cap, bw_out, bw_in, mode=None, max_iters=2 ** 64 - 1, rank=0, area=0):
        p = self._params(gpu_cap, host_cap, bw_out, bw_in, rank, area)
        s = _Summary()
        rc = lib().g10o_plan(self._h, C.byref(p), self.mode if mode is None else mode,
                             int(max_iters), C.byref(s))
        if rc:
            raise OracleError(rc)
        cnt = self._counts()
        return Plan(self, s, cnt[4], cnt[5])

    def close(self):
        if self._h:
            lib().g10o_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Prefetch:
    """Smart prefetching (Section 4.4) applied to a plan: per record the kernel
    slots by which its prefetch moved back, the last absent slot that is left
    (mod K; one before the first absent slot if none is left), the visiting
    order and the pressure curve with the earlier prefetches."""

    def __init__(self, plan: "Plan", mode: int):
        v = plan._v
        rc = lib().g10o_prefetch(v._h, mode)
        if rc:
            raise OracleError(rc)
        n = len(plan.records)
        self.order = v._get(20, n, np.uint32)
        self.gained = v._get(21, n, np.uint32)
        self.pressure = v._get(22, v.K, np.uint64)
        self.absent_last = ((plan.b2.astype(np.int64) - self.gained) % v.K).astype(np.uint32)
        self.n_moved = int((self.gained > 0).sum())
        self.slots_gained = int(self.gained.astype(np.uint64).sum())
        self.peak = int(self.pressure.max()) if v.K else 0


class Replay:
    """Slot-level replay of a plan (see g10_oracle.cpp): steady-state iteration time, stall time,
    stalled kernels, traffic and channel time per destination, lateness per migration."""

    def __init__(self, plan: "Plan", dur=None, eager=False):
        v = plan._v
        out = np.zeros(10, np.uint64)
        self.late = np.zeros(len(plan.records), np.uint64)
        d = None if dur is None else np.ascontiguousarray(dur, np.uint64)
        assert d is None or d.shape[0] == v.K
        rc = lib().g10o_replay(v._h, None if d is None else _ptr(d), int(eager), _ptr(out),
                               _ptr(self.late) if len(self.late) else None)
        if rc:
            raise OracleError(rc)
        o = [int(x) for x in out]
        self.iter_ns, self.planned_ns, self.stall_ns, self.n_stalled = o[0], o[1], o[2], o[3]
        self.bytes, self.busy_out_ns, self.busy_in_ns = o[4:6], o[6:8], o[8:10]


class Plan:
    def replay(self, dur=None, eager=False) -> "Replay":
        """Must be called before the handle plans again (eager: after prefetch())."""
        return Replay(self, dur, eager)

    def prefetch(self, mode=None) -> "Prefetch":
        """Must be called before the handle plans again."""
        return Prefetch(self, self._v.mode if mode is None else mode)

    def __init__(self, v: Vitality, s: _Summary, n_rec: int, n_null: int):
        self._v = v
        self.a2 = v._get(23, n_rec, np.uint32)      # absent window in doubled coordinates
        self.b2 = v._get(24, n_rec, np.uint32)
        for f, _ in _Summary._fields_:
            setattr(self, f, int(getattr(s, f)))
        self.records = v._get(9, n_rec, RECORD)
        self.pressure_after = v._get(10, v.K, np.uint64)
        self.null_cands = v._get(11, n_null, np.uint32)
        self.null_iters = v._get(13, n_null, np.uint64)
        self.host_after = v._get(12, v.K, np.uint64)
        self.busy_after = [[v._get(16 + 2 * d + r, v.K, np.uint64) for r in range(2)] for d in range(2)]
