"""Thin ctypes binding over the C ABI of include/g10.h (argument marshalling only).

Every step of the analysis and of the planning loop runs in the HIP library
`libg10.so`; this module allocates nothing but the small argument structs and
uses torch only for device buffers and the current stream.  If the library has
not been built the import of the library fails loudly: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libg10.so")

OK, EINVAL, EOVERFLOW, ENOMEM, EDEVICE, ELIMIT = 0, -1, -2, -3, -4, -5
FLASH, HOST = 0, 1
FITS, RESIDUAL, TRUNCATED = 0, 1, 2
NO_WRAP = 1

EXPORTS = ["g10_vitality", "g10_vitality_info", "g10_vitality_read", "g10_vitality_static", "g10_plan", "g10_plan_batch",
           "g10_plan_counters", "g10_plan_limits", "g10_prefetch", "g10_replay", "g10_plan_free", "g10_trim"]
STATIC_MAX_K, STATIC_MAX_N, STATIC_MAX_P = 131072, 262144, 262144

MIGRATION = np.dtype([("cand", "<u4"), ("tensor", "<u4"), ("evict_after", "<u4"),
                      ("absent_first", "<u4"), ("absent_last", "<u4"), ("next_use", "<u4"),
                      ("dest", "<u4"), ("wraps", "<u4"), ("size", "<u8"), ("t_out", "<u8"),
                      ("t_in", "<u8"), ("benefit_lo", "<u8"), ("benefit_hi", "<u8")])
DROPPED = np.dtype([("iteration", "<u8"), ("cand", "<u4"), ("reserved", "<u4")])
assert MIGRATION.itemsize == 72 and DROPPED.itemsize == 16


class G10Error(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what} failed with code {code}")
        self.code = code


class _Trace(C.Structure):
    _fields_ = [("K", C.c_uint32), ("N", C.c_uint32), ("P", C.c_uint64),
                ("dur_ns", C.c_void_p), ("size_bytes", C.c_void_p), ("is_global", C.c_void_p),
                ("use_kernel", C.c_void_p), ("use_tensor", C.c_void_p), ("flags", C.c_uint32)]


class _Stats(C.Structure):
    _fields_ = [("n_uses", C.c_uint64), ("n_periods", C.c_uint64), ("peak_bytes", C.c_uint64),
                ("iter_ns", C.c_uint64)]


class _VitalityBuffers(C.Structure):
    _fields_ = [("use_off", C.c_void_p), ("use_k", C.c_void_p), ("per_tensor", C.c_void_p), ("per_L", C.c_void_p),
                ("per_R", C.c_void_p), ("start", C.c_void_p), ("pressure", C.c_void_p)]


class _Params(C.Structure):
    _fields_ = [("gpu_cap_bytes", C.c_uint64), ("host_cap_bytes", C.c_uint64),
                ("bw_out_Bpus", C.c_uint64 * 2), ("bw_in_Bpus", C.c_uint64 * 2),
                ("max_iterations", C.c_uint64),
                ("dur_ns", C.c_void_p), ("rank", C.c_uint32), ("area", C.c_uint32)]


class _Result(C.Structure):
    _fields_ = [("status", C.c_int32),
                ("n_migrations", C.c_uint64), ("n_iterations", C.c_uint64), ("n_dropped", C.c_uint64),
                ("n_cand_evals", C.c_uint64), ("peak_before", C.c_uint64), ("peak_after", C.c_uint64),
                ("overtime_before_ns", C.c_uint64), ("overtime_after_ns", C.c_uint64),
                ("migrations", C.c_void_p), ("dropped", C.c_void_p), ("pressure_after", C.c_void_p),
                ("plan_ms", C.c_double)]


class _Counters(C.Structure):
    _fields_ = [("score_full_ms", C.c_double), ("score_full_cands", C.c_uint64),
                ("loop_ms", C.c_double), ("loop_launches", C.c_uint64), ("loop_passes", C.c_uint64), ("loop_more_rounds", C.c_uint64),
                ("loop_retiles", C.c_uint64), ("retile_cands", C.c_uint64), ("loop_cands_scored", C.c_uint64),
                ("loop_second_rounds", C.c_uint64), ("loop_chunk_jobs", C.c_uint64),
                ("loop_area_evals", C.c_uint64), ("loop_area_refused", C.c_uint64), ("loop_wide_rounds", C.c_uint64),
                ("batch_prepare_ms", C.c_double), ("batch_loops_ms", C.c_double), ("batch_retile_ms", C.c_double),
                ("batch_results_ms", C.c_double)]


class _PrefetchResult(C.Structure):
    _fields_ = [("n_migrations", C.c_uint64), ("n_moved", C.c_uint64), ("slots_gained", C.c_uint64),
                ("peak_bytes", C.c_uint64), ("order", C.c_void_p), ("gained", C.c_void_p),
                ("absent_last", C.c_void_p), ("pressure", C.c_void_p), ("ms", C.c_double)]


class _ReplayResult(C.Structure):
    _fields_ = [("iter_ns", C.c_uint64), ("planned_ns", C.c_uint64), ("stall_ns", C.c_uint64), ("n_stalled", C.c_uint64),
                ("bytes", C.c_uint64 * 2), ("busy_out_ns", C.c_uint64 * 2), ("busy_in_ns", C.c_uint64 * 2),
                ("n_migrations", C.c_uint64), ("late_ns", C.c_void_p), ("ms", C.c_double)]


_lib = None


def load():
    """Loads libg10.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2310_09443_amd.build` "
                              "(hipcc, gfx950); there is no CPU fallback")
        # torch brings its own HIP runtime; it must be the one in the process before this library
        # resolves its HIP symbols, or the two would not share streams and device memory
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        lib.g10_vitality.argtypes = [C.POINTER(_Trace), C.c_void_p, C.POINTER(C.c_void_p)]
        lib.g10_vitality_info.argtypes = [C.c_void_p, C.POINTER(_Stats)]
        lib.g10_vitality_read.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_uint64]
        lib.g10_vitality_static.argtypes = [C.POINTER(_Trace), C.c_void_p, C.POINTER(_VitalityBuffers), C.POINTER(_Stats)]
        lib.g10_plan.argtypes = [C.c_void_p, C.POINTER(_Params), C.POINTER(_Result)]
        lib.g10_plan_batch.argtypes = [C.c_void_p, C.POINTER(_Params), C.c_uint32, C.POINTER(_Result)]
        lib.g10_plan_counters.argtypes = [C.c_void_p, C.c_uint32, C.POINTER(_Counters)]
        lib.g10_plan_limits.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32]
        lib.g10_prefetch.argtypes = [C.c_void_p, C.POINTER(_PrefetchResult)]
        lib.g10_replay.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.POINTER(_ReplayResult)]
        lib.g10_plan_free.argtypes = [C.c_void_p]
        lib.g10_plan_free.restype = None
        lib.g10_trim.argtypes = []
        lib.g10_trim.restype = None
        _lib = lib
    return _lib


class DeviceTrace:
    """A trace resident in HBM (torch tensors own the memory)."""

    def __init__(self, trace, device="cuda:0"):
        import torch
        self.K, self.N, self.P = trace.K, trace.N, trace.P
        dev = torch.device(device)
        # torch has no uint64 arithmetic, but these are only buffers: ship the bits as int64 / int32
        self.dur = torch.from_numpy(trace.dur_ns.view(np.int64)).to(dev)
        self.size = torch.from_numpy(trace.size_bytes.view(np.int64)).to(dev)
        self.glob = torch.from_numpy(np.ascontiguousarray(trace.is_global, np.uint8)).to(dev)
        self.uk = torch.from_numpy(trace.use_kernel.view(np.int32)).to(dev)
        self.ut = torch.from_numpy(trace.use_tensor.view(np.int32)).to(dev)
        self.device = dev


class Result:
    def __init__(self, r: _Result, K: int, pool=None, counters: _Counters = None):
        """pool: a _Pool that takes this result's arrays (the results of a batch share one allocation).
        counters: what g10_plan_counters says of this plan; kept as attributes of the same names."""
        for f, _ in _Result._fields_:
            if f not in ("migrations", "dropped", "pressure_after"):
                setattr(self, f, getattr(r, f))
        if counters is not None:
            for f, _ in _Counters._fields_:
                setattr(self, f, getattr(counters, f))
        take = pool.take if pool is not None else self._copy
        self.records = take(r.migrations, int(r.n_migrations), MIGRATION)
        self.dropped = take(r.dropped, int(r.n_dropped), DROPPED)
        self.pressure_after = take(r.pressure_after, K, np.dtype("<u8"))
        if pool is None:
            self._dropped_views()

    def _dropped_views(self):
        self.null_iters = self.dropped["iteration"].copy()
        self.null_cands = self.dropped["cand"].copy()

    @staticmethod
    def nbytes(r: _Result, K: int) -> int:
        return int(r.n_migrations) * MIGRATION.itemsize + int(r.n_dropped) * DROPPED.itemsize + K * 8

    @staticmethod
    def _copy(ptr, n, dtype):
        if not n or not ptr:
            return np.zeros(0, dtype)
        buf = (C.c_char * (n * dtype.itemsize)).from_address(ptr)
        return np.frombuffer(buf, dtype=dtype, count=n).copy()


class _Pool:
    """One allocation for the host copies of many results: a few large pages instead of many small ones.
    The copies themselves are collected and run together by flush(), over a few threads where there is
    much to copy (ctypes releases the interpreter lock around memmove)."""

    def __init__(self, nbytes: int):
        self.buf = np.empty(max(nbytes, 1), np.uint8)
        self.at = 0
        self.todo = []

    def take(self, ptr, n, dtype):
        if not n or not ptr:
            return np.zeros(0, dtype)
        size = n * dtype.itemsize
        out = self.buf[self.at:self.at + size]
        self.at += size
        self.todo.append((out.ctypes.data, ptr, size))
        return out.view(dtype)

    def flush(self):
        todo, self.todo = self.todo, []
        if sum(t[2] for t in todo) < (32 << 20):
            for dst, src, size in todo:
                C.memmove(dst, src, size)
            return
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(lambda t: C.memmove(*t), todo))


class PrefetchResult:
    def __init__(self, r: _PrefetchResult, K: int):
        n = int(r.n_migrations)
        self.n_migrations, self.n_moved, self.slots_gained = n, int(r.n_moved), int(r.slots_gained)
        self.peak, self.ms = int(r.peak_bytes), float(r.ms)
        self.order = Result._copy(r.order, n, np.dtype("<u4"))
        self.gained = Result._copy(r.gained, n, np.dtype("<u4"))
        self.absent_last = Result._copy(r.absent_last, n, np.dtype("<u4"))
        self.pressure = Result._copy(r.pressure, K, np.dtype("<u8"))


class ReplayResult:
    def __init__(self, r: _ReplayResult):
        self.iter_ns, self.planned_ns, self.stall_ns = int(r.iter_ns), int(r.planned_ns), int(r.stall_ns)
        self.n_stalled, self.ms = int(r.n_stalled), float(r.ms)
        self.bytes, self.busy_out_ns, self.busy_in_ns = list(r.bytes), list(r.busy_out_ns), list(r.busy_in_ns)
        self.late = Result._copy(r.late_ns, int(r.n_migrations), np.dtype("<u8"))


class Handle:
    """g10_vitality on construction; g10_plan via .plan(); g10_prefetch via .prefetch();
    g10_plan_free on close."""

    def __init__(self, dtrace: DeviceTrace, no_wrap: bool = False, stream=None):
        import torch
        lib = load()
        self._h = C.c_void_p()
        self.K, self.N = dtrace.K, dtrace.N
        if stream is None:
            stream = torch.cuda.current_stream(dtrace.device).cuda_stream
        t = _Trace(dtrace.K, dtrace.N, dtrace.P, dtrace.dur.data_ptr(), dtrace.size.data_ptr(),
                   dtrace.glob.data_ptr(), dtrace.uk.data_ptr() if dtrace.P else None,
                   dtrace.ut.data_ptr() if dtrace.P else None, NO_WRAP if no_wrap else 0)
        with torch.cuda.device(dtrace.device):
            rc = lib.g10_vitality(C.byref(t), C.c_void_p(stream), C.byref(self._h))
        if rc:
            self._h = None
            raise G10Error(rc, "g10_vitality")
        s = _Stats()
        lib.g10_vitality_info(self._h, C.byref(s))
        self.n_uses, self.C, self.peak, self.T = int(s.n_uses), int(s.n_periods), int(s.peak_bytes), int(s.iter_ns)
        self._dev = dtrace.device

    def read(self, which: int):
        n, dt = {0: (self.N + 1, np.uint64), 1: (self.n_uses, np.uint32), 2: (self.C, np.uint32),
                 3: (self.C, np.uint32), 4: (self.C, np.uint32), 5: (self.K + 1, np.uint64),
                 6: (self.K, np.uint64)}[which]
        a = np.zeros(n, dt)
        rc = load().g10_vitality_read(self._h, which, a.ctypes.data, a.nbytes)
        if rc:
            raise G10Error(rc, "g10_vitality_read")
        return a

    use_off = property(lambda self: self.read(0))
    use_k = property(lambda self: self.read(1))
    per_tensor = property(lambda self: self.read(2))
    per_L = property(lambda self: self.read(3))
    per_R = property(lambda self: self.read(4))
    start = property(lambda self: self.read(5))
    pressure = property(lambda self: self.read(6))

    def limits(self, max_tiles=0, max_chunks=0):
        """g10_plan_limits: bounds of the loop's on-chip structures for the planning calls that follow (0 = default)."""
        rc = load().g10_plan_limits(self._h, int(max_tiles), int(max_chunks))
        if rc:
            raise G10Error(rc, "g10_plan_limits")

    def _counters(self, i):
        c = _Counters()
        rc = load().g10_plan_counters(self._h, i, C.byref(c))
        if rc:
            raise G10Error(rc, "g10_plan_counters")
        return c

    def _fill(self, p, gpu_cap, host_cap, bw_out, bw_in, max_iters=0, dur=None, rank=0, area=0):
        """dur: None, or a device tensor of K 64-bit durations (ns) that replace the trace's for this plan."""
        p.gpu_cap_bytes, p.host_cap_bytes = int(gpu_cap), int(host_cap)
        p.bw_out_Bpus[0], p.bw_out_Bpus[1] = int(bw_out[0]), int(bw_out[1])
        p.bw_in_Bpus[0], p.bw_in_Bpus[1] = int(bw_in[0]), int(bw_in[1])
        p.max_iterations = int(max_iters)
        p.rank, p.area = int(rank), int(area)
        if dur is None:
            p.dur_ns = None
        else:
            if not (dur.is_cuda and dur.is_contiguous() and dur.element_size() == 8 and dur.numel() == self.K):
                raise ValueError("dur must be a contiguous device tensor of K 64-bit integers")
            p.dur_ns = dur.data_ptr()

    def plan_batch(self, param_dicts, max_tiles=0, max_chunks=0):
        """g10_plan_batch: one plan per dict of plan() keyword arguments (max_tiles / max_chunks, which
        belong to the handle, may also come in the first dict)."""
        import torch
        n = len(param_dicts)
        ps = (_Params * n)()
        param_dicts = [dict(d) for d in param_dicts]
        for d in param_dicts:
            max_tiles = d.pop("max_tiles", max_tiles) or max_tiles
            max_chunks = d.pop("max_chunks", max_chunks) or max_chunks
        self.limits(max_tiles, max_chunks)
        for p, d in zip(ps, param_dicts):
            self._fill(p, **d)
        rs = (_Result * n)()
        with torch.cuda.device(self._dev):
            rc = load().g10_plan_batch(self._h, ps, n, rs)
        if rc:
            raise G10Error(rc, "g10_plan_batch")
        pool = _Pool(sum(Result.nbytes(r, self.K) for r in rs))
        out = [Result(r, self.K, pool, self._counters(i)) for i, r in enumerate(rs)]
        pool.flush()
        for x in out:
            x._dropped_views()
        return out

    def plan(self, gpu_cap, host_cap, bw_out, bw_in, max_iters=0, max_tiles=0, max_chunks=0, dur=None, rank=0, area=0) -> Result:
        import torch
        p = _Params()
        self._fill(p, gpu_cap, host_cap, bw_out, bw_in, max_iters, dur, rank, area)
        self.limits(max_tiles, max_chunks)
        r = _Result()
        with torch.cuda.device(self._dev):
            rc = load().g10_plan(self._h, C.byref(p), C.byref(r))
        if rc:
            raise G10Error(rc, "g10_plan")
        return Result(r, self.K, None, self._counters(0))

    def prefetch(self) -> PrefetchResult:
        import torch
        r = _PrefetchResult()
        with torch.cuda.device(self._dev):
            rc = load().g10_prefetch(self._h, C.byref(r))
        if rc:
            raise G10Error(rc, "g10_prefetch")
        return PrefetchResult(r, self.K)

    def replay(self, dur=None, eager=False) -> ReplayResult:
        """dur: None, or a device tensor of K 64-bit durations (ns) to replay the plan with."""
        import torch
        if dur is not None and not (dur.is_cuda and dur.is_contiguous() and dur.element_size() == 8 and dur.numel() == self.K):
            raise ValueError("dur must be a contiguous device tensor of K 64-bit integers")
        r = _ReplayResult()
        with torch.cuda.device(self._dev):
            rc = load().g10_replay(self._h, None if dur is None else dur.data_ptr(), int(bool(eager)), C.byref(r))
        if rc:
            raise G10Error(rc, "g10_replay")
        return ReplayResult(r)

    def close(self):
        if self._h:
            load().g10_plan_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def g10_vitality(dtrace: DeviceTrace, no_wrap: bool = False, stream=None) -> Handle:
    return Handle(dtrace, no_wrap, stream)


class StaticVitality:
    """Results of g10_vitality_static: the caller's device buffers (torch tensors made here, before
    the call) and the counts.  The arrays come back as numpy copies through the properties."""

    def __init__(self, dtrace: DeviceTrace, no_wrap: bool = False, stream=None, buffers=None):
        import torch
        lib = load()
        dev = dtrace.device
        K, N, P = dtrace.K, dtrace.N, dtrace.P
        if buffers is None:                         # (a caller may bring tensors it already holds)
            buffers = dict(use_off=torch.empty(N + 1, dtype=torch.int64, device=dev),
                           use_k=torch.empty(max(P, 1), dtype=torch.int32, device=dev),
                           per_tensor=torch.empty(max(P, 1), dtype=torch.int32, device=dev),
                           per_L=torch.empty(max(P, 1), dtype=torch.int32, device=dev),
                           per_R=torch.empty(max(P, 1), dtype=torch.int32, device=dev),
                           start=torch.empty(K + 1, dtype=torch.int64, device=dev),
                           pressure=torch.empty(K, dtype=torch.int64, device=dev))
        self.buffers = buffers
        b = _VitalityBuffers(*(buffers[f].data_ptr() for f, _ in _VitalityBuffers._fields_))
        if stream is None:
            stream = torch.cuda.current_stream(dev).cuda_stream
        t = _Trace(K, N, P, dtrace.dur.data_ptr(), dtrace.size.data_ptr(), dtrace.glob.data_ptr(),
                   dtrace.uk.data_ptr() if P else None, dtrace.ut.data_ptr() if P else None, NO_WRAP if no_wrap else 0)
        s = _Stats()
        with torch.cuda.device(dev):
            rc = lib.g10_vitality_static(C.byref(t), C.c_void_p(stream), C.byref(b), C.byref(s))
        if rc:
            raise G10Error(rc, "g10_vitality_static")
        self.K, self.N = K, N
        self.n_uses, self.C, self.peak, self.T = int(s.n_uses), int(s.n_periods), int(s.peak_bytes), int(s.iter_ns)

    def _get(self, name, n, dtype):
        return self.buffers[name][:n].cpu().numpy().view(dtype).copy()

    use_off = property(lambda self: self._get("use_off", self.N + 1, np.uint64))
    use_k = property(lambda self: self._get("use_k", self.n_uses, np.uint32))
    per_tensor = property(lambda self: self._get("per_tensor", self.C, np.uint32))
    per_L = property(lambda self: self._get("per_L", self.C, np.uint32))
    per_R = property(lambda self: self._get("per_R", self.C, np.uint32))
    start = property(lambda self: self._get("start", self.K + 1, np.uint64))
    pressure = property(lambda self: self._get("pressure", self.K, np.uint64))


def g10_vitality_static(dtrace: DeviceTrace, no_wrap: bool = False, stream=None, buffers=None) -> StaticVitality:
    return StaticVitality(dtrace, no_wrap, stream, buffers)


def g10_plan(handle: Handle, gpu_cap, host_cap, bw_out, bw_in, max_iters=0, max_tiles=0, max_chunks=0, dur=None, rank=0, area=0) -> Result:
    return handle.plan(gpu_cap, host_cap, bw_out, bw_in, max_iters, max_tiles, max_chunks, dur, rank, area)


def g10_plan_batch(handle: Handle, param_dicts):
    return handle.plan_batch(param_dicts)


def g10_prefetch(handle: Handle) -> PrefetchResult:
    return handle.prefetch()


def g10_replay(handle: Handle, dur=None, eager=False) -> ReplayResult:
    return handle.replay(dur, eager)


def g10_plan_free(handle: Handle) -> None:
    handle.close()


def g10_trim() -> None:
    load().g10_trim()
