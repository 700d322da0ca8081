"""g10_vitality_static, the analysis for callers that cannot allocate, against g10_vitality:
every array and count equal, on two calls in a row (the second on a smaller trace, so that what
the first call left in the library's fixed device array must not show), and the size limit."""
import numpy as np
import pytest

from paper_2310_09443_amd import binding, traces

pytestmark = pytest.mark.gpu

FIELDS = ("use_off", "use_k", "per_tensor", "per_L", "per_R", "start", "pressure")


def check_equal(dt, no_wrap=False):
    h = binding.g10_vitality(dt, no_wrap=no_wrap)
    try:
        s = binding.g10_vitality_static(dt, no_wrap=no_wrap)
        assert (s.n_uses, s.C, s.peak, s.T) == (h.n_uses, h.C, h.peak, h.T)
        for f in FIELDS:
            a, b = getattr(s, f), getattr(h, f)
            assert a.shape == b.shape and (a == b).all(), f
        return s
    finally:
        h.close()


def test_two_calls_in_a_row_the_second_smaller():
    big = binding.DeviceTrace(traces.config(4).trace, "cuda:0")       # tens of thousands of pairs: several sort tiles
    small = binding.DeviceTrace(traces.config(2).trace, "cuda:0")
    tiny = binding.DeviceTrace(traces.config(1).trace, "cuda:0")
    a = check_equal(big)
    b = check_equal(small)
    c = check_equal(tiny, no_wrap=True)
    d = check_equal(big)                                                # and a larger one again
    assert a.C > b.C > c.C and d.C == a.C
    assert (a.pressure == d.pressure).all()


def test_own_buffers_and_a_ragged_random_trace():
    import torch
    tr = traces.stress(K=2500, N=30000, seed=77).trace                 # duplicates, global tensors, a ragged last sort tile
    dt = binding.DeviceTrace(tr, "cuda:0")
    dev = dt.device
    bufs = dict(use_off=torch.full((dt.N + 1,), -1, dtype=torch.int64, device=dev),
                use_k=torch.full((max(dt.P, 1),), -1, dtype=torch.int32, device=dev),
                per_tensor=torch.full((max(dt.P, 1),), -1, dtype=torch.int32, device=dev),
                per_L=torch.full((max(dt.P, 1),), -1, dtype=torch.int32, device=dev),
                per_R=torch.full((max(dt.P, 1),), -1, dtype=torch.int32, device=dev),
                start=torch.full((dt.K + 1,), -1, dtype=torch.int64, device=dev),
                pressure=torch.full((dt.K,), -1, dtype=torch.int64, device=dev))
    s = binding.g10_vitality_static(dt, buffers=bufs)
    h = binding.g10_vitality(dt)
    try:
        for f in FIELDS:
            assert (getattr(s, f) == getattr(h, f)).all(), f
        # nothing is written past the counted entries
        assert (bufs["use_k"][s.n_uses:] == -1).all() and (bufs["per_L"][s.C:] == -1).all()
    finally:
        h.close()


def test_a_trace_beyond_the_limit_is_refused_before_any_work():
    w = traces.config(5)                                               # 2.7 M pairs
    dt = binding.DeviceTrace(w.trace, "cuda:0")
    assert dt.P > binding.STATIC_MAX_P
    with pytest.raises(binding.G10Error) as e:
        binding.g10_vitality_static(dt)
    assert e.value.code == binding.ELIMIT
    # missing output buffers are refused as well
    import ctypes as C
    small = binding.DeviceTrace(traces.config(1).trace, "cuda:0")
    t = binding._Trace(small.K, small.N, small.P, small.dur.data_ptr(), small.size.data_ptr(), small.glob.data_ptr(),
                       small.uk.data_ptr(), small.ut.data_ptr(), 0)
    st = binding._Stats()
    assert binding.load().g10_vitality_static(C.byref(t), None, C.byref(binding._VitalityBuffers()), C.byref(st)) == binding.EINVAL
    assert binding.load().g10_vitality_static(C.byref(t), None, None, C.byref(st)) == binding.EINVAL
