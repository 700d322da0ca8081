"""Pins for the oracle's smart prefetching (Section 4.4): a hand-worked example
with two periods competing for one slot, closed forms, the two evaluation
modes against each other and against an independent replay, invariants."""
import numpy as np
import pytest

import prefetchcheck
from goldenio import Golden
from oracle import oracle as O
from paper_2310_09443_amd import traces
from paper_2310_09443_amd.traces import Trace


@pytest.mark.parametrize("mode", [O.DIRECT, O.PREFIX])
def test_hand_worked_prefetch(mode):
    g = Golden("hand_prefetch.txt")
    v = O.Vitality(g.trace, mode)
    p = v.plan(**g.plan_args())
    e = g.expect
    fields = ["cand", "tensor", "evict_after", "absent_first", "absent_last", "next_use", "dest",
              "wraps", "size", "t_out", "t_in"]
    got = [[int(r[f]) for f in fields] + [int(r["benefit_lo"]) + (int(r["benefit_hi"]) << 64)] for r in p.records]
    assert got == e["record"] and p.status == e["status"][0][0] and p.n_iterations == e["iterations"][0][0]
    assert p.pressure_after.tolist() == e["pressure_after"][0]
    f = p.prefetch()
    assert f.order.tolist() == e["prefetch_order"][0]
    assert f.gained.tolist() == e["gained"][0]
    assert f.absent_last.tolist() == e["absent_last_eager"][0]
    assert f.pressure.tolist() == e["pressure_eager"][0]
    assert (f.n_moved, f.slots_gained) == (1, 1)


def test_order_decides_who_gets_the_room():
    """The same two periods visited in the other order (Y's prefetch made the
    earlier one by a faster host link for X... here simply by swapping the
    prefetch times through the bandwidths) give the slot to the other tensor."""
    g = Golden("hand_prefetch.txt")
    v = O.Vitality(g.trace, O.DIRECT)
    args = g.plan_args()
    p = v.plan(**args)
    a2, b2 = prefetchcheck.doubled_windows(g.K, p.records)
    assert a2.tolist() == p.a2.tolist() and b2.tolist() == p.b2.tolist()
    # replay with the plan order reversed by hand: Y first takes slot 6, X then cannot
    rec = p.records.copy()
    rec["t_in"][0], rec["t_in"][1] = 1, 79999          # X's latest safe time 89999, Y's 1 -> Y first
    order, gained, pr = prefetchcheck.replay(g.K, v.start, args["gpu_cap"], rec, a2, b2, p.pressure_after)
    assert order.tolist() == [1, 0] and gained.tolist() == [0, 1]
    assert pr.tolist() == [20000, 32000, 32000, 0, 30000, 30000, 12000, 32000, 32000, 20000]


def _uniform(K, sizes, uses, glob=None, dur=1000):
    uk = np.array([u[0] for u in uses], np.uint32)
    ut = np.array([u[1] for u in uses], np.uint32)
    return Trace("uniform", np.full(K, dur, np.uint64), np.array(sizes, np.uint64),
                 np.array(glob if glob is not None else [0] * len(sizes), np.uint8), uk, ut)


@pytest.mark.parametrize("mode", [O.DIRECT, O.PREFIX])
def test_closed_forms(mode):
    # one evicted tensor A (100 B, used by kernels 0 and 19) under a bump B (100 B, kernels 9,10):
    # pressure 100 everywhere, 200 in slots 9,10.  Bandwidth 1 B/ns... 100 B at 100 B/us = 1000 ns = 1 slot.
    tr = _uniform(20, [100, 100], [(0, 0), (19, 0), (9, 1), (10, 1)])
    v = O.Vitality(tr, mode)
    # capacity 150: slots 9,10 over.  A to flash: eviction slot 1, prefetch slot 18, absent [2,17].
    p = v.plan(gpu_cap=150, host_cap=0, bw_out=(100, 100), bw_in=(100, 100))
    assert p.status == O.FITS and len(p.records) == 1
    assert (int(p.a2[0]), int(p.b2[0])) == (2, 17)
    f = p.prefetch()
    # walking back from slot 17: slots 17..11 hold A (0 + 100 <= 150); slot 10 (100 + 100) does not
    assert f.gained.tolist() == [7] and f.absent_last.tolist() == [10]
    assert f.pressure.tolist() == [100, 100] + [0] * 7 + [100, 100] + [100] * 7 + [100, 100]
    # capacity 100: still fits after the eviction (slots 9,10 at 100), and no slot can take A back
    # together with ... slot 17 holds 0 + 100 <= 100: every free slot holds it, up to the bump
    p = v.plan(gpu_cap=100, host_cap=0, bw_out=(100, 100), bw_in=(100, 100))
    assert p.prefetch().gained.tolist() == [7]
    # capacity 99 < size: nothing can ever hold the tensor again; the plan ends residual
    p = v.plan(gpu_cap=99, host_cap=0, bw_out=(100, 100), bw_in=(100, 100))
    f = p.prefetch()
    assert f.gained.tolist() == [0] * len(p.records) and (f.pressure == p.pressure_after).all()
    # without the bump the plan is empty and so is the prefetch pass
    p = v.plan(gpu_cap=1000, host_cap=0, bw_out=(100, 100), bw_in=(100, 100))
    f = p.prefetch()
    assert len(f.gained) == 0 and (f.pressure == v.pressure).all()


@pytest.mark.parametrize("mode", [O.DIRECT, O.PREFIX])
def test_whole_window_can_come_back(mode):
    # the bump that forced the eviction belongs to a tensor evicted later itself: afterwards A's
    # whole absent window has room, and the search stops at the first absent slot
    tr = _uniform(12, [100, 300], [(0, 0), (11, 0), (0, 1), (5, 1), (6, 1), (11, 1)])
    v = O.Vitality(tr, mode)
    p = v.plan(gpu_cap=350, host_cap=0, bw_out=(1000, 1000), bw_in=(1000, 1000))
    f = p.prefetch()
    for i in range(len(p.records)):
        assert f.gained[i] <= p.b2[i] - p.a2[i] + 1
    o, g, pr = prefetchcheck.replay(v.K, v.start, 350, p.records, p.a2, p.b2, p.pressure_after)
    assert (f.order == o).all() and (f.gained == g).all() and (f.pressure == pr).all()
    assert (f.pressure <= np.maximum(p.pressure_after, 350)).all()


def _invariants(v, p, f, cap):
    K = v.K
    n = len(p.records)
    # visiting order: by latest safe prefetch time, ties in plan order
    T = int(v.start[K])
    R2 = p.records["next_use"].astype(np.int64) + np.where(p.records["wraps"] > 0, K, 0)
    st2 = np.concatenate([v.start[:K].astype(np.int64), v.start[:K].astype(np.int64) + T])
    t_safe = st2[R2] - p.records["t_in"].astype(np.int64)
    key = list(zip(t_safe[f.order].tolist(), f.order.tolist()))
    assert key == sorted(key) and sorted(f.order.tolist()) == list(range(n))
    # the pressure rises exactly by the tensors over the slots gained
    add = np.zeros(K, np.int64)
    for i in range(n):
        for j in range(int(p.b2[i]) - int(f.gained[i]) + 1, int(p.b2[i]) + 1):
            add[j % K] += int(p.records["size"][i])
    assert (f.pressure.astype(np.int64) == p.pressure_after.astype(np.int64) + add).all()
    # no slot that took a tensor back exceeds the capacity; untouched slots are unchanged
    assert (f.pressure[add > 0] <= cap).all()
    assert (f.gained <= p.b2 - p.a2 + 1).all()
    assert (f.absent_last == (p.b2.astype(np.int64) - f.gained) % K).all()


@pytest.mark.parametrize("seed", range(30))
def test_random_small_against_replay(seed):
    w = traces.random_small(7000 + seed, K=8 + seed % 25, N=5 + seed % 14, max_uses=5)
    no_wrap = seed % 5 == 0
    v0 = O.Vitality(w.trace, O.DIRECT, no_wrap=no_wrap)
    v1 = O.Vitality(w.trace, O.PREFIX, no_wrap=no_wrap)
    cap, hcap = traces.resolve_caps(w, v0.peak)
    for frac in (1.0, 1.3):
        args = dict(gpu_cap=int(cap * frac), host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
        p0, p1 = v0.plan(**args), v1.plan(**args)
        f0, f1 = p0.prefetch(), p1.prefetch()
        assert (f0.order == f1.order).all() and (f0.gained == f1.gained).all() and (f0.pressure == f1.pressure).all()
        a2, b2 = prefetchcheck.doubled_windows(v0.K, p0.records)
        assert (a2 == p0.a2).all() and (b2 == p0.b2).all()
        o, g, pr = prefetchcheck.replay(v0.K, v0.start, args["gpu_cap"], p0.records, a2, b2, p0.pressure_after)
        assert (f0.order == o).all() and (f0.gained == g).all() and (f0.pressure == pr).all()
        _invariants(v0, p0, f0, args["gpu_cap"])


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_configs_invariants(cfg):
    w = traces.config(cfg)
    v = O.Vitality(w.trace, O.PREFIX)
    cap, hcap = traces.resolve_caps(w, v.peak)
    args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    p = v.plan(**args)
    f = p.prefetch()
    _invariants(v, p, f, cap)
    o, g, pr = prefetchcheck.replay(v.K, v.start, cap, p.records, p.a2, p.b2, p.pressure_after)
    assert (f.order == o).all() and (f.gained == g).all() and (f.pressure == pr).all()
    o, g, pr = prefetchcheck.replay_numpy(v.K, v.start, cap, p.records, p.a2, p.b2, p.pressure_after)
    assert (f.order == o).all() and (f.gained == g).all() and (f.pressure == pr).all()
