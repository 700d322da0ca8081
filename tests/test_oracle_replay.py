"""Pins for the oracle's slot-level plan replay: a hand-worked example, closed forms for one
migration, a differently formulated solver on small traces, invariants."""
import numpy as np
import pytest

import replaycheck
from goldenio import Golden
from oracle import oracle as O
from paper_2310_09443_amd import traces
from paper_2310_09443_amd.traces import Trace


def _plan(w, v, **over):
    cap, hcap = traces.resolve_caps(w, v.peak)
    args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    args.update(over)
    return v.plan(**args)


def test_hand_worked_replay():
    g = Golden("hand_replay.txt")
    v = O.Vitality(g.trace)
    p = v.plan(**g.plan_args())
    fields = ["cand", "tensor", "evict_after", "absent_first", "absent_last", "next_use", "dest", "wraps", "size", "t_out", "t_in"]
    assert [[int(r[f]) for f in fields] + [int(r["benefit_lo"])] for r in p.records] == g.expect["record"]
    e = g.expect
    r = p.replay()
    assert [r.iter_ns, r.planned_ns, r.stall_ns, r.n_stalled] == e["replay_planned"][0] and r.late.tolist() == e["late_planned"][0]
    r = p.replay(dur=np.array(g.params["replay_dur"], np.uint64))
    assert [r.iter_ns, r.planned_ns, r.stall_ns, r.n_stalled] == e["replay"][0] and r.late.tolist() == e["late"][0]
    assert r.bytes + r.busy_out_ns + r.busy_in_ns == e["traffic"][0]


def test_hand_worked_replay_two_iteration_copies_at_one_point():
    """A cross-iteration period's prefetch (first copy) and the second copy's prefetch of a
    migration ranked before it are issued at the same point on the same channel:
    they queue in plan order, whichever copy they belong to.  The other order would stall 8000 ns."""
    g = Golden("hand_replay_two_copies.txt")
    v = O.Vitality(g.trace)
    p = v.plan(**g.plan_args(), **g.variant_args())
    fields = ["cand", "tensor", "evict_after", "absent_first", "absent_last", "next_use", "dest", "wraps", "size", "t_out", "t_in"]
    assert [[int(r[f]) for f in fields] + [int(r["benefit_lo"])] for r in p.records] == g.expect["record"]
    e = g.expect
    r = p.replay()
    assert [r.iter_ns, r.planned_ns, r.stall_ns, r.n_stalled] == e["replay_planned"][0] and r.late.tolist() == e["late_planned"][0]
    assert r.bytes + r.busy_out_ns + r.busy_in_ns == e["traffic"][0]
    # the differently formulated solver agrees, and a queue in the other order is what it would cost
    recs = [{k: int(x[k]) for k in ("evict_after", "dest", "t_out", "t_in")} for x in p.records]
    K = g.trace.K
    b2 = [int(x["absent_last"]) + (K if int(x["absent_last"]) < int(x["evict_after"]) else 0) for x in p.records]
    R2 = [int(x["next_use"]) + (K if x["wraps"] else 0) for x in p.records]
    assert replaycheck.solve(K, g.trace.dur_ns, recs, b2, R2)[:4] == (100000, 100000, 0, 0)
    swapped = replaycheck.solve(K, g.trace.dur_ns, recs[::-1], b2[::-1], R2[::-1])
    assert swapped[:4] == (108000, 100000, 8000, 1) and swapped[4] == [0, 8000]


def test_no_migration_no_stall():
    w = traces.encoder12()
    v = O.Vitality(w.trace, O.PREFIX)
    p = _plan(w, v, gpu_cap=v.peak)
    assert len(p.records) == 0
    r = p.replay()
    assert (r.iter_ns, r.stall_ns, r.n_stalled, r.bytes) == (v.T, 0, 0, [0, 0])
    d = traces.noisy_durations(w.trace, 20, seed=3)
    r = p.replay(dur=d)
    assert (r.iter_ns, r.planned_ns, r.stall_ns) == (int(d.sum()), int(d.sum()), 0)


@pytest.mark.parametrize("seed", range(12))
def test_one_migration_closed_form(seed):
    """One migration alone on its channels: with the planned durations it never stalls (that is
    what the window's ends mean); with other durations the wait is
    max(0, max(end of the last absent kernel, end of the eviction) + t_in - end of kernel R - 1)."""
    K = 30
    rng = np.random.default_rng(seed)
    dur = rng.integers(1000, 20000, K).astype(np.uint64)
    L, R = int(rng.integers(0, 5)), int(rng.integers(20, K))
    tr = Trace("one", dur, np.array([4000 * (1 + seed)], np.uint64), np.array([0], np.uint8),
               np.array([L, R], np.uint32), np.array([0, 0], np.uint32))
    v = O.Vitality(tr)
    p = v.plan(gpu_cap=1, host_cap=0, bw_out=(900, 900), bw_in=(700, 700))
    assert len(p.records) == 1
    rec = p.records[0]
    assert p.replay().stall_ns == 0
    d2 = rng.integers(100, 30000, K).astype(np.uint64)
    end = np.cumsum(d2.astype(np.int64))                    # end of kernel j without stalls
    b = int(rec["absent_last"])
    wait = max(0, max(int(end[b]), int(end[L]) + int(rec["t_out"])) + int(rec["t_in"]) - int(end[R - 1]))
    r = p.replay(dur=d2)
    assert (r.stall_ns, r.n_stalled, r.late.tolist()) == (wait, int(wait > 0), [wait])
    assert r.iter_ns == int(d2.sum()) + wait


@pytest.mark.parametrize("seed", range(40))
def test_small_traces_against_the_equations(seed):
    w = traces.random_small(9000 + seed, K=8 + seed % 9, N=5 + seed % 6, max_uses=4)
    v = O.Vitality(w.trace, O.DIRECT)
    cap, hcap = traces.resolve_caps(w, v.peak)
    bw = (300, 900) if seed % 2 else w.bw_out_Bpus
    p = v.plan(gpu_cap=cap, host_cap=max(hcap, int(v.peak)), bw_out=bw, bw_in=bw)
    f = p.prefetch()
    recs = [{k: int(r[k]) for k in ("evict_after", "dest", "t_out", "t_in")} for r in p.records]
    R2 = [int(r["next_use"]) + (w.trace.K if r["wraps"] else 0) for r in p.records]
    for dur in (w.trace.dur_ns, traces.noisy_durations(w.trace, 25, seed=seed),
                np.maximum(w.trace.dur_ns // 7, 1).astype(np.uint64)):
        for eager in (False, True):
            r = p.replay(dur=dur, eager=eager)
            exp = replaycheck.solve(w.trace.K, dur, recs, p.b2, R2, f.gained if eager else None)
            assert (r.iter_ns, r.planned_ns, r.stall_ns, r.n_stalled, r.late.tolist()) == exp
            assert r.iter_ns == r.planned_ns + r.stall_ns


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_configs_invariants(cfg):
    w = traces.config(cfg)
    v = O.Vitality(w.trace, O.PREFIX)
    p = _plan(w, v)
    f = p.prefetch()
    for eager in (False, True):
        r = p.replay(eager=eager)
        assert r.iter_ns == r.planned_ns + r.stall_ns and r.planned_ns == v.T
        assert r.n_stalled <= int((r.late > 0).sum()) <= len(p.records)
        assert int(r.late.max(initial=0)) <= r.stall_ns or r.n_stalled > 0
        for d in range(2):
            sel = p.records["dest"] == d
            assert r.bytes[d] == int(p.records["size"][sel].sum())
            assert r.busy_out_ns[d] == int(p.records["t_out"][sel].sum()) and r.busy_in_ns[d] == int(p.records["t_in"][sel].sum())


def test_bad_durations_are_errors():
    w = traces.mlp_tiny()
    v = O.Vitality(w.trace)
    p = _plan(w, v)
    d = w.trace.dur_ns.copy()
    d[2] = 0
    with pytest.raises(O.OracleError):
        p.replay(dur=d)
    with pytest.raises(O.OracleError):
        v2 = O.Vitality(w.trace)
        _plan(w, v2).replay(eager=True)            # smart prefetching has not run on this plan
