"""Parity of g10_replay (slot-level replay of a plan) against the oracle's replay, through the
C ABI.  Integer work: every comparison is exact."""
import numpy as np
import pytest

from goldenio import Golden
from oracle import oracle as O
from paper_2310_09443_amd import traces
from test_gpu_parity import assert_plan_equal, g10, run_both  # noqa: F401  (g10 is a fixture)

pytestmark = pytest.mark.gpu


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, np.uint64).view(np.int64)).to("cuda:0")


def assert_replay_equal(r, o):
    assert (r.iter_ns, r.planned_ns, r.stall_ns, r.n_stalled) == (o.iter_ns, o.planned_ns, o.stall_ns, o.n_stalled)
    assert (r.bytes, r.busy_out_ns, r.busy_in_ns) == (o.bytes, o.busy_out_ns, o.busy_in_ns)
    assert (r.late == o.late).all()


def both(h, p, durs):
    """Replays of the plan on the handle against the oracle plan p: as planned and with smart prefetching."""
    for dur in durs:
        assert_replay_equal(h.replay(None if dur is None else dev(dur)), p.replay(dur))
    f = p.prefetch()
    h.prefetch()
    for dur in durs:
        assert_replay_equal(h.replay(None if dur is None else dev(dur), eager=True), p.replay(dur, eager=True))


def test_worked_example(g10):
    g = Golden("hand_replay.txt")
    v = O.Vitality(g.trace, O.DIRECT)
    h = g10.g10_vitality(g10.DeviceTrace(g.trace))
    assert_plan_equal(h.plan(**g.plan_args()), v.plan(**g.plan_args()))
    e = g.expect
    r = h.replay()
    assert [r.iter_ns, r.planned_ns, r.stall_ns, r.n_stalled] == e["replay_planned"][0] and r.late.tolist() == e["late_planned"][0]
    r = h.replay(dev(np.array(g.params["replay_dur"], np.uint64)))
    assert [r.iter_ns, r.planned_ns, r.stall_ns, r.n_stalled] == e["replay"][0] and r.late.tolist() == e["late"][0]
    assert r.bytes + r.busy_out_ns + r.busy_in_ns == e["traffic"][0]
    h.close()


@pytest.mark.parametrize("seed", range(40))
def test_random_small(g10, seed):
    w = traces.random_small(9000 + seed, K=6 + seed % 20, N=4 + seed % 13, max_uses=5)
    h, v, args = run_both(g10, w, no_wrap=seed % 4 == 0)
    bw = (300, 900) if seed % 2 else args["bw_out"]
    args = dict(args, host_cap=max(args["host_cap"], int(v.peak)), bw_out=bw, bw_in=bw)
    p = v.plan(**args)
    assert_plan_equal(h.plan(**args), p)
    tr = w.trace
    both(h, p, [None, traces.noisy_durations(tr, 25, seed=seed), np.maximum(tr.dur_ns // 7, 1).astype(np.uint64),
                (tr.dur_ns * np.uint64(3)).astype(np.uint64)])
    h.close()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_configs(g10, cfg):
    w = traces.config(cfg)
    h, v, args = run_both(g10, w)
    p = v.plan(**args)
    assert_plan_equal(h.plan(**args), p)
    both(h, p, [None, traces.noisy_durations(w.trace, 5, seed=1), traces.noisy_durations(w.trace, 25, seed=2),
                np.maximum(w.trace.dur_ns // 2, 1).astype(np.uint64)])
    # a plan made for durations of its own is replayed with those unless told otherwise
    d = traces.noisy_durations(w.trace, 20, seed=3)
    vo = O.Vitality(traces.with_durations(w.trace, d), O.PREFIX)
    po = vo.plan(**args)
    assert_plan_equal(h.plan(dur=dev(d), **args), po)
    assert_replay_equal(h.replay(), po.replay())
    assert_replay_equal(h.replay(dev(w.trace.dur_ns)), po.replay(w.trace.dur_ns))
    h.close()


@pytest.mark.parametrize("K,N,seed", [(2048, 20000, 2), (5000, 60000, 3)])
def test_stress_scaled(g10, K, N, seed):
    """More events than one block of the sort; many transfers queue on the same channel."""
    w = traces.stress(K=K, N=N, seed=seed)
    h, v, args = run_both(g10, w)
    p = v.plan(**args)
    assert_plan_equal(h.plan(**args), p)
    both(h, p, [None, traces.noisy_durations(w.trace, 20, seed=5)])
    h.close()


def test_errors_and_no_migrations(g10):
    w = traces.encoder12()
    h, v, args = run_both(g10, w)
    with pytest.raises(g10.G10Error) as e:
        h.replay()                                           # no plan on the handle yet
    assert e.value.code == g10.EINVAL
    p = v.plan(**dict(args, gpu_cap=v.peak))
    h.plan(**dict(args, gpu_cap=v.peak))
    assert_replay_equal(h.replay(), p.replay())              # nothing migrates: the iteration as profiled
    assert h.replay().iter_ns == v.T
    h.plan(**args)
    with pytest.raises(g10.G10Error) as e:
        h.replay(eager=True)                                 # smart prefetching has not run on this plan
    assert e.value.code == g10.EINVAL
    d = w.trace.dur_ns.copy()
    d[3] = 0
    with pytest.raises(g10.G10Error) as e:
        h.replay(dev(d))
    assert e.value.code == g10.EINVAL
    assert_replay_equal(h.replay(), v.plan(**args).replay())
    h.close()


def test_stress_full_size(g10):
    """Config 5 at full size: 9246 migrations, 55 476 events."""
    w = traces.config(5)
    h, v, args = run_both(g10, w)
    p = v.plan(max_iters=200, **args)                        # the oracle's plan: a prefix (the full one takes minutes)
    r = h.plan(max_iters=200, **args)
    assert_plan_equal(r, p, prefix=True)
    both(h, p, [None, traces.noisy_durations(w.trace, 20, seed=9)])
    # the whole plan: the figures must be consistent (the oracle has no plan to replay here)
    h.plan(**args)
    full = h.replay()
    assert full.iter_ns == full.planned_ns + full.stall_ns and full.planned_ns == v.T
    assert int(full.late.max()) <= full.stall_ns and full.n_stalled <= int((full.late > 0).sum())
    h.close()
