"""Parity of the HIP library against the CPU oracle, through the C ABI.

Integer work throughout: every comparison is exact (bit-for-bit)."""
import numpy as np
import pytest

import plancheck
import prefetchcheck
from goldenio import Golden
from oracle import oracle as O
from paper_2310_09443_amd import traces
from paper_2310_09443_amd.traces import Trace

pytestmark = pytest.mark.gpu

FIELDS = ["cand", "tensor", "evict_after", "absent_first", "absent_last", "next_use", "dest", "wraps",
          "size", "t_out", "t_in", "benefit_lo", "benefit_hi"]


@pytest.fixture(scope="module")
def g10():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2310_09443_amd import binding
    binding.load()
    return binding


def assert_vitality_equal(h, v):
    assert (h.n_uses, h.C, h.peak, h.T) == (v.n_uses, v.C, v.peak, v.T)
    assert (h.use_off == v.use_off).all()
    assert (h.use_k == v.use_k).all()
    assert (h.per_tensor == v.per_tensor).all()
    assert (h.per_L == v.per_L).all()
    assert (h.per_R == v.per_R).all()
    assert (h.start == v.start).all()
    assert (h.pressure == v.pressure).all()


def assert_plan_equal(r, p, prefix=False):
    n = len(p.records)
    if prefix:
        assert len(r.records) >= n
    else:
        assert len(r.records) == n
        assert r.status == p.status
        assert (r.n_iterations, r.n_dropped, r.n_cand_evals) == (p.n_iterations, p.n_null, p.n_cand_evals)
        assert (r.peak_before, r.peak_after) == (p.peak_before, p.peak_after)
        assert (r.overtime_before_ns, r.overtime_after_ns) == (p.overtime_before, p.overtime_after)
        assert (r.pressure_after == p.pressure_after).all()
        assert (r.null_iters == p.null_iters).all() and (r.null_cands == p.null_cands).all()
    for f in FIELDS:
        assert (r.records[f][:n] == p.records[f]).all(), f


def assert_prefetch_equal(f, fo):
    """g10_prefetch against the oracle's smart prefetching on the same plan."""
    assert (f.n_migrations, f.n_moved, f.slots_gained) == (len(fo.gained), fo.n_moved, fo.slots_gained)
    assert (f.order == fo.order).all()
    assert (f.gained == fo.gained).all()
    assert (f.absent_last == fo.absent_last).all()
    assert (f.pressure == fo.pressure).all() and f.peak == fo.peak


def run_both(g10, w, no_wrap=False, **over):
    tr = w.trace
    v = O.Vitality(tr, O.PREFIX, no_wrap=no_wrap)
    h = g10.g10_vitality(g10.DeviceTrace(tr), no_wrap=no_wrap)
    assert_vitality_equal(h, v)
    cap, hcap = traces.resolve_caps(w, v.peak)
    args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    args.update(over)
    return h, v, args


@pytest.mark.parametrize("name", ["fig6_listing.txt", "hand_plan_a.txt", "hand_plan_b.txt", "hand_prefetch.txt"])
def test_worked_examples(g10, name):
    g = Golden(name)
    v = O.Vitality(g.trace, O.DIRECT)
    h = g10.g10_vitality(g10.DeviceTrace(g.trace))
    assert_vitality_equal(h, v)
    if "gpu_cap" in g.params:
        r = h.plan(**g.plan_args())
        assert_plan_equal(r, v.plan(**g.plan_args()))
        fields = FIELDS[:-2]
        got = [[int(x[f]) for f in fields] + [int(x["benefit_lo"]) + (int(x["benefit_hi"]) << 64)] for x in r.records]
        assert got == g.expect["record"]            # the values derived by hand, directly
        f = h.prefetch()
        assert_prefetch_equal(f, v.plan(**g.plan_args()).prefetch())
        if "gained" in g.expect:
            assert f.order.tolist() == g.expect["prefetch_order"][0] and f.gained.tolist() == g.expect["gained"][0]
            assert f.absent_last.tolist() == g.expect["absent_last_eager"][0]
            assert f.pressure.tolist() == g.expect["pressure_eager"][0]
    h.close()


@pytest.mark.parametrize("seed", range(40))
def test_random_small(g10, seed):
    w = traces.random_small(5000 + seed, K=6 + seed % 20, N=4 + seed % 13, max_uses=5)
    no_wrap = seed % 4 == 0
    h, v, args = run_both(g10, w, no_wrap=no_wrap)
    p = v.plan(mode=O.DIRECT, **args)
    assert_plan_equal(h.plan(**args), p)
    assert_prefetch_equal(h.prefetch(), p.prefetch(O.DIRECT))
    args2 = dict(args, gpu_cap=int(args["gpu_cap"] * 1.3))      # more room: prefetches do move
    p = v.plan(mode=O.DIRECT, **args2)
    assert_plan_equal(h.plan(**args2), p)
    assert_prefetch_equal(h.prefetch(), p.prefetch(O.DIRECT))
    h.close()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_configs(g10, cfg):
    w = traces.config(cfg)
    h, v, args = run_both(g10, w)
    p = v.plan(**args)
    r = h.plan(**args)
    assert_plan_equal(r, p)
    assert_prefetch_equal(h.prefetch(), p.prefetch())
    # same handle, different machine: the analysis is not modified by planning
    args2 = dict(args, gpu_cap=int(v.peak * 0.9), host_cap=0)
    assert_plan_equal(h.plan(**args2), v.plan(**args2))
    assert_plan_equal(h.plan(**args), p)
    h.close()


@pytest.mark.parametrize("K,N,seed", [(257, 3000, 1), (2048, 20000, 2), (5000, 60000, 3), (300, 100000, 4)])
def test_stress_scaled(g10, K, N, seed):
    """Several sort tiles, several timeline chunks, ragged tails."""
    w = traces.stress(K=K, N=N, seed=seed)
    h, v, args = run_both(g10, w)
    assert_plan_equal(h.plan(**args), v.plan(**args))
    # a capacity that can be reached: ends with FITS
    args2 = dict(args, gpu_cap=int(v.peak * 0.97), host_cap=2 ** 62)
    p2 = v.plan(**args2)
    assert_plan_equal(h.plan(**args2), p2)
    f2 = h.prefetch()
    assert_prefetch_equal(f2, p2.prefetch())
    assert f2.n_moved > 0
    h.close()


@pytest.mark.parametrize("max_tiles,max_chunks", [(1, 1), (3, 2), (16, 5), (0, 3), (2, 0)])
def test_tile_and_chunk_limits(g10, max_tiles, max_chunks):
    """Large tiles (several scoring units per tile) and long chunks (several strips per
    chunk job), reached with a small trace by lowering the limits; the plan does not
    depend on them.  The same handle is laid out again when the chunk limit changes."""
    w = traces.stress(K=2048, N=20000, seed=2)
    h, v, args = run_both(g10, w)
    p = v.plan(**args)
    assert_plan_equal(h.plan(max_tiles=max_tiles, max_chunks=max_chunks, **args), p)
    assert_plan_equal(h.plan(**args), p)
    args2 = dict(args, gpu_cap=int(v.peak * 0.97), host_cap=2 ** 62)
    p2 = v.plan(**args2)
    assert_plan_equal(h.plan(max_tiles=max_tiles, max_chunks=max_chunks, **args2), p2)
    assert_prefetch_equal(h.prefetch(), p2.prefetch())        # chunks of the same length as the plan's
    h.close()


@pytest.mark.parametrize("frac", [0.002, 0.004, 0.1])
def test_tight_host_memory(g10, frac):
    """Host memory fills up: winners are dropped, the exact per-slot host check runs."""
    w = traces.stress(K=3000, N=30000, seed=7)
    h, v, args = run_both(g10, w)
    args = dict(args, host_cap=int(v.peak * frac), bw_out=(50, 25000), bw_in=(50, 25000))   # flash too slow for most
    p = v.plan(**args)
    r = h.plan(**args)
    assert_plan_equal(r, p)
    assert (r.records["dest"] == 1).any() and (r.n_dropped > 0 or frac > 0.05)
    h.close()


def test_long_timeline(g10):
    """More kernels than 512 chunks of 256 slots hold: two strips per chunk job by default."""
    w = traces.stress(K=140000, N=6000, seed=11)
    h, v, args = run_both(g10, w)
    p = v.plan(max_iters=600, **args)
    r = h.plan(max_iters=600, **args)
    assert r.status == g10.TRUNCATED == p.status and r.n_iterations == 600
    assert_plan_equal(r, p, prefix=True)
    assert (r.pressure_after == p.pressure_after).all()
    h.close()


def test_plan_batch(g10):
    """A sweep in one call: every plan of the batch equals the plan made alone (and the oracle's)."""
    w = traces.stress(K=2048, N=20000, seed=2)
    h, v, args = run_both(g10, w)
    sweep = []
    for cap_frac in (0.25, 0.5, 0.9, 1.0):
        for hfrac, bw in ((0.25, (6000, 25000)), (0.0, (12000, 25000)), (0.01, (50, 25000))):
            sweep.append(dict(gpu_cap=int(v.peak * cap_frac), host_cap=int(v.peak * hfrac), bw_out=bw, bw_in=bw))
    sweep.append(dict(sweep[0], max_iters=37))
    sweep.append(dict(sweep[1], max_tiles=2, max_chunks=3))
    first = h.plan_batch(sweep[:2])                      # a small batch first: the next one needs more workspaces
    rs = h.plan_batch(sweep)
    assert len(rs) == len(sweep)
    assert all(x.records.tobytes() == y.records.tobytes() and (x.pressure_after == y.pressure_after).all()
               for x, y in zip(first, rs))
    for d, r in zip(sweep, rs):
        oa = {k: x for k, x in d.items() if k not in ("max_tiles", "max_chunks")}
        p = v.plan(**oa) if "max_iters" in oa else v.plan(**oa)
        if "max_iters" in d:
            assert r.status == g10.TRUNCATED == p.status and r.n_iterations == 37
            assert_plan_equal(r, p, prefix=True)
        else:
            assert_plan_equal(r, p)
    # the prefetch pass refers to the first plan of the batch
    assert_prefetch_equal(h.prefetch(), v.plan(**sweep[0]).prefetch())
    # a smaller batch and a single plan on the same handle afterwards
    rs2 = h.plan_batch(sweep[3:5])
    assert rs2[0].records.tobytes() == rs[3].records.tobytes() and rs2[1].records.tobytes() == rs[4].records.tobytes()
    assert_plan_equal(h.plan(**args), v.plan(**args))
    h.close()


def test_plan_batch_shared_windows_and_retilings(g10):
    """Plans of a batch with equal bandwidths and durations share their candidate windows (also when the first
    of them has nothing to do), and long lists are put back into score order for all plans at once."""
    w = traces.stress(K=16384, N=120000, seed=5)
    h, v, args = run_both(g10, w)
    a, b = (6000, 25000), (3000, 25000)
    sweep = [dict(gpu_cap=v.peak, host_cap=v.peak // 4, bw_out=a, bw_in=a),            # fits: no pass at all
             dict(gpu_cap=int(v.peak * 0.3), host_cap=v.peak // 4, bw_out=b, bw_in=b),
             dict(gpu_cap=int(v.peak * 0.3), host_cap=v.peak // 4, bw_out=a, bw_in=a),
             dict(gpu_cap=int(v.peak * 0.2), host_cap=v.peak // 8, bw_out=a, bw_in=a),
             dict(gpu_cap=int(v.peak * 0.25), host_cap=v.peak // 4, bw_out=b, bw_in=b),
             dict(gpu_cap=int(v.peak * 0.25), host_cap=v.peak // 4, bw_out=b, bw_in=a, rank=1, max_iters=1200)]
    rs = h.plan_batch(sweep)
    assert rs[0].status == g10.FITS and rs[0].n_iterations == 0
    for d, r in zip(sweep, rs):
        assert_plan_equal(r, v.plan(**d), prefix="max_iters" in d)
    # (the launches of a batch end by the clock, so whether a plan of some 300 rounds of commits is re-tiled before it
    # is done varies from run to run: most of them are, and several in the same launches)
    assert sum(r.loop_retiles > 0 for r in rs[1:]) >= 3, [(r.n_iterations, r.score_full_cands, r.loop_retiles) for r in rs]
    # the same plans in another order, and alone
    rs2 = h.plan_batch(sweep[::-1])
    for r, q in zip(rs, rs2[::-1]):
        assert r.records.tobytes() == q.records.tobytes() and (r.pressure_after == q.pressure_after).all()
    assert h.plan(**sweep[3]).records.tobytes() == rs[3].records.tobytes()
    h.close()


@pytest.mark.parametrize("one_beyond", [False, True])
def test_first_scoring_pass_both_copy_forms(g10, one_beyond):
    """The first scoring pass reads a 16-byte copy of every candidate when no tensor has 2^43 bytes or more
    (and 2 K <= 2^21), a 24-byte one otherwise: sizes that use all 43 bits, and the same with one tensor beyond."""
    w = traces.stress(K=2048, N=20000, seed=9)
    tr = w.trace
    size = tr.size_bytes << np.uint64(14)
    assert (1 << 42) <= int(size.max()) < (1 << 43)
    if one_beyond:
        size[int(np.argmax(size))] = 1 << 43
    big = Trace("sizes", tr.dur_ns, size, tr.is_global, tr.use_kernel, tr.use_tensor)
    v = O.Vitality(big, O.PREFIX)
    h = g10.g10_vitality(g10.DeviceTrace(big))
    assert_vitality_equal(h, v)
    bw = (6000 << 14, 25000 << 14)
    args = dict(gpu_cap=int(v.peak * 0.3), host_cap=int(v.peak // 4), bw_out=bw, bw_in=bw)
    for va in (dict(), dict(rank=1, max_iters=300)):
        r, p = h.plan(**args, **va), v.plan(**args, **va)
        assert_plan_equal(r, p, prefix="max_iters" in va)
        assert "rank" in va or int((p.records["size"] >= (1 << 42)).sum()) > 0      # candidates whose size has bit 42 set
    h.close()


@pytest.mark.parametrize("block", range(4))
def test_random_batches(g10, block):
    """Random traces, random batches: capacities, host capacities and bandwidths drawn from small sets (so some
    plans share their candidate windows and some do not), the readings, pass limits and lowered on-chip limits
    mixed; every plan against the oracle, then one of them alone with its prefetch pass and its replay."""
    import random
    for case in range(12 * block, 12 * block + 12):
        rnd = random.Random(424200 + case)
        kind = rnd.choice(["small", "small", "mid", "stress"])
        if kind == "small":
            w = traces.random_small(70000 + case, K=rnd.randint(4, 40), N=rnd.randint(3, 30), max_uses=rnd.randint(2, 5))
        elif kind == "mid":
            w = traces.random_small(80000 + case, K=rnd.randint(100, 600), N=rnd.randint(50, 800), max_uses=rnd.randint(2, 4))
        else:
            w = traces.stress(K=rnd.choice([512, 1024, 3000]), N=rnd.choice([2000, 9000, 20000]), seed=90000 + case)
        h, v, args = run_both(g10, w)
        b0 = w.bw_out_Bpus
        bws = [b0, (max(1, b0[0] // 2), b0[1]), (b0[0], max(1, b0[1] // 3))]
        sweep = []
        for _ in range(rnd.randint(2, 7)):
            bw = rnd.choice(bws)
            d = dict(gpu_cap=max(1, int(v.peak * rnd.choice([0.1, 0.25, 0.5, 0.8, 1.0, 1.2]))),
                     host_cap=int(v.peak * rnd.choice([0.0, 0.05, 0.25, 2.0])), bw_out=bw, bw_in=rnd.choice([bw, b0]))
            if rnd.random() < 0.3:
                d["rank"] = 1
            if rnd.random() < 0.3 and kind != "stress":
                d["area"] = 1
            if rnd.random() < 0.2:
                d["max_iters"] = rnd.randint(1, 60)
            if "rank" in d and kind == "stress" and "max_iters" not in d:
                d["max_iters"] = 400
            sweep.append(d)
        limits = [dict(d) for d in sweep]
        for d in limits:
            if rnd.random() < 0.3:
                d["max_tiles"] = rnd.randint(1, 4)
            if rnd.random() < 0.3:
                d["max_chunks"] = rnd.randint(1, 5)
        for d, r in zip(sweep, h.plan_batch(limits)):
            p = v.plan(**d)
            assert_plan_equal(r, p, prefix=p.status == O.TRUNCATED)
            assert (r.status, r.n_iterations) == (p.status, p.n_iterations), (case, d)
            assert (r.pressure_after == p.pressure_after).all() and (r.null_cands == p.null_cands).all(), (case, d)
        r, p = h.plan(**sweep[0]), v.plan(**sweep[0])
        assert r.records.tobytes() == p.records.tobytes(), (case, sweep[0])
        assert_prefetch_equal(h.prefetch(), p.prefetch())
        y, yo = h.replay(eager=True), p.replay(eager=True)
        assert (y.iter_ns, y.stall_ns, y.n_stalled) == (yo.iter_ns, yo.stall_ns, yo.n_stalled) and (y.late == yo.late).all()
        h.close()


def test_plan_with_other_durations(g10):
    """Re-planning under kernel-time noise: a plan made with durations of its own equals the
    oracle's plan of the trace that has these durations, alone and inside a batch, and so does
    the smart prefetching on it; the handle's own analysis stays as it was."""
    import torch
    for w in (traces.encoder12(), traces.stress(K=2048, N=20000, seed=2)):
        h, v, args = run_both(g10, w)
        base = v.plan(**args)
        sweep, oracles = [dict(args)], [v]
        keep = []
        for pct in (5.0, 20.0, 25.0):
            d = traces.noisy_durations(w.trace, pct, seed=int(pct))
            dv = torch.from_numpy(d.view(np.int64)).to("cuda:0")
            keep.append(dv)
            sweep.append(dict(args, dur=dv))
            oracles.append(O.Vitality(traces.with_durations(w.trace, d), O.PREFIX))
            assert (oracles[-1].per_L == v.per_L).all() and (oracles[-1].pressure == v.pressure).all()
        oargs = {k: x for k, x in args.items()}
        # alone
        r = h.plan(**sweep[2])
        po = oracles[2].plan(**oargs)
        assert_plan_equal(r, po)
        assert_prefetch_equal(h.prefetch(), po.prefetch())
        # in a batch, next to a plan on the analysed durations
        rs = h.plan_batch(sweep)
        plans = [o.plan(**oargs) for o in oracles]
        for r, po in zip(rs, plans):
            assert_plan_equal(r, po)
        assert any(len(po.records) != len(base.records) or po.records.tobytes() != base.records.tobytes() for po in plans[1:])
        # the analysis is untouched: the plain plan again
        assert (h.start == v.start).all()
        assert_plan_equal(h.plan(**args), base)
        assert_prefetch_equal(h.prefetch(), base.prefetch())
        h.close()


def test_other_durations_errors(g10):
    import torch
    w = traces.random_small(3)
    h, v, args = run_both(g10, w)
    d = w.trace.dur_ns.copy()
    d[1] = 0
    with pytest.raises(g10.G10Error) as e:
        h.plan(**dict(args, dur=torch.from_numpy(d.view(np.int64)).to("cuda:0")))
    assert e.value.code == g10.EINVAL
    d[1] = 2 ** 62
    with pytest.raises(g10.G10Error) as e:
        h.plan(**dict(args, dur=torch.from_numpy(d.view(np.int64)).to("cuda:0")))
    assert e.value.code == g10.EOVERFLOW
    with pytest.raises(ValueError):
        h.plan(**dict(args, dur=torch.zeros(w.trace.K + 1, dtype=torch.int64, device="cuda:0")))
    assert_plan_equal(h.plan(**args), v.plan(**args))          # the handle still plans
    h.close()


def test_iteration_limit(g10):
    w = traces.resnet152()
    h, v, args = run_both(g10, w)
    p = v.plan(max_iters=70, **args)
    r = h.plan(max_iters=70, **args)
    assert r.status == g10.TRUNCATED == p.status
    assert r.n_iterations == 70 and len(r.records) == len(p.records)
    assert_plan_equal(r, p, prefix=True)
    h.close()


def test_degenerate(g10):
    w = traces.encoder12()
    h, v, args = run_both(g10, w)
    r = h.plan(**dict(args, gpu_cap=v.peak))                    # nothing to do
    assert (r.status, r.n_iterations, len(r.records), r.n_cand_evals) == (g10.FITS, 0, 0, 0)
    r = h.plan(**dict(args, host_cap=0))                        # no host memory
    assert_plan_equal(r, v.plan(**dict(args, host_cap=0)))
    assert (r.records["dest"] == 0).all() and r.n_dropped > 0
    h.close()
    w1 = traces.mlp_tiny()                                      # no transfer fits any period
    h, v, args = run_both(g10, w1)
    r = h.plan(**dict(args, bw_out=(1, 1), bw_in=(1, 1)))
    assert (r.status, r.n_iterations, len(r.records), r.n_cand_evals) == (g10.RESIDUAL, 1, 0, v.C)
    h.close()


def test_edge_shapes(g10):
    # one kernel, one tensor; no pairs at all; a tensor used by every kernel
    one = Trace("one", np.array([5], np.uint64), np.array([7], np.uint64), np.array([1], np.uint8),
                np.array([0], np.uint32), np.array([0], np.uint32))
    nop = Trace("nopairs", np.array([5, 6], np.uint64), np.array([7, 8], np.uint64), np.zeros(2, np.uint8),
                np.zeros(0, np.uint32), np.zeros(0, np.uint32))
    K = 600
    every = Trace("every", np.full(K, 9, np.uint64), np.array([100, 200], np.uint64), np.array([0, 1], np.uint8),
                  np.concatenate([np.arange(K), [3, 599]]).astype(np.uint32),
                  np.concatenate([np.zeros(K), [1, 1]]).astype(np.uint32))
    for tr in (one, nop, every):
        v = O.Vitality(tr, O.DIRECT)
        h = g10.g10_vitality(g10.DeviceTrace(tr))
        assert_vitality_equal(h, v)
        args = dict(gpu_cap=max(v.peak // 2, 1), host_cap=10 ** 6, bw_out=(50, 100), bw_in=(50, 100))
        assert_plan_equal(h.plan(**args), v.plan(**args))
        h.close()


def test_errors(g10):
    w = traces.random_small(1)
    tr = w.trace

    def code(**ch):
        t2 = Trace(tr.name, tr.dur_ns.copy(), tr.size_bytes.copy(), tr.is_global.copy(),
                   tr.use_kernel.copy(), tr.use_tensor.copy())
        for k, (i, val) in ch.items():
            getattr(t2, k)[i] = val
        try:
            g10.g10_vitality(g10.DeviceTrace(t2)).close()
            gpu = 0
        except g10.G10Error as e:
            gpu = e.code
        try:
            O.Vitality(t2)
            cpu = 0
        except O.OracleError as e:
            cpu = e.code
        assert gpu == cpu
        return gpu

    assert code() == 0
    assert code(dur_ns=(0, 0)) == g10.EINVAL
    assert code(size_bytes=(1, 0)) == g10.EINVAL
    assert code(use_kernel=(0, tr.K)) == g10.EINVAL
    assert code(use_tensor=(0, tr.N)) == g10.EINVAL
    assert code(size_bytes=(0, 2 ** 63)) == g10.EOVERFLOW
    assert code(dur_ns=(0, 2 ** 62)) == g10.EOVERFLOW
    h = g10.g10_vitality(g10.DeviceTrace(tr))
    with pytest.raises(g10.G10Error) as e:
        h.plan(gpu_cap=1, host_cap=1, bw_out=(0, 1), bw_in=(1, 1))
    assert e.value.code == g10.EINVAL
    with pytest.raises(g10.G10Error) as e:
        h.prefetch()                                  # no plan on the handle yet
    assert e.value.code == g10.EINVAL
    h.close()


def test_stress_full_size_prefix_and_properties(g10):
    """Config 5 at full size, in the launch configuration the benchmark times.
    The oracle computes the first ranking passes outright; the rest of the plan
    is judged by the property checker, with the arg-max property verified on a
    sample of passes spread over the whole run."""
    w = traces.config(5)
    tr = w.trace
    h, v, args = run_both(g10, w)
    r = h.plan(**args)
    n = 150
    p = v.plan(max_iters=n, **args)
    assert_plan_equal(r, p, prefix=True)
    assert (r.null_iters[r.null_iters < n] == p.null_iters).all()
    m = plancheck.Machine(args["gpu_cap"], args["host_cap"], args["bw_out"], args["bw_in"])
    passes = r.n_iterations
    sample = sorted(set(np.linspace(0, passes - 1, 40).astype(int).tolist()))
    plancheck.check_plan(tr, m, r.records, r.null_iters, r.null_cands, r.status,
                         pressure_after=r.pressure_after, n_iterations=r.n_iterations,
                         n_cand_evals=r.n_cand_evals, greedy=sample)
    # determinism: a second run returns the same bytes
    r2 = h.plan(**args)
    assert r2.records.tobytes() == r.records.tobytes()
    # smart prefetching on the full plan, against the independent replay of the definitions
    f = h.prefetch()
    a2, b2 = prefetchcheck.doubled_windows(tr.K, r.records)
    o, g, pr = prefetchcheck.replay_numpy(tr.K, v.start, args["gpu_cap"], r.records, a2, b2, r.pressure_after)
    assert (f.order == o).all() and (f.gained == g).all() and (f.pressure == pr).all()
    assert (f.n_moved, f.slots_gained, f.peak) == (int((g > 0).sum()), int(g.astype(np.uint64).sum()), int(pr.max()))
    # the sweeps the benchmark times: the same trace planned in batches (capacities that share their candidate
    # windows; flash bandwidths that do not).  The plan at the default point must be the one above, the others
    # the ones made alone, and one of each kind is judged by the property checker
    caps = [int(v.peak * f) for f in (0.20, 0.25, 0.35)] + [args["gpu_cap"]]
    sweep = [dict(args, gpu_cap=c) for c in caps]
    for f in (6400, 32000):
        sweep.append(dict(args, bw_out=(f, args["bw_out"][1]), bw_in=(f, args["bw_in"][1])))
    rs = h.plan_batch(sweep)
    assert rs[3].records.tobytes() == r.records.tobytes() and (rs[3].pressure_after == r.pressure_after).all()
    for d, x in zip(sweep, rs):
        alone = h.plan(**d)
        assert (x.status, x.n_iterations, x.n_cand_evals) == (alone.status, alone.n_iterations, alone.n_cand_evals)
        assert x.records.tobytes() == alone.records.tobytes() and (x.pressure_after == alone.pressure_after).all()
    for i in (0, 5):
        d, x = sweep[i], rs[i]
        mi = plancheck.Machine(d["gpu_cap"], d["host_cap"], d["bw_out"], d["bw_in"])
        si = sorted(set(np.linspace(0, x.n_iterations - 1, 12).astype(int).tolist()))
        plancheck.check_plan(tr, mi, x.records, x.null_iters, x.null_cands, x.status, pressure_after=x.pressure_after,
                             n_iterations=x.n_iterations, n_cand_evals=x.n_cand_evals, greedy=si)
    h.close()
    # the oracle's complete plan, stored as digests (tests/golden/make_config5_digest.py)
    import hashlib
    import os
    import sys
    sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden"))
    import make_config5_digest as gd
    gold = dict(line.split() for line in open(os.path.join(gd.HERE, "config5_plan_digest.txt")) if not line.startswith("#"))
    if gd.trace_digest(tr) != gold["trace_sha256"]:
        pytest.skip("this machine's numpy generates a different stress trace than the stored digests were made from; "
                    "prefix and property checks above passed")
    assert gd.records_digest(r.records) == gold["records_sha256"]
    assert hashlib.sha256(r.pressure_after.astype("<u8").tobytes()).hexdigest() == gold["pressure_after_sha256"]
    assert (r.status, r.n_iterations, r.n_migrations, r.n_dropped, r.n_cand_evals) == \
        tuple(int(gold[k]) for k in ("status", "passes", "migrations", "dropped", "cand_evals"))


def test_released_memory_is_reused_and_trim_returns_it(g10):
    """What g10_plan_free releases stays in the library's cache and serves the next handle (same
    results from memory that holds the last call's contents); g10_trim hands it back to the driver."""
    import torch
    w = traces.config(3)
    dt = g10.DeviceTrace(w.trace)
    v = O.Vitality(w.trace, O.PREFIX)
    cap, hcap = traces.resolve_caps(w, v.peak)
    p = v.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus)
    g10.g10_trim()
    torch.cuda.synchronize()
    free_start = torch.cuda.mem_get_info()[0]
    for _ in range(3):                              # the second and third run in released blocks
        h = g10.g10_vitality(dt)
        assert_vitality_equal(h, v)
        r = h.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus)
        assert_plan_equal(r, p)
        in_use = torch.cuda.mem_get_info()[0]
        h.close()
    kept = torch.cuda.mem_get_info()[0]
    assert kept <= in_use + (1 << 20)               # nothing went back to the driver with the handle
    # a different, smaller trace afterwards: blocks that do not fit are not handed out
    w2 = traces.config(1)
    h2, v2, args2 = run_both(g10, w2)
    assert_plan_equal(h2.plan(**args2), v2.plan(args2["gpu_cap"], args2["host_cap"], w2.bw_out_Bpus, w2.bw_in_Bpus))
    h2.close()
    g10.g10_trim()
    assert torch.cuda.mem_get_info()[0] >= free_start - (8 << 20)
    assert torch.cuda.mem_get_info()[0] > kept
