"""Pins for the two alternative readings of Section 4.3 in the oracle: ranking by
benefit / cost, and the benefit as the area removed between the pressure curve
and the capacity line.  Hand-worked examples, brute force on tiny traces, closed
forms, special cases that reduce to the default reading, the independent checker."""
import numpy as np
import pytest

import brute
import plancheck
from goldenio import Golden
from oracle import oracle as O
from paper_2310_09443_amd import traces

RANKS = {O.BY_BENEFIT: "benefit", O.BY_RATIO: "ratio"}
AREAS = {O.BAND: "band", O.CLIPPED: "clipped"}
VARIANTS = [(O.BY_RATIO, O.BAND), (O.BY_BENEFIT, O.CLIPPED), (O.BY_RATIO, O.CLIPPED)]


def _check(trace, args, p, rank, area, greedy="all", no_wrap=False, complete=True):
    m = plancheck.Machine(args["gpu_cap"], args["host_cap"], args["bw_out"], args["bw_in"],
                          rank=RANKS[rank], area=AREAS[area])
    return plancheck.check_plan(trace, m, p.records, p.null_iters, p.null_cands, p.status,
                                pressure_after=p.pressure_after if complete else None,
                                n_iterations=p.n_iterations if complete else None,
                                n_cand_evals=p.n_cand_evals if complete else None,
                                greedy=greedy, no_wrap=no_wrap, complete=complete)


def _tuples(records):
    return [(int(r["cand"]), int(r["dest"]), int(r["benefit_lo"]) + (int(r["benefit_hi"]) << 64)) for r in records]


FIELDS = ["cand", "tensor", "evict_after", "absent_first", "absent_last", "next_use", "dest",
          "wraps", "size", "t_out", "t_in"]


def _rows(records):
    return [[int(r[f]) for f in FIELDS] + [int(r["benefit_lo"]) + (int(r["benefit_hi"]) << 64)] for r in records]


# ------------------------------------------------------------------ worked examples
@pytest.mark.parametrize("name", ["hand_plan_clipped.txt", "hand_plan_ratio.txt"])
@pytest.mark.parametrize("mode", [O.DIRECT, O.PREFIX])
def test_hand_worked_variants(name, mode):
    g = Golden(name)
    v = O.Vitality(g.trace, mode)
    assert list(zip(v.per_tensor.tolist(), v.per_L.tolist(), v.per_R.tolist())) == [tuple(r) for r in g.expect["period"]]
    va = g.variant_args()
    assert va != dict(rank=0, area=0)
    p = v.plan(**g.plan_args(), **va)
    e = g.expect
    assert (p.status, p.n_iterations, p.n_null, p.n_cand_evals) == \
        (e["status"][0][0], e["iterations"][0][0], e["nulls"][0][0], e["evals"][0][0])
    assert _rows(p.records) == e["record"]
    assert p.pressure_after.tolist() == e["pressure_after"][0]
    for row in e["busy"]:
        assert p.busy_after[row[0]][row[1]].tolist() == row[2:]
    assert p.host_after.tolist() == e["host_used"][0]
    _check(g.trace, g.plan_args(), p, va["rank"], va["area"])
    # the default reading decides differently on the same input
    d = v.plan(**g.plan_args())
    assert _rows(d.records)[0] != e["record"][0]
    if "default_record" in e:
        assert _rows(d.records) == e["default_record"]


# ------------------------------------------------------------------ brute force
@pytest.mark.parametrize("seed", range(40))
@pytest.mark.parametrize("rank,area", VARIANTS)
def test_tiny_traces_against_brute_force(seed, rank, area):
    w = traces.random_small(5000 + seed, K=8 + seed % 7, N=5 + seed % 4, max_uses=4)
    tr = w.trace
    no_wrap = seed % 5 == 0
    v = O.Vitality(tr, O.DIRECT, no_wrap=no_wrap)
    cap, hcap = traces.resolve_caps(w, v.peak)
    if seed % 3 == 0:                      # close under the peak: most excesses are smaller than the tensors
        cap = int(v.peak * 0.9)
    args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    bf = brute.Brute(tr, no_wrap=no_wrap, rank=RANKS[rank], area=AREAS[area], **args)
    committed, dropped, status, passes = bf.run()
    for mode in (O.DIRECT, O.PREFIX):
        p = v.plan(mode=mode, rank=rank, area=area, **args)
        assert _tuples(p.records) == committed
        assert list(zip(p.null_iters.tolist(), p.null_cands.tolist())) == dropped
        assert (p.status, p.n_iterations) == (status, passes)
        _check(tr, args, p, rank, area, no_wrap=no_wrap)


def test_variants_do_decide_differently_somewhere():
    """Over the tiny random traces every variant must differ from the default at least once:
    a switch that is silently ignored would pass the equalities above only if brute ignored it too."""
    differs = {v: 0 for v in VARIANTS}
    for seed in range(40):
        w = traces.random_small(5000 + seed, K=8 + seed % 7, N=5 + seed % 4, max_uses=4)
        v = O.Vitality(w.trace, O.PREFIX)
        args = dict(gpu_cap=int(v.peak * 0.9), host_cap=traces.resolve_caps(w, v.peak)[1],
                    bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
        base = v.plan(**args).records.tobytes()
        for rank, area in VARIANTS:
            differs[(rank, area)] += v.plan(rank=rank, area=area, **args).records.tobytes() != base
    assert all(n > 0 for n in differs.values()), differs


# ------------------------------------------------------------------ special cases that reduce to the default
@pytest.mark.parametrize("cfg", [1, 2])
def test_clipped_equals_band_when_capacity_is_zero(cfg):
    """With no capacity at all every slot of a tensor's window is over by at least the tensor
    itself (it is resident there), so min(size, excess) = size in every slot: same plan."""
    w = traces.config(cfg)
    v = O.Vitality(w.trace, O.PREFIX)
    args = dict(gpu_cap=0, host_cap=v.peak // 4, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    for rank in (O.BY_BENEFIT, O.BY_RATIO):
        a = v.plan(rank=rank, area=O.BAND, **args)
        b = v.plan(rank=rank, area=O.CLIPPED, **args)
        assert len(a.records) > 0 and a.records.tobytes() == b.records.tobytes()
        assert (a.status, a.n_iterations, a.n_null) == (b.status, b.n_iterations, b.n_null)


def test_clipped_never_exceeds_band_and_meets_it_far_above_capacity():
    w = traces.encoder12()
    v = O.Vitality(w.trace, O.PREFIX)
    cap, hcap = traces.resolve_caps(w, v.peak)
    args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    p = v.plan(area=O.CLIPPED, **args)
    m = plancheck.Machine(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus, area="clipped")
    mb = plancheck.Machine(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus)
    rp, rb = plancheck.Replay(plancheck.Problem(w.trace), m), plancheck.Replay(plancheck.Problem(w.trace), mb)
    equal = 0
    for r in p.records:
        c, d = int(r["cand"]), int(r["dest"])
        clipped, band = rp.benefit(c, d), rb.benefit(c, d)
        assert 0 < clipped <= band
        ab = rp._slots(int(rp.a[d][c]), int(rp.b[d][c]))
        ex = rp.pressure[ab] - cap
        if (ex[ex > 0] >= int(r["size"])).all():
            assert clipped == band
            equal += 1
        else:
            assert clipped < band
        rp.commit(c, d); rb.commit(c, d)
    assert 0 < equal < len(p.records)


def test_ratio_is_the_over_capacity_time_when_times_are_exact():
    """Equal bandwidth both ways and sizes that divide evenly: cost = 2 * size * 1000 / bw, so
    benefit / cost = over-capacity time of the window * bw / 2000 whatever the size: the first
    pick on free channels is the period with the longest over-capacity time in its flash window."""
    w = traces.random_small(77, K=40, N=30, max_uses=3)
    tr = w.trace
    v = O.Vitality(tr, O.DIRECT)
    bw = 1000                                        # sizes are multiples of 1000 B: exact microseconds
    args = dict(gpu_cap=int(v.peak * 0.5), host_cap=0, bw_out=(bw, bw), bw_in=(bw, bw))
    p = v.plan(rank=O.BY_RATIO, **args)
    valid, a, b, to, ti = v.windows(0, **args)
    assert valid.any() and ((to == ti) | ~valid.astype(bool)).all()
    over = v.pressure > args["gpu_cap"]
    ot = [int(sum(int(tr.dur_ns[j % tr.K]) for j in range(int(a[c]), int(b[c]) + 1) if over[j % tr.K])) if valid[c] else 0
          for c in range(v.C)]
    assert int(p.records["cand"][0]) == int(np.argmax(ot)) and max(ot) > 0
    first = p.records[0]
    assert int(first["dest"]) == 0 and int(first["benefit_lo"]) == int(first["size"]) * max(ot)


# ------------------------------------------------------------------ invariants at scale
@pytest.mark.parametrize("cfg", [1, 2, 3])
@pytest.mark.parametrize("rank,area", VARIANTS)
def test_configs_invariants_and_mode_equality(cfg, rank, area):
    w = traces.config(cfg)
    v = O.Vitality(w.trace, O.PREFIX)
    cap, hcap = traces.resolve_caps(w, v.peak)
    args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    limit = 2 ** 64 - 1 if cfg <= 2 else 60
    p = v.plan(rank=rank, area=area, max_iters=limit, **args)
    if cfg <= 2:
        p0 = v.plan(mode=O.DIRECT, rank=rank, area=area, **args)
        assert p0.records.tobytes() == p.records.tobytes()
        assert (p0.status, p0.n_iterations, p0.n_null, p0.n_cand_evals) == (p.status, p.n_iterations, p.n_null, p.n_cand_evals)
    complete = cfg <= 2
    step = 1 if cfg == 1 else 17
    _check(w.trace, args, p, rank, area, greedy=range(0, p.n_iterations, step), complete=complete)
    assert len(p.records) > 0


def test_bad_variant_is_an_error():
    w = traces.mlp_tiny()
    v = O.Vitality(w.trace)
    with pytest.raises(O.OracleError):
        v.plan(gpu_cap=1, host_cap=1, bw_out=(1, 1), bw_in=(1, 1), rank=2)
    with pytest.raises(O.OracleError):
        v.plan(gpu_cap=1, host_cap=1, bw_out=(1, 1), bw_in=(1, 1), area=2)


# ------------------------------------------------------------------ the checker tells the readings apart
def test_checker_rejects_a_plan_of_the_other_reading():
    for name in ("hand_plan_clipped.txt", "hand_plan_ratio.txt"):
        g = Golden(name)
        v = O.Vitality(g.trace)
        va = g.variant_args()
        p = v.plan(**g.plan_args(), **va)
        d = v.plan(**g.plan_args())
        _check(g.trace, g.plan_args(), p, va["rank"], va["area"])
        with pytest.raises(plancheck.CheckError):
            _check(g.trace, g.plan_args(), d, va["rank"], va["area"])
        with pytest.raises(plancheck.CheckError):
            _check(g.trace, g.plan_args(), p, O.BY_BENEFIT, O.BAND)
