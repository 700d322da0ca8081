"""Pins for the oracle's candidate windows and eviction loop (Sections 4.2-4.4,
Algorithm 1): hand-worked examples, closed forms, degenerate cases, brute
force on tiny traces, invariants through the independent plan checker."""
import numpy as np
import pytest

import brute
import plancheck
from goldenio import Golden
from oracle import oracle as O
from paper_2310_09443_amd import traces
from paper_2310_09443_amd.traces import Trace


def _plan(w, v, mode=None, **over):
    cap, hcap = traces.resolve_caps(w, v.peak)
    args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    args.update(over)
    return v.plan(mode=mode, **args), args


def _check(trace, args, p, greedy="all", no_wrap=False):
    m = plancheck.Machine(args["gpu_cap"], args["host_cap"], args["bw_out"], args["bw_in"])
    return plancheck.check_plan(trace, m, p.records, p.null_iters, p.null_cands, p.status,
                                pressure_after=p.pressure_after, n_iterations=p.n_iterations,
                                n_cand_evals=p.n_cand_evals, greedy=greedy, no_wrap=no_wrap)


# ------------------------------------------------------------------ worked examples
@pytest.mark.parametrize("name", ["hand_plan_a.txt", "hand_plan_b.txt"])
@pytest.mark.parametrize("mode", [O.DIRECT, O.PREFIX])
def test_hand_worked_plans(name, mode):
    g = Golden(name)
    v = O.Vitality(g.trace, mode)
    if "period" in g.expect:
        assert list(zip(v.per_tensor.tolist(), v.per_L.tolist(), v.per_R.tolist())) == \
            [tuple(r) for r in g.expect["period"]]
    p = v.plan(**g.plan_args())
    e = g.expect
    assert p.status == e["status"][0][0]
    assert p.n_iterations == e["iterations"][0][0]
    assert p.n_null == e["nulls"][0][0]
    assert p.n_cand_evals == e["evals"][0][0]
    fields = ["cand", "tensor", "evict_after", "absent_first", "absent_last", "next_use", "dest",
              "wraps", "size", "t_out", "t_in"]
    got = [[int(r[f]) for f in fields] + [int(r["benefit_lo"]) + (int(r["benefit_hi"]) << 64)]
           for r in p.records]
    assert got == e["record"]
    assert list(zip(p.null_iters.tolist(), p.null_cands.tolist())) == [tuple(x) for x in e.get("null_cand", [])]
    assert p.pressure_after.tolist() == e["pressure_after"][0]
    for row in e["busy"]:
        assert p.busy_after[row[0]][row[1]].tolist() == row[2:]
    assert p.host_after.tolist() == e["host_used"][0]
    _check(g.trace, g.plan_args(), p)


def test_transfer_time_example():
    """77073360 B (Figure 6's tensor22) at the 3.0 GB/s flash write bandwidth
    of Table 2 = 25691120 ns; at 3.2 GB/s read: 24085425 ns (size / bandwidth,
    Algorithm 1's t_s)."""
    tr = Trace("one", np.full(6, 10 ** 8, np.uint64), np.array([77073360], np.uint64),
               np.zeros(1, np.uint8), np.array([0, 5], np.uint32), np.zeros(2, np.uint32))
    v = O.Vitality(tr)
    valid, a, b, to, ti = v.windows(0, 1, 1, (3000, 15754), (3200, 15754))
    assert to[0] == 25691120 and ti[0] == 24085425
    assert valid[0] and a[0] == 2 and b[0] == 3          # one 100 ms slot each way


# ------------------------------------------------------------------ closed forms
@pytest.mark.parametrize("mode", [O.DIRECT, O.PREFIX])
@pytest.mark.parametrize("seed", range(6))
def test_windows_closed_form_equal_durations(mode, seed):
    """With every kernel lasting D: a = L + 1 + ceil(tau_o / D), b = R - 1 - ceil(tau_i / D)."""
    w = traces.stress(K=300, N=1500, seed=100 + seed)
    D = 7000 + seed
    tr = w.trace
    tr = Trace(tr.name, np.full(tr.K, D, np.uint64), tr.size_bytes // np.uint64(2000) + np.uint64(1),
               tr.is_global, tr.use_kernel, tr.use_tensor)
    v = O.Vitality(tr, mode)
    bw_out, bw_in = (37, 91), (41, 89)
    s = tr.size_bytes[v.per_tensor].astype(np.int64)
    L, R = v.per_L.astype(np.int64), v.per_R.astype(np.int64)
    for d in (0, 1):
        valid, a, b, to, ti = v.windows(d, 1, 1, bw_out, bw_in)
        eto = -(-s * 1000 // bw_out[d])
        eti = -(-s * 1000 // bw_in[d])
        assert (to.astype(np.int64) == eto).all() and (ti.astype(np.int64) == eti).all()
        ea = L + 1 + -(-eto // D)
        eb = R - 1 - -(-eti // D)
        ev = (ea <= R) & (eb >= L) & (ea <= eb)
        assert (valid.astype(bool) == ev).all()
        assert (a[ev] == ea[ev]).all() and (b[ev] == eb[ev]).all()
        assert ev.any() and (~ev).any()
        # a valid window leaves at least one slot for each transfer
        assert (ea[ev] >= L[ev] + 2).all() and (eb[ev] <= R[ev] - 2).all()


@pytest.mark.parametrize("seed", range(8))
def test_windows_binary_search_equals_linear_scan(seed):
    w = traces.stress(K=500, N=2500, seed=200 + seed, min_log2=14, max_log2=27)
    v = O.Vitality(w.trace, O.PREFIX)
    for d in (0, 1):
        r0 = v.windows(d, 1, 1, w.bw_out_Bpus, (5000, 20000), mode=O.DIRECT)
        r1 = v.windows(d, 1, 1, w.bw_out_Bpus, (5000, 20000), mode=O.PREFIX)
        assert (r0[0] == r1[0]).all()
        ok = r0[0].astype(bool)
        assert ok.any() and (~ok).any()
        for x, y in zip(r0[1:], r1[1:]):
            assert (x[ok] == y[ok]).all()


def test_single_candidate_closed_form():
    """One tensor used by the first and last kernel: benefit = size x duration
    of the slots it is absent from (all of them over capacity)."""
    K, D, s = 12, 5000, 8000
    tr = Trace("single", np.full(K, D, np.uint64), np.array([s], np.uint64), np.zeros(1, np.uint8),
               np.array([0, K - 1], np.uint32), np.zeros(2, np.uint32))
    v = O.Vitality(tr)
    p = v.plan(gpu_cap=s - 1, host_cap=0, bw_out=(1000, 1000), bw_in=(2000, 2000))
    # tau_o = 8000 ns -> 2 slots, tau_i = 4000 ns -> 1 slot: absent [3, 9]
    assert len(p.records) == 1
    r = p.records[0]
    assert (r["absent_first"], r["absent_last"], r["t_out"], r["t_in"]) == (3, 9, 8000, 4000)
    assert r["benefit_lo"] == s * 7 * D and r["dest"] == 0
    assert p.status == O.RESIDUAL                       # the using kernels still need it
    assert p.pressure_after.tolist() == [s] * 3 + [0] * 7 + [s] * 2


# ------------------------------------------------------------------ degenerate cases
def test_degenerate_cases():
    w = traces.encoder12()
    v = O.Vitality(w.trace, O.PREFIX)
    # capacity at or above the peak: nothing to do
    p = v.plan(gpu_cap=v.peak, host_cap=0, bw_out=(6000, 25000), bw_in=(6000, 25000))
    assert (p.status, p.n_iterations, len(p.records), p.n_cand_evals) == (O.FITS, 0, 0, 0)
    # bandwidth so low that no transfer fits any period
    # (config 1: the smallest tensor needs 1 ms at 1 B/us, the whole step lasts 0.7 ms)
    w1 = traces.mlp_tiny()
    v1 = O.Vitality(w1.trace, O.DIRECT)
    p = v1.plan(gpu_cap=v1.peak // 2, host_cap=2 ** 62, bw_out=(1, 1), bw_in=(1, 1))
    assert (p.status, p.n_iterations, len(p.records)) == (O.RESIDUAL, 1, 0)
    assert p.n_cand_evals == v1.C
    # no host memory: no host records, host-bound winners are dropped
    p, args = _plan(w, v, host_cap=0)
    assert (p.records["dest"] == 0).all() and p.n_null > 0
    _check(w.trace, args, p, greedy=range(0, p.n_iterations, 37))
    # flash at least as fast as host and ample: flash first means flash only
    p, args = _plan(w, v, bw_out=(10 ** 10, 10 ** 10), bw_in=(10 ** 10, 10 ** 10))
    assert len(p.records) > 0 and (p.records["dest"] == 0).all()


def test_no_wrap_without_globals_changes_nothing():
    w = traces.random_small(11, K=16, N=9, frac_global=0.0)
    a = O.Vitality(w.trace)
    b = O.Vitality(w.trace, no_wrap=True)
    pa, _ = _plan(w, a)
    pb, _ = _plan(w, b)
    assert pa.records.tobytes() == pb.records.tobytes()


def test_active_bytes_over_capacity_is_residual():
    """If a single kernel's own tensors exceed the capacity no plan can fit."""
    w = traces.resnet152()
    v = O.Vitality(w.trace, O.PREFIX)
    tr = w.trace
    pairs = np.unique(tr.use_tensor.astype(np.int64) * tr.K + tr.use_kernel)
    active = np.zeros(tr.K, np.int64)
    np.add.at(active, pairs % tr.K, tr.size_bytes[pairs // tr.K].astype(np.int64))
    cap = int(active.max()) - 1
    p = v.plan(gpu_cap=cap, host_cap=2 ** 62, bw_out=(10 ** 6, 10 ** 6), bw_in=(10 ** 6, 10 ** 6))
    assert p.status == O.RESIDUAL and p.peak_after > cap


# ------------------------------------------------------------------ brute force
@pytest.mark.parametrize("seed", range(60))
def test_tiny_traces_against_brute_force(seed):
    w = traces.random_small(1000 + seed, K=8 + seed % 7, N=5 + seed % 4, max_uses=4)
    tr = w.trace
    no_wrap = seed % 5 == 0
    v = O.Vitality(tr, O.DIRECT, no_wrap=no_wrap)
    cap, hcap = traces.resolve_caps(w, v.peak)
    args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    bf = brute.Brute(tr, no_wrap=no_wrap, **args)
    committed, dropped, status, passes = bf.run()
    for mode in (O.DIRECT, O.PREFIX):
        p = v.plan(mode=mode, **args)
        got = [(int(r["cand"]), int(r["dest"]), int(r["benefit_lo"]) + (int(r["benefit_hi"]) << 64))
               for r in p.records]
        assert got == committed
        assert list(zip(p.null_iters.tolist(), p.null_cands.tolist())) == dropped
        assert (p.status, p.n_iterations) == (status, passes)
        _check(tr, args, p, no_wrap=no_wrap)


@pytest.mark.parametrize("seed", range(25))
def test_greedy_within_exhaustive_bound(seed):
    """The plan is one assignment period -> {stay, flash, host}; no assignment
    that ignores channel contention can leave less over-capacity time than the
    best of all 3^C of them."""
    w = traces.random_small(3000 + seed, K=9, N=5, max_uses=3)
    v = O.Vitality(w.trace, O.DIRECT)
    if v.C == 0 or v.C > 8:
        pytest.skip("no candidates / too many to enumerate")
    cap, hcap = traces.resolve_caps(w, v.peak)
    args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
    p = v.plan(**args)
    bound = brute.Brute(w.trace, **args).best_static_overtime()
    assert bound <= p.overtime_after
    if p.status == O.FITS:
        assert bound == 0


# ------------------------------------------------------------------ invariants at scale
@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_configs_invariants_and_mode_equality(cfg):
    w = traces.config(cfg)
    v = O.Vitality(w.trace, O.PREFIX)
    p, args = _plan(w, v)
    if cfg <= 2:
        p0, _ = _plan(w, v, mode=O.DIRECT)
        assert p0.records.tobytes() == p.records.tobytes()
        assert (p0.status, p0.n_iterations, p0.n_null, p0.n_cand_evals) == \
            (p.status, p.n_iterations, p.n_null, p.n_cand_evals)
    step = 1 if cfg <= 2 else 23
    _check(w.trace, args, p, greedy=range(0, p.n_iterations, step))
    assert p.status == (O.FITS if p.peak_after <= args["gpu_cap"] else O.RESIDUAL)
    assert 0 < len(p.records)


def test_plan_that_fits():
    w = traces.encoder12()
    v = O.Vitality(w.trace, O.PREFIX)
    p, args = _plan(w, v, gpu_cap=int(v.peak * 0.93))
    assert p.status == O.FITS and len(p.records) > 0 and p.peak_after <= args["gpu_cap"]
    _check(w.trace, args, p)


def test_iteration_limit_returns_prefix():
    w = traces.resnet152()
    v = O.Vitality(w.trace, O.PREFIX)
    full, args = _plan(w, v)
    part = v.plan(max_iters=50, **args)
    assert part.status == O.TRUNCATED and part.n_iterations == 50
    n = len(part.records)
    assert part.records.tobytes() == full.records[:n].tobytes()


# ------------------------------------------------------------------ the checker itself rejects planted mistakes
def test_checker_rejects_planted_mistakes():
    g = Golden("hand_plan_a.txt")
    v = O.Vitality(g.trace)
    p = v.plan(**g.plan_args())
    m = plancheck.Machine(**{k: g.plan_args()[k] for k in ("gpu_cap", "host_cap", "bw_out", "bw_in")})

    def run(records, status=p.status, nulls=(p.null_iters, p.null_cands)):
        plancheck.check_plan(g.trace, m, records, nulls[0], nulls[1], status,
                             pressure_after=None, n_iterations=None)

    run(p.records)
    bad = p.records.copy(); bad["dest"][0] = 1                     # wrong destination
    with pytest.raises(plancheck.CheckError):
        run(bad)
    bad = p.records.copy(); bad["benefit_lo"][1] += 1              # wrong benefit
    with pytest.raises(plancheck.CheckError):
        run(bad)
    bad = p.records[[1, 0, 2]]                                      # wrong order
    with pytest.raises(plancheck.CheckError):
        run(bad)
    with pytest.raises(plancheck.CheckError):                       # stopped early
        run(p.records[:2], nulls=(p.null_iters[:0], p.null_cands[:0]))
    with pytest.raises(plancheck.CheckError):                       # wrong status
        run(p.records, status=0)
    bad = p.records.copy(); bad["absent_first"][2] += 1             # wrong window
    with pytest.raises(plancheck.CheckError):
        run(bad)
