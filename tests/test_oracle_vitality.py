"""Pins for the oracle's vitality analysis (Sections 3 and 4.2)."""
import numpy as np
import pytest

import brute
from goldenio import Golden
from oracle import oracle as O
from paper_2310_09443_amd import traces
from paper_2310_09443_amd.traces import Trace


def _uses(v, t):
    return v.use_k[int(v.use_off[t]):int(v.use_off[t + 1])].tolist()


@pytest.mark.parametrize("mode", [O.DIRECT, O.PREFIX])
def test_fig6_listing(mode):
    g = Golden("fig6_listing.txt")
    v = O.Vitality(g.trace, mode)
    for row in g.expect["uses"]:
        assert _uses(v, row[0]) == row[1:]
    got = list(zip(v.per_tensor.tolist(), v.per_L.tolist(), v.per_R.tolist()))
    assert got == [tuple(r) for r in g.expect["period"]]
    assert v.pressure.tolist() == g.expect["pressure"][0]
    assert v.peak == g.expect["peak"][0][0]
    # with cross-iteration periods switched off the filter has no period at all
    assert O.Vitality(g.trace, mode, no_wrap=True).C == 0


def residual_block():
    """Residual basic block in the spirit of Figure 3: forward conv1, conv2,
    add; backward in reverse.  A0 feeds conv1 and the skip connection, W1 is
    used in forward, backward-data and by the optimizer."""
    names = ["A0", "W1", "A1", "W2", "A2", "A3", "dA3", "dA2", "dW2", "dA1", "dW1", "dA0"]
    ix = {n: i for i, n in enumerate(names)}
    kernels = [["A0", "W1", "A1"],            # 0 conv1(F)
               ["A1", "W2", "A2"],            # 1 conv2(F)
               ["A2", "A0", "A3"],            # 2 add(F)
               ["A3", "dA3"],                 # 3 loss
               ["dA3", "dA2", "dA0"],         # 4 add(B)
               ["dA2", "W2", "dA1"],          # 5 conv2(B) data
               ["dA2", "A1", "dW2"],          # 6 conv2(B) weight
               ["dA1", "W1", "dA0"],          # 7 conv1(B) data
               ["dA1", "A0", "dW1"],          # 8 conv1(B) weight
               ["W1", "dW1"],                 # 9 update W1
               ["W2", "dW2"]]                 # 10 update W2
    uk = [k for k, us in enumerate(kernels) for _ in us]
    ut = [ix[u] for us in kernels for u in us]
    glob = [1 if n.startswith("W") else 0 for n in names]
    tr = Trace("resblock", np.full(len(kernels), 1000, np.uint64), np.full(len(names), 4096, np.uint64),
               np.array(glob, np.uint8), np.array(uk, np.uint32), np.array(ut, np.uint32))
    return tr, ix


def test_residual_block_multiple_periods_and_wrap():
    tr, ix = residual_block()
    v = O.Vitality(tr, O.DIRECT)
    per = {}
    for t, L, R in zip(v.per_tensor, v.per_L, v.per_R):
        per.setdefault(int(t), []).append((int(L), int(R)))
    # A0: used by kernels 0, 2, 8 -> two periods (the caption's "A0" example)
    assert per[ix["A0"]] == [(0, 2), (2, 8)]
    # W1: used by 0, 7, 9 -> periods 0..7 and (no gap 7..9 of 2? 9-7 = 2 -> one slot) and the wrap
    assert per[ix["W1"]] == [(0, 7), (7, 9), (9, 11)]
    # W2: 1, 5, 10 and wrap 10 -> 1+11
    assert per[ix["W2"]] == [(1, 5), (5, 10), (10, 12)]
    # a gradient produced and consumed by adjacent kernels has none
    assert ix["dA3"] not in per


@pytest.mark.parametrize("seed", range(40))
def test_periods_and_pressure_against_activity_table(seed):
    w = traces.random_small(seed, K=6 + seed % 9, N=4 + seed % 7, max_uses=5)
    for no_wrap in (False, True):
        for mode in (O.DIRECT, O.PREFIX):
            v = O.Vitality(w.trace, mode, no_wrap=no_wrap)
            got = list(zip(v.per_tensor.tolist(), v.per_L.tolist(), v.per_R.tolist()))
            assert got == brute.periods_from_table(w.trace, no_wrap)
            assert v.pressure.tolist() == brute.pressure_from_table(w.trace)
            assert v.peak == max(brute.pressure_from_table(w.trace))


@pytest.mark.parametrize("seed", range(10))
def test_identities(seed):
    w = traces.stress(K=400, N=3000, seed=seed)
    tr = w.trace
    v = O.Vitality(tr, O.PREFIX)
    pairs = np.unique(tr.use_tensor.astype(np.int64) * tr.K + tr.use_kernel)
    assert v.n_uses == len(pairs)
    assert (np.diff(v.use_off.astype(np.int64)) == np.bincount(pairs // tr.K, minlength=tr.N)).all()
    m = np.diff(v.use_off.astype(np.int64))
    # lifetime of each used tensor = uses + unit gaps(0 slots) + interior slots of its periods
    interior = np.zeros(tr.N, np.int64)
    inner = v.per_R < tr.K
    np.add.at(interior, v.per_tensor[inner], (v.per_R[inner].astype(np.int64) - v.per_L[inner] - 1))
    used = m > 0
    life = v.death.astype(np.int64) - v.birth + 1
    assert (life[used] == (m + interior)[used]).all()
    # pressure is at least the bytes of the tensors the kernel itself touches
    active = np.zeros(tr.K, np.int64)
    np.add.at(active, pairs % tr.K, tr.size_bytes[pairs // tr.K].astype(np.int64))
    assert (v.pressure.astype(np.int64) >= active).all()
    # direct and prefix modes agree
    v0 = O.Vitality(tr, O.DIRECT)
    assert (v0.pressure == v.pressure).all() and v0.peak == v.peak


def test_mlp_closed_form():
    """Config 1: sizes are shape products, residency follows from the op list."""
    w = traces.mlp_tiny()
    v = O.Vitality(w.trace, O.DIRECT)
    act, wsz, bsz = 64 * 256 * 4, 256 * 256 * 4, 256 * 4
    assert act == 65536 and wsz == 262144
    glob = 4 * (wsz + bsz)
    # slot 0 (GEMM_1): globals + A0 + Z1
    assert v.pressure[0] == glob + 2 * act
    # last slot (SGD_4): globals + dW4 + db4 (dW_l, db_l live from their dW kernel to their SGD)
    assert v.pressure[23] == glob + wsz + bsz
    # slot 8 (dReLU_4): globals + A0..A3 + Z1..Z4 + dA4 + dZ4 (A4 is touched by ReLU_4 only: dead)
    assert v.pressure[8] == glob + (4 + 4 + 2) * act
    assert v.K == 24 and v.N == 34
    # weights W_l are used by GEMM_l, dX_l and SGD_l; biases by GEMM_l and SGD_l
    assert v.n_uses == 80


def test_intermediate_only_trace_is_empty_outside_lifetimes():
    w = traces.random_small(7, K=14, N=6, frac_global=0.0)
    v = O.Vitality(w.trace, O.DIRECT)
    used = np.diff(v.use_off.astype(np.int64)) > 0
    lo, hi = v.birth[used].min(), v.death[used].max()
    assert (v.pressure[:lo] == 0).all() and (v.pressure[hi + 1:] == 0).all()
    assert O.Vitality(w.trace, O.DIRECT, no_wrap=True).C == v.C


def test_rejects_invalid():
    w = traces.random_small(1)
    tr = w.trace
    for bad in ("dur", "size", "kernel", "tensor"):
        t2 = Trace(tr.name, tr.dur_ns.copy(), tr.size_bytes.copy(), tr.is_global.copy(),
                   tr.use_kernel.copy(), tr.use_tensor.copy())
        if bad == "dur":
            t2.dur_ns[0] = 0
        elif bad == "size":
            t2.size_bytes[0] = 0
        elif bad == "kernel":
            t2.use_kernel[0] = tr.K
        else:
            t2.use_tensor[0] = tr.N
        with pytest.raises(O.OracleError):
            O.Vitality(t2)
