"""Property checker for eviction plans (numpy, independent of oracle/ and of
the GPU library; it never produces a plan, it only judges one).

Given a trace, the machine parameters and a plan (committed migrations in
commit order plus the candidates dropped for lack of host memory), it replays
the plan from the definitions of Sections 4.2-4.4 / Algorithm 1 and checks
properties that must hold for any correct run at any size:

  * every record's windows and transfer times are the ones its tensor, period
    and destination imply; the tensor is never absent at a kernel using it;
    eviction + prefetch fit inside the inactive period;
  * at the moment of its commit the chosen destination was the policy one
    (flash unless the flash channel could not carry it) and had channel room;
    channel reservations never exceed a slot's duration and add up to the
    committed transfer times; host memory never exceeds its capacity;
  * the recorded benefit is size x over-capacity time of the absent window in
    the state just before the commit (area="clipped": the area between the
    pressure curve and the capacity line that the eviction removes, per slot
    duration x min(size, pressure - capacity));
  * greedy consistency, on every pass or on a sample of passes: the chosen
    candidate is the highest-benefit live candidate (rank="ratio": the one with
    the highest benefit / (eviction + prefetch time)), lowest index on ties,
    and a dropped candidate was the best one, bound for host, with no room;
  * the final state matches the reported status (fits <=> no slot over
    capacity; otherwise no live candidate has a positive benefit) and the
    reported pressure timeline.
"""
from __future__ import annotations

import numpy as np

FLASH, HOST = 0, 1


class CheckError(AssertionError):
    pass


def _req(cond, msg):
    if not cond:
        raise CheckError(msg)


class Problem:
    """Trace-side facts, derived here from the pair list by numpy sorting."""

    def __init__(self, trace, no_wrap=False):
        K, N = trace.K, trace.N
        self.K, self.N = K, N
        self.dur = trace.dur_ns.astype(np.int64)
        self.size = trace.size_bytes.astype(np.int64)
        glob = trace.is_global.astype(bool)
        keys = np.unique(trace.use_tensor.astype(np.int64) * K + trace.use_kernel.astype(np.int64))
        t, k = keys // K, keys % K
        self.use_t, self.use_k = t, k
        self.start = np.concatenate([[0], np.cumsum(self.dur)]).astype(np.int64)
        self.T = int(self.start[K])
        self.start2 = np.concatenate([self.start[:K], self.start[:K] + self.T, [2 * self.T]])
        head = np.ones(len(t), bool)
        head[1:] = t[1:] != t[:-1]
        tail = np.ones(len(t), bool)
        tail[:-1] = t[1:] != t[:-1]
        inner = np.flatnonzero(~head & (np.concatenate([[0], k[1:] - k[:-1]]) >= 2))
        pt, pL, pR = t[inner], k[inner - 1], k[inner]
        first = np.full(N, -1, np.int64)
        last = np.full(N, -1, np.int64)
        first[t[head]] = k[head]
        last[t[tail]] = k[tail]
        self.first, self.last = first, last
        used = first >= 0
        wt = np.flatnonzero(used & glob & ((first + K - last) >= 2)) if not no_wrap else np.zeros(0, np.int64)
        allt = np.concatenate([pt, wt])
        allL = np.concatenate([pL, last[wt]])
        allR = np.concatenate([pR, first[wt] + K])
        isw = np.concatenate([np.zeros(len(pt), np.int64), np.ones(len(wt), np.int64)])
        order = np.lexsort((allL, isw, allt))
        self.per_t, self.per_L, self.per_R = allt[order], allL[order], allR[order]
        self.C = len(order)
        self.per_s = self.size[self.per_t]
        lo = np.where(glob, 0, first)
        hi = np.where(glob, K - 1, last)
        diff = np.zeros(K + 1, np.int64)
        np.add.at(diff, lo[used], self.size[used])
        np.add.at(diff, hi[used] + 1, -self.size[used])
        self.pressure0 = np.cumsum(diff[:K])
        self.peak = int(self.pressure0.max())


class Machine:
    def __init__(self, gpu_cap, host_cap, bw_out, bw_in, rank="benefit", area="band"):
        assert rank in ("benefit", "ratio") and area in ("band", "clipped")
        self.rank, self.area = rank, area
        self.gpu_cap, self.host_cap = int(gpu_cap), int(host_cap)
        self.bw_out = [int(x) for x in bw_out]
        self.bw_in = [int(x) for x in bw_in]


def _ceil_div(x, y):
    return (x + (y - 1)) // y


def _dot_exact(x, y):
    """Sum of x[i] * y[i] as a Python int, for non-negative int64 arrays below 2^60 with fewer
    than 2^22 elements: 20-bit limbs, so no partial sum leaves the int64 range."""
    x, y = np.asarray(x, np.int64), np.asarray(y, np.int64)
    assert len(x) < (1 << 22)
    mask = (1 << 20) - 1
    total = 0
    for i in range(3):
        xi = (x >> (20 * i)) & mask
        if not xi.any():
            continue
        for j in range(3):
            yj = (y >> (20 * j)) & mask
            total += int(np.dot(xi, yj)) << (20 * (i + j))
    return total


class Replay:
    def __init__(self, pb: Problem, m: Machine):
        self.pb, self.m = pb, m
        K = pb.K
        _req(int(pb.per_s.max(initial=0)) < 2 ** 52, "checker limited to sizes below 2^52")
        s = pb.per_s
        L, R = pb.per_L, pb.per_R
        self.tau_o, self.tau_i, self.a, self.b, self.valid = [], [], [], [], []
        for d in (FLASH, HOST):
            to = _ceil_div(s * 1000, m.bw_out[d])
            ti = _ceil_div(s * 1000, m.bw_in[d])
            t_r = pb.start2[L + 1]
            t_use = pb.start2[R]
            a = np.searchsorted(pb.start2, t_r + to, side="left")
            y = t_use - ti
            b = np.searchsorted(pb.start2, np.maximum(y, -1), side="right") - 2
            valid = (a <= R) & (y >= 0) & (b >= L) & (a <= b)
            self.tau_o.append(to); self.tau_i.append(ti)
            self.a.append(np.where(valid, a, 1)); self.b.append(np.where(valid, b, 0))
            self.valid.append(valid)
        self.live = np.ones(pb.C, bool)
        self.pressure = pb.pressure0.copy()
        self.busy = [[np.zeros(K, np.int64) for _ in range(2)] for _ in range(2)]
        self.host_used = np.zeros(K, np.int64)

    # ---- helpers on doubled-coordinate ranges -------------------------------
    def _slots(self, x, y):
        return np.arange(x, y + 1) % self.pb.K

    def _pref2(self, v):
        p = np.concatenate([[0], np.cumsum(v)])
        return np.concatenate([p, p[1:] + p[-1]])          # length 2K+1

    def over(self):
        return self.pressure > self.m.gpu_cap

    # ---- vectorised scoring of every candidate ------------------------------
    def score_all(self):
        pb = self.pb
        L, R = pb.per_L, pb.per_R
        OT = self._pref2(np.where(self.over(), pb.dur, 0))
        dest = np.full(pb.C, -1, np.int64)
        ot = np.zeros(pb.C, np.int64)
        for d in (HOST, FLASH):                            # flash written last: it has priority
            FO = self._pref2(pb.dur - self.busy[d][0])
            FI = self._pref2(pb.dur - self.busy[d][1])
            a, b = self.a[d], self.b[d]
            feas = self.valid[d] & (FO[a] - FO[L + 1] >= self.tau_o[d]) & (FI[R] - FI[b + 1] >= self.tau_i[d])
            dest = np.where(feas, d, dest)
            ot = np.where(feas, OT[b + 1] - OT[a], ot)
        dest = np.where(self.live, dest, -1)
        ot = np.where(dest >= 0, ot, 0)
        return dest, ot

    def best(self):
        """(cand, dest, exact benefit) of the argmax, ties to the lowest index.

        The band (size x over-capacity time) is computed for every candidate at once; it equals the
        benefit (area="band") or bounds it (area="clipped").  Candidates are then looked at in the
        order of that bound, each evaluated exactly from the definitions, until no candidate left
        could reach the best exact key found."""
        from fractions import Fraction
        dest, ot = self.score_all()
        s = self.pb.per_s
        bound = s.astype(np.float64) * ot.astype(np.float64)
        if bound.size == 0 or bound.max() <= 0:
            return -1, -1, 0
        if self.m.rank == "ratio":
            cost = np.ones(len(s), np.float64)
            for d in (FLASH, HOST):
                cost = np.where(dest == d, (self.tau_o[d] + self.tau_i[d]).astype(np.float64), cost)
            bound = bound / cost
        best = None                                            # (key, cand, benefit)
        for i in np.argsort(-bound, kind="stable"):
            i = int(i)
            if bound[i] <= 0:
                break
            if best is not None and bound[i] < float(best[0]) * (1.0 - 1e-9):
                break
            d = int(dest[i])
            B = self.benefit(i, d) if self.m.area == "clipped" else int(s[i]) * int(ot[i])
            key = Fraction(B, int(self.tau_o[d][i]) + int(self.tau_i[d][i])) if self.m.rank == "ratio" else Fraction(B)
            if best is None or key > best[0] or (key == best[0] and i < best[1]):
                best = (key, i, B)
        if best is None or best[2] == 0:
            return -1, -1, 0
        return best[1], int(dest[best[1]]), best[2]

    # ---- one candidate, straight from the definitions -----------------------
    def feasible(self, c, d):
        pb = self.pb
        if not self.valid[d][c]:
            return False
        L, R, a, b = int(pb.per_L[c]), int(pb.per_R[c]), int(self.a[d][c]), int(self.b[d][c])
        ew, pw = self._slots(L + 1, a - 1), self._slots(b + 1, R - 1)
        fo = int((pb.dur[ew] - self.busy[d][0][ew]).sum())
        fi = int((pb.dur[pw] - self.busy[d][1][pw]).sum())
        return fo >= int(self.tau_o[d][c]) and fi >= int(self.tau_i[d][c])

    def benefit(self, c, d):
        ab = self._slots(int(self.a[d][c]), int(self.b[d][c]))
        size = int(self.pb.per_s[c])
        if self.m.area == "clipped":
            excess = np.clip(self.pressure[ab] - self.m.gpu_cap, 0, size)
            return _dot_exact(self.pb.dur[ab], excess)
        return size * int(self.pb.dur[ab][self.over()[ab]].sum())

    def host_room(self, c):
        pb = self.pb
        sl = self._slots(int(pb.per_L[c]) + 1, int(pb.per_R[c]) - 1)
        return int(self.host_used[sl].max()) + int(pb.per_s[c]) <= self.m.host_cap

    def commit(self, c, d):
        pb = self.pb
        L, R, a, b = int(pb.per_L[c]), int(pb.per_R[c]), int(self.a[d][c]), int(self.b[d][c])
        s = int(pb.per_s[c])
        self.pressure[self._slots(a, b)] -= s
        ew = self._slots(L + 1, a - 1)
        free = pb.dur[ew] - self.busy[d][0][ew]
        before = np.cumsum(free) - free
        self.busy[d][0][ew] += np.clip(int(self.tau_o[d][c]) - before, 0, free)
        pw = self._slots(b + 1, R - 1)[::-1]
        free = pb.dur[pw] - self.busy[d][1][pw]
        before = np.cumsum(free) - free
        self.busy[d][1][pw] += np.clip(int(self.tau_i[d][c]) - before, 0, free)
        if d == HOST:
            self.host_used[self._slots(L + 1, R - 1)] += s
        self.live[c] = False


def check_plan(trace, machine: Machine, records, null_iters, null_cands, status,
               pressure_after=None, n_iterations=None, n_cand_evals=None,
               greedy="all", no_wrap=False, complete=True, problem=None):
    """Raises CheckError on the first violated property.

    greedy: "all", "none", or an iterable of pass indices at which the argmax
    property is verified (the final stop condition is always verified when
    `complete`).  complete=False: the plan is a prefix cut by an iteration limit.
    """
    pb = problem or Problem(trace, no_wrap)
    rp = Replay(pb, machine)
    K = pb.K
    nulls = {int(i): int(c) for i, c in zip(null_iters, null_cands)}
    n_pass = len(records) + len(nulls)
    sample = set(range(n_pass)) if greedy == "all" else (set() if greedy == "none" else set(int(x) for x in greedy))
    evals, ri = 0, 0
    for p in range(n_pass):
        _req(bool(rp.over().any()), f"pass {p}: ran although nothing was over capacity")
        evals += int(rp.live.sum())
        if p in sample:
            bc, bd, bB = rp.best()
        if p in nulls:
            c = nulls[p]
            _req(rp.live[c], f"pass {p}: dropped candidate {c} was not live")
            _req(not rp.feasible(c, FLASH) and rp.feasible(c, HOST), f"pass {p}: dropped {c} was not host-bound")
            _req(rp.benefit(c, HOST) > 0, f"pass {p}: dropped {c} had no benefit")
            _req(not rp.host_room(c), f"pass {p}: dropped {c} although host memory had room")
            if p in sample:
                _req(bc == c and bd == HOST, f"pass {p}: dropped {c} but the best candidate was {bc}")
            rp.live[c] = False
            continue
        r = records[ri]; ri += 1
        c, d = int(r["cand"]), int(r["dest"])
        _req(0 <= c < pb.C and d in (FLASH, HOST), f"record {ri - 1}: bad cand/dest")
        _req(rp.live[c], f"record {ri - 1}: candidate {c} committed twice or after a drop")
        L, R = int(pb.per_L[c]), int(pb.per_R[c])
        a, b = int(rp.a[d][c]), int(rp.b[d][c])
        _req(bool(rp.valid[d][c]) and L < a <= b < R, f"record {ri - 1}: window not valid")
        exp = dict(tensor=int(pb.per_t[c]), evict_after=L, absent_first=a % K, absent_last=b % K,
                   next_use=R % K, wraps=int(R >= K), size=int(pb.per_s[c]),
                   t_out=int(rp.tau_o[d][c]), t_in=int(rp.tau_i[d][c]))
        for f, v in exp.items():
            _req(int(r[f]) == v, f"record {ri - 1}: field {f} = {int(r[f])}, expected {v}")
        _req(exp["t_out"] + exp["t_in"] <= int(pb.start2[R] - pb.start2[L + 1]),
             f"record {ri - 1}: transfers longer than the inactive period")
        _req(rp.feasible(c, d), f"record {ri - 1}: channel had no room")
        if d == HOST:
            _req(not rp.feasible(c, FLASH), f"record {ri - 1}: host chosen while flash could carry it")
            _req(rp.host_room(c), f"record {ri - 1}: host memory over capacity")
        B = rp.benefit(c, d)
        _req(B > 0, f"record {ri - 1}: zero benefit committed")
        _req(int(r["benefit_lo"]) + (int(r["benefit_hi"]) << 64) == B, f"record {ri - 1}: benefit mismatch")
        if p in sample:
            _req((bc, bd, bB) == (c, d, B), f"pass {p}: committed {(c, d, B)} but argmax is {(bc, bd, bB)}")
        rp.commit(c, d)
        for dd in range(2):
            for rr in range(2):
                _req(bool((rp.busy[dd][rr] <= pb.dur).all()), f"record {ri - 1}: channel over-reserved")
        _req(int(rp.host_used.max()) <= machine.host_cap, f"record {ri - 1}: host over capacity")
    # reservations add up to the committed transfer times
    for d in range(2):
        sel = records["dest"] == d
        _req(int(rp.busy[d][0].sum()) == int(records["t_out"][sel].astype(object).sum() if sel.any() else 0),
             "eviction reservations do not add up")
        _req(int(rp.busy[d][1].sum()) == int(records["t_in"][sel].astype(object).sum() if sel.any() else 0),
             "prefetch reservations do not add up")
    fits = not bool(rp.over().any())
    if complete:
        if fits:
            _req(status == 0, "pressure fits but status is not FITS")
            final_pass = 0
        else:
            _req(status == 1, "pressure over capacity but status is not RESIDUAL")
            bc, bd, bB = rp.best()
            _req(bB == 0, f"stopped although candidate {bc} still has benefit {bB}")
            evals += int(rp.live.sum())
            final_pass = 1
        if n_iterations is not None:
            _req(int(n_iterations) == n_pass + final_pass, "n_iterations mismatch")
        if n_cand_evals is not None:
            _req(int(n_cand_evals) == evals, "n_cand_evals mismatch")
    if pressure_after is not None:
        _req(bool((np.asarray(pressure_after).astype(np.int64) == rp.pressure).all()), "pressure_after mismatch")
    return rp
