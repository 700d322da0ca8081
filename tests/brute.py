"""Brute force for tiny traces, in plain Python loops.

Nothing here keeps incremental state: every pass of the eviction loop
recomputes the pressure of every slot from the tensors' residency and the
list of migrations committed so far, and re-derives every channel reservation
by replaying those migrations from an empty channel.  Sums are loops over
slots.  Usable only for a handful of kernels and tensors; it pins the oracle
(Sections 4.2-4.3, Algorithm 1) on random tiny inputs.
"""
from fractions import Fraction
from itertools import product

FLASH, HOST = 0, 1


def activity_table(trace):
    """state[t][k] in {'A' active, 'I' inactive (will be used again within the
    iteration), 'W' inactive global waiting for the next iteration, 'D' not
    alive}: Section 4.2 applied to every (tensor, kernel) pair directly."""
    K, N = trace.K, trace.N
    pairs = set(zip(trace.use_tensor.tolist(), trace.use_kernel.tolist()))
    table = []
    for t in range(N):
        used = [k for k in range(K) if (t, k) in pairs]
        row = []
        for k in range(K):
            if k in used:
                row.append("A")
            elif not used:
                row.append("D")
            elif any(u < k for u in used) and any(u > k for u in used):
                row.append("I")
            elif trace.is_global[t]:
                row.append("W")
            else:
                row.append("D")
        table.append(row)
    return table


def periods_from_table(trace, no_wrap=False):
    """Maximal runs of inactive slots, as (tensor, L, R) in the planner's order."""
    K = trace.K
    out = []
    for t, row in enumerate(activity_table(trace)):
        k = 0
        runs = []
        while k < K:
            if row[k] == "I":
                j = k
                while row[j] == "I":
                    j += 1
                runs.append((t, k - 1, j))
                k = j
            else:
                k += 1
        out += runs
        if trace.is_global[t] and "A" in row and not no_wrap:
            last = max(k for k in range(K) if row[k] == "A")
            first = min(k for k in range(K) if row[k] == "A")
            if (K - 1 - last) + first >= 1:              # at least one waiting slot
                out.append((t, last, first + K))
    return out


def pressure_from_table(trace):
    """Bytes resident per slot: a used global tensor always, an intermediate
    tensor from its first to its last use."""
    table = activity_table(trace)
    out = []
    for k in range(trace.K):
        tot = 0
        for t in range(trace.N):
            if trace.is_global[t]:
                resident = "A" in table[t]
            else:
                resident = table[t][k] in "AI"
            if resident:
                tot += int(trace.size_bytes[t])
        out.append(tot)
    return out


class Brute:
    def __init__(self, trace, gpu_cap, host_cap, bw_out, bw_in, no_wrap=False, rank="benefit", area="band"):
        """rank="ratio": periods are ranked by benefit / (eviction + prefetch time) instead of the
        benefit alone; area="clipped": the benefit is the area between the pressure curve and the
        capacity line that goes away (Section 4.3's two alternatives)."""
        self.rank, self.area = rank, area
        self.tr = trace
        self.K = trace.K
        self.dur = [int(x) for x in trace.dur_ns]
        self.cap, self.host_cap = int(gpu_cap), int(host_cap)
        self.bw_out, self.bw_in = [int(x) for x in bw_out], [int(x) for x in bw_in]
        self.periods = periods_from_table(trace, no_wrap)
        self.base_pressure = pressure_from_table(trace)
        self.T = sum(self.dur)

    def t0(self, j):                       # start time of doubled slot j
        return sum(self.dur[i % self.K] for i in range(j))

    def window(self, c, d):
        """(a, b, tau_o, tau_i) or None: first slot starting at/after the end
        of the eviction, last slot ending at/before the start of the prefetch."""
        t, L, R = self.periods[c]
        s = int(self.tr.size_bytes[t])
        tau_o = -(-s * 1000 // self.bw_out[d])
        tau_i = -(-s * 1000 // self.bw_in[d])
        evict_end = self.t0(L + 1) + tau_o
        fetch_start = self.t0(R) - tau_i
        a = next((j for j in range(L + 1, R + 1) if self.t0(j) >= evict_end), None)
        b = next((j for j in range(R - 1, L - 1, -1) if self.t0(j + 1) <= fetch_start), None)
        if a is None or b is None or a > b:
            return None
        return a, b, tau_o, tau_i

    # -- state recomputed from the committed list ---------------------------
    def state(self, committed):
        K = self.K
        pressure = list(self.base_pressure)
        busy = [[[0] * K for _ in range(2)] for _ in range(2)]
        host = [0] * K
        for c, d in committed:
            t, L, R = self.periods[c]
            s = int(self.tr.size_bytes[t])
            a, b, tau_o, tau_i = self.window(c, d)
            for j in range(a, b + 1):
                pressure[j % K] -= s
            rem = tau_o
            for j in range(L + 1, a):
                x = min(rem, self.dur[j % K] - busy[d][0][j % K])
                busy[d][0][j % K] += x
                rem -= x
            assert rem == 0
            rem = tau_i
            for j in range(R - 1, b, -1):
                x = min(rem, self.dur[j % K] - busy[d][1][j % K])
                busy[d][1][j % K] += x
                rem -= x
            assert rem == 0
            if d == HOST:
                for j in range(L + 1, R):
                    host[j % K] += s
        return pressure, busy, host

    def score(self, c, pressure, busy):
        t, L, R = self.periods[c]
        s = int(self.tr.size_bytes[t])
        K = self.K
        for d in (FLASH, HOST):
            w = self.window(c, d)
            if w is None:
                continue
            a, b, tau_o, tau_i = w
            free_o = sum(self.dur[j % K] - busy[d][0][j % K] for j in range(L + 1, a))
            free_i = sum(self.dur[j % K] - busy[d][1][j % K] for j in range(b + 1, R))
            if free_o < tau_o or free_i < tau_i:
                continue
            if self.area == "clipped":
                B = 0
                for j in range(a, b + 1):
                    before = max(pressure[j % K] - self.cap, 0)           # over the line with the tensor
                    after = max(pressure[j % K] - s - self.cap, 0)        # and without it
                    B += self.dur[j % K] * (before - after)
                return d, B, tau_o + tau_i
            over = sum(self.dur[j % K] for j in range(a, b + 1) if pressure[j % K] > self.cap)
            return d, s * over, tau_o + tau_i
        return None, 0, 1

    def run(self):
        """Returns (committed [(cand, dest, benefit)], dropped [(pass, cand)], status, passes)."""
        live = set(range(len(self.periods)))
        committed, dropped, out = [], [], []
        passes = 0
        while True:
            pressure, busy, host = self.state(committed)
            if max(pressure) <= self.cap:
                return out, dropped, 0, passes
            passes += 1
            best = (0, None, None)
            best_key = Fraction(0)
            for c in sorted(live):
                d, B, cost = self.score(c, pressure, busy)
                key = Fraction(B, cost) if self.rank == "ratio" else Fraction(B)
                if key > best_key:
                    best, best_key = (B, c, d), key
            B, c, d = best
            if B == 0:
                return out, dropped, 1, passes
            live.discard(c)
            t, L, R = self.periods[c]
            s = int(self.tr.size_bytes[t])
            if d == HOST and max(host[j % self.K] for j in range(L + 1, R)) + s > self.host_cap:
                dropped.append((passes - 1, c))
                continue
            committed.append((c, d))
            out.append((c, d, B))

    # -- exhaustive bound ------------------------------------------------------
    def best_static_overtime(self):
        """Minimum over ALL assignments period -> {stay, flash, host} that
        respect window validity and host capacity (channel contention ignored)
        of the total over-capacity time.  A greedy plan is one such assignment,
        so its residual over-capacity time can not be below this."""
        C = len(self.periods)
        K = self.K
        win = [[self.window(c, d) for d in (FLASH, HOST)] for c in range(C)]
        best = None
        for assign in product((None, FLASH, HOST), repeat=C):
            if any(d is not None and win[c][d] is None for c, d in enumerate(assign)):
                continue
            pressure = list(self.base_pressure)
            host = [0] * K
            for c, d in enumerate(assign):
                if d is None:
                    continue
                t, L, R = self.periods[c]
                s = int(self.tr.size_bytes[t])
                a, b, _, _ = win[c][d]
                for j in range(a, b + 1):
                    pressure[j % K] -= s
                if d == HOST:
                    for j in range(L + 1, R):
                        host[j % K] += s
            if max(host) > self.host_cap:
                continue
            ot = sum(self.dur[k] for k in range(K) if pressure[k] > self.cap)
            best = ot if best is None else min(best, ot)
        return best
