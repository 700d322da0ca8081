"""Independent statement of the plan replay (plain Python, no oracle/ code): the completion
times are written as one system of equations in (max, +) form,

    end[j]      = max(end[j - 1], done_fetch of every migration used by kernel j) + dur[j]
    done_evict  = max(end[issue point - 1], done of the transfer before it on its channel) + t_out
    done_fetch  = max(end[issue point - 1], done_evict, done of the transfer before it) + t_in

over two iterations laid end to end, and solved by relaxing all equations from zero until
nothing changes (the least fixed point; every right-hand side is monotone).  The oracle walks
the kernels once in order instead.  Only for small inputs."""


def solve(K, dur, records, b2, R2, gained=None):
    """records: list of dicts with evict_after, dest, t_out, t_in; b2 / R2: last absent slot and
    next use in doubled coordinates.  Returns (iter_ns, planned_ns, stall_ns, n_stalled, late)."""
    n = len(records)
    dur = [int(x) for x in dur]
    inst = []                                          # (copy, rec, evict point, fetch point, use)
    for c in range(2):
        for i, r in enumerate(records):
            issue = int(b2[i]) + 1 - (int(gained[i]) if gained is not None else 0)
            inst.append((c, i, int(r["evict_after"]) + 1 + c * K, issue + c * K, int(R2[i]) + c * K))
    # channel order: by issue point, then plan order
    def queue(kind):
        q = {}
        for x, (c, i, je, jf, ju) in enumerate(inst):
            j = je if kind == "out" else jf
            if j < 2 * K:
                q.setdefault(int(records[i]["dest"]), []).append((j, i, x))
        return {d: [x for _, _, x in sorted(v)] for d, v in q.items()}
    prev_out, prev_in = {}, {}
    for kind, prev in (("out", prev_out), ("in", prev_in)):
        for d, order in queue(kind).items():
            for a, b in zip(order, order[1:]):
                prev[b] = a
    end = [0] * (2 * K)
    E = [0] * len(inst)
    F = [0] * len(inst)
    uses = {}
    for x, (c, i, je, jf, ju) in enumerate(inst):
        if ju < 2 * K and jf < 2 * K:
            uses.setdefault(ju, []).append(x)
    changed = True
    while changed:
        changed = False
        for x, (c, i, je, jf, ju) in enumerate(inst):
            r = records[i]
            if je < 2 * K:
                t = max(end[je - 1] if je else 0, E[prev_out[x]] if x in prev_out else 0) + int(r["t_out"])
                if t != E[x]:
                    E[x], changed = t, True
            if jf < 2 * K:
                t = max(end[jf - 1] if jf else 0, E[x], F[prev_in[x]] if x in prev_in else 0) + int(r["t_in"])
                if t != F[x]:
                    F[x], changed = t, True
        for j in range(2 * K):
            t = max([end[j - 1] if j else 0] + [F[x] for x in uses.get(j, [])]) + dur[j % K]
            if t != end[j]:
                end[j], changed = t, True
    stall, n_stalled = 0, 0
    late = [0] * n
    for j in range(K, 2 * K):
        start = end[j] - dur[j % K]
        if start > end[j - 1]:
            stall += start - end[j - 1]
            n_stalled += 1
        for x in uses.get(j, []):
            late[inst[x][1]] = max(0, F[x] - end[j - 1])
    return end[2 * K - 1] - end[K - 1], sum(dur), stall, n_stalled, late
