"""Independent replay of smart prefetching (Section 4.4), written from the
definitions with plain Python integers and no shared code: visit the evicted
periods by latest safe prefetch time (ties in plan order); walk back from the
slot before the prefetch while the slot can hold the tensor, not past the first
absent slot; raise the pressure of the slots gained."""
import numpy as np


def replay(K, start, gpu_cap, records, a2, b2, pressure_after):
    """records: structured array of the plan; a2 / b2: absent windows in doubled
    slot coordinates.  Returns (order, gained, pressure)."""
    T = int(start[K])

    def start2(j):
        return int(start[j]) if j < K else int(start[j - K]) + T

    n = len(records)
    R2 = [int(r["next_use"]) + (K if int(r["wraps"]) else 0) for r in records]
    t_safe = [start2(R2[i]) - int(records[i]["t_in"]) for i in range(n)]
    order = sorted(range(n), key=lambda i: (t_safe[i], i))
    pr = [int(x) for x in pressure_after]
    gained = [0] * n
    for i in order:
        s, a, b = int(records[i]["size"]), int(a2[i]), int(b2[i])
        j = b
        while j >= a and pr[j % K] + s <= gpu_cap:
            pr[j % K] += s
            gained[i] += 1
            j -= 1
    return np.array(order, np.uint32), np.array(gained, np.uint32), np.array(pr, np.uint64)


def doubled_windows(K, records):
    """Absent windows of plan records in doubled coordinates, rebuilt from the
    record fields alone (the first absent slot lies after the period start)."""
    a2, b2 = [], []
    for r in records:
        L1 = int(r["evict_after"]) + 1
        a = int(r["absent_first"])
        if a < L1:
            a += K
        b = int(r["absent_last"])
        while b < a:
            b += K
        a2.append(a)
        b2.append(b)
    return np.array(a2, np.uint32), np.array(b2, np.uint32)


def replay_numpy(K, start, gpu_cap, records, a2, b2, pressure_after):
    """The same replay with the backward walk done on numpy slices (for long plans)."""
    T = int(start[K])
    st2 = np.concatenate([np.asarray(start[:K], np.uint64), np.asarray(start[:K], np.uint64) + np.uint64(T)])
    n = len(records)
    R2 = records["next_use"].astype(np.int64) + np.where(records["wraps"] > 0, K, 0)
    t_safe = st2[R2].astype(np.int64) - records["t_in"].astype(np.int64)
    order = np.lexsort((np.arange(n), t_safe))
    pr = np.asarray(pressure_after, np.uint64).copy()
    gained = np.zeros(n, np.uint32)
    cap = np.uint64(gpu_cap)
    for i in order:
        s, a, b = np.uint64(records["size"][i]), int(a2[i]), int(b2[i])
        if s > cap:
            continue
        idx = np.arange(a, b + 1) % K
        bad = np.flatnonzero(pr[idx] > cap - s)
        p = a + (int(bad[-1]) + 1 if len(bad) else 0)
        if p <= b:
            pr[idx[p - a:]] += s
            gained[i] = b + 1 - p
    return order.astype(np.uint32), gained, pr
