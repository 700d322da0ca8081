"""Writes tests/golden/config5_plan_digest.txt: digests of the oracle's complete
plan for the stress workload (config 5), and tests/golden/config5_ratio_digest.txt:
digests of the first 4000 ranking passes of the oracle's plan with the benefit /
cost ranking key on the same workload (that key's complete plan has some 200 000
migrations); with `clipped`, tests/golden/config5_clipped_digest.txt: the first three passes with
the benefit read as the clipped area.  Calls only the trace generator and oracle/.  Takes about ten
minutes of one CPU core (`clipped`: seven more).

    python tests/golden/make_config5_digest.py [default|ratio|clipped]
"""
import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import oracle as O                      # noqa: E402
from paper_2310_09443_amd import traces             # noqa: E402

FIELDS = ["cand", "tensor", "evict_after", "absent_first", "absent_last", "next_use", "dest", "wraps",
          "size", "t_out", "t_in", "benefit_lo", "benefit_hi"]


def trace_digest(tr):
    h = hashlib.sha256()
    for a in (tr.dur_ns, tr.size_bytes, tr.is_global, tr.use_kernel, tr.use_tensor):
        h.update(np.ascontiguousarray(a).tobytes())
    return h.hexdigest()


def records_digest(rec):
    h = hashlib.sha256()
    for f in FIELDS:
        h.update(np.ascontiguousarray(rec[f]).astype("<u8").tobytes())
    return h.hexdigest()


RATIO_PASSES = 4000
CLIPPED_PASSES = 3           # (the oracle sums every live candidate's window slot by slot: two minutes per pass here)


def main():
    which = sys.argv[1] if len(sys.argv) > 1 else "both"
    w = traces.config(5)
    v = O.Vitality(w.trace, O.PREFIX)
    cap, hcap = traces.resolve_caps(w, v.peak)
    if which == "clipped":
        p = v.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus, max_iters=CLIPPED_PASSES, area=O.CLIPPED)
        with open(os.path.join(HERE, "config5_clipped_digest.txt"), "w") as f:
            f.write("# First ranking passes of the CPU oracle's plan for the stress workload (config 5) with the benefit read\n")
            f.write("# as the clipped area, as digests.  Written by tests/golden/make_config5_digest.py clipped, which calls\n")
            f.write("# only oracle/.\n")
            f.write(f"trace_sha256 {trace_digest(w.trace)}\n")
            f.write(f"records_sha256 {records_digest(p.records)}\n")
            f.write(f"status {p.status}\npasses {p.n_iterations}\nmigrations {p.n_migrations}\n"
                    f"dropped {p.n_null}\ncand_evals {p.n_cand_evals}\n")
        print("clipped written")
        return
    if which in ("ratio", "both"):
        p = v.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus, max_iters=RATIO_PASSES, rank=O.BY_RATIO)
        with open(os.path.join(HERE, "config5_ratio_digest.txt"), "w") as f:
            f.write("# First 4000 ranking passes of the CPU oracle's plan for the stress workload (config 5) with the\n")
            f.write("# benefit / cost ranking key, as digests.  Written by tests/golden/make_config5_digest.py, which\n")
            f.write("# calls only oracle/.  The digest per hundred records lets a test say where a plan first differs.\n")
            f.write(f"trace_sha256 {trace_digest(w.trace)}\n")
            f.write(f"records_sha256 {records_digest(p.records)}\n")
            f.write(f"pressure_after_sha256 {hashlib.sha256(p.pressure_after.astype('<u8').tobytes()).hexdigest()}\n")
            f.write(f"status {p.status}\npasses {p.n_iterations}\nmigrations {p.n_migrations}\n"
                    f"dropped {p.n_null}\ncand_evals {p.n_cand_evals}\n")
            for k in range(0, len(p.records), 100):
                f.write(f"records_{k}_sha256 {records_digest(p.records[k:k + 100])}\n")
        print("ratio written")
        if which == "ratio":
            return
    p = v.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus)
    with open(os.path.join(HERE, "config5_plan_digest.txt"), "w") as f:
        f.write("# Complete plan of the CPU oracle for the stress workload (config 5), as digests.\n")
        f.write("# Written by tests/golden/make_config5_digest.py, which calls only oracle/.\n")
        f.write(f"trace_sha256 {trace_digest(w.trace)}\n")
        f.write(f"records_sha256 {records_digest(p.records)}\n")
        f.write(f"pressure_after_sha256 {hashlib.sha256(p.pressure_after.astype('<u8').tobytes()).hexdigest()}\n")
        f.write(f"status {p.status}\npasses {p.n_iterations}\nmigrations {p.n_migrations}\n"
                f"dropped {p.n_null}\ncand_evals {p.n_cand_evals}\n")
    print("written")


if __name__ == "__main__":
    main()
