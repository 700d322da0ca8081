#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A step = g10_vitality + g10_plan (tensor vitality analysis, candidate
preparation and the complete greedy eviction loop) on the stress trace
(100 000 kernels, 1 000 000 tensors), the trace already resident in HBM.
Prints one JSON line.  `value` = candidate evaluations per second over the
whole step (sum over ranking passes of the live candidates / step time).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


BYTES_PER_CAND = 36            # what a scoring pass over a candidate moves by definition: L+1, R, 2 x (a, b) as u32 + size u64
                               # read, a 4-byte key written
BYTES_PER_CAND_READ_ONLY = 32  # the same without the key (the arg-max fused into the pass: nothing written)
BYTES_PER_CAND_MOVED = 20      # what k_score_full itself streams per candidate: a 16-byte packed copy (four window
                               # ends of 21 bits, 43 bits of size; 24 bytes where a trace exceeds that) + the 4-byte key;
                               # its gathers (two 8-byte words per window) hit a table that stays in L2


# HBM traffic of the loop kernel on config 5 from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, scaled by what the
# same counters read for a 256 MiB copy): profiles/loop_stress_hbm_counters.md has the commands and the sums.  The
# figures hold for the kernel they were taken on: reported only while the kernel's sources hash to what they did then.
LOOP_TRAFFIC = {"sha256": {"g10_loop.hip": "3c6f01f2fb00ae43315726b03d712aece9ec43d892a9cca014e32bd24dc844ee",
                           "g10_plan_defs.h": "29da48963f0aaf9bd88314d48c4f2f465f7d1896872937d584d8bbcd3c7fc7d0"},
                "workload": "config 5", "fetch_bytes_per_plan": 57.8e6, "write_bytes_per_plan": 81.7e6, "launches_per_plan": 11}


def loop_traffic_per_launch(config):
    """Bytes per launch of k_loop by the stored counters, or None where they do not apply (another workload, or the
    kernel has changed since they were taken)."""
    import hashlib
    if config != 5:
        return None
    for name, want in LOOP_TRAFFIC["sha256"].items():
        try:
            got = hashlib.sha256(open(os.path.join(ROOT, "paper_2310_09443_amd", "csrc", name), "rb").read()).hexdigest()
        except OSError:
            return None
        if got != want:
            return None
    return (LOOP_TRAFFIC["fetch_bytes_per_plan"] + LOOP_TRAFFIC["write_bytes_per_plan"]) / LOOP_TRAFFIC["launches_per_plan"]


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def oracle_pinned(fn):
    """Runs fn() with this process pinned to one core (the oracle is single-threaded); returns (result, core or None)."""
    try:
        allowed = sorted(os.sched_getaffinity(0))
        os.sched_setaffinity(0, {allowed[-1]})
    except (AttributeError, OSError):
        return fn(), None
    try:
        return fn(), allowed[-1]
    finally:
        os.sched_setaffinity(0, set(allowed))


def one_config(binding, traces, cfg, dev, steps, with_oracle):
    """One of the smaller workloads: the step (analysis + plan) on the GPU, and the oracle's whole plan on one core."""
    import torch
    w = traces.config(cfg)
    tr = w.trace
    dt = binding.DeviceTrace(tr, dev)

    def step():
        h = binding.g10_vitality(dt)
        cap, hcap = traces.resolve_caps(w, h.peak)
        r = h.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus)
        C = h.C
        h.close()
        return r, C
    step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        r, C = step()
    torch.cuda.synchronize()
    dt_s = (time.perf_counter() - t0) / steps
    row = {"config": cfg, "workload": tr.name, "K": tr.K, "N": tr.N, "P": tr.P, "periods": C,
           "passes": int(r.n_iterations), "migrations": int(r.n_migrations), "status": int(r.status),
           "ms_per_step": dt_s * 1e3, "plan_ms": r.plan_ms, "loop_ms": r.loop_ms,
           "loop_kernel_passes": int(r.loop_passes), "candidates_per_s": r.n_cand_evals / dt_s}
    if with_oracle:
        from oracle import oracle as O

        def run():
            t0 = time.perf_counter()
            v = O.Vitality(tr, O.PREFIX)
            cap, hcap = traces.resolve_caps(w, v.peak)
            p = v.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus)
            return p, time.perf_counter() - t0
        (p, t), _ = oracle_pinned(run)
        row["oracle_ms"] = t * 1e3
        row["oracle_candidates_per_s"] = p.n_cand_evals / t
        row["oracle_matches"] = bool(p.records.tobytes() == r.records.tobytes())
    return row


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the stress trace)")
    ap.add_argument("--cpu-passes", type=int, default=0,
                    help="ranking passes of the CPU oracle to time (0 = sized to roughly 15 s)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--batch", type=int, default=256,
                    help="plans of the extra capacity-sweep measurement with g10_plan_batch (0 or 1: skip)")
    ap.add_argument("--no-configs", dest="configs", action="store_false",
                    help="skip the per-workload rows for configs 1-4")
    ap.add_argument("--probe", action="store_true",
                    help="counter probe: one 256 MiB device copy (calibration), one analysis and a plan cut after 8 passes")
    ap.add_argument("--peak-check", action="store_true",
                    help="what the HBM peak of the roofline is checked against: device properties and measured copy / read rates")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: the planner runs on one GPU only (planning one trace is a serial greedy loop; "
                 "several GPUs would each plan their own trace independently). Use --gpus 1.")

    import torch
    from paper_2310_09443_amd import binding, traces
    binding.load()
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = "cuda:0"

    if a.peak_check:
        p = torch.cuda.get_device_properties(0)
        clk_khz, bus = getattr(p, "memory_clock_rate", None), getattr(p, "memory_bus_width", None)
        out = {"peak_check": True, "device": p.name, "compute_units": p.multi_processor_count,
               "memory_clock_khz": clk_khz, "memory_bus_bits": bus, "published_GBps": HBM_PEAK_GBS,
               # HBM3E moves four bits per pin per reported clock
               "clock_x_bus_x4_GBps": (clk_khz * 1e3 * bus / 8 * 4 / 1e9) if clk_khz and bus else None,
               "copy": [], "read": []}
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for mb in (64, 256, 1024, 4096):
            n = mb << 20
            x = torch.empty(n, dtype=torch.uint8, device=dev)
            y = torch.empty_like(x)
            x.fill_(1)
            y.copy_(x)
            v = x.view(torch.int64)
            best_c = best_r = 1e9
            for _ in range(10):
                e0.record(); y.copy_(x); e1.record(); torch.cuda.synchronize()
                best_c = min(best_c, e0.elapsed_time(e1))
                e0.record(); v.sum(); e1.record(); torch.cuda.synchronize()
                best_r = min(best_r, e0.elapsed_time(e1))
            out["copy"].append({"MiB": mb, "ms": best_c, "GBps_read_plus_write": 2 * n / best_c / 1e6})
            out["read"].append({"MiB": mb, "ms": best_r, "GBps": n / best_r / 1e6})
            del x, y, v
        print(json.dumps(out))
        return

    w = traces.config(a.config)
    tr = w.trace
    dt = binding.DeviceTrace(tr, dev)
    torch.cuda.synchronize()

    if a.probe:
        src = torch.zeros(32 << 20, dtype=torch.int64, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)                          # reads 256 MiB, writes 256 MiB
        h = binding.g10_vitality(dt)
        cap, hcap = traces.resolve_caps(w, h.peak)
        r = h.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus, max_iters=8)
        torch.cuda.synchronize()
        print(json.dumps({"probe": True, "copy_bytes_each_way": 256 << 20, "passes": int(r.n_iterations),
                          "cands_in_scoring_pass": int(r.score_full_cands)}))
        return

    def step():
        h = binding.g10_vitality(dt)
        cap, hcap = traces.resolve_caps(w, h.peak)
        r = h.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus)
        h.close()
        return h, r

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    runs = []
    t0 = time.perf_counter()
    for _ in range(a.steps):
        h, r = step()
        runs.append(r)
    torch.cuda.synchronize()
    dt_s = (time.perf_counter() - t0) / a.steps
    assert all(x.records.tobytes() == r.records.tobytes() for x in runs)

    # Two kernels are reported.  k_loop takes the time (the greedy loop, one persistent workgroup): its
    # roofline entry counts the bytes it really moves, from its own counters, which is far under any
    # bandwidth roof - it is bound by the latency of a serial chain of dependent steps.  k_score_full is
    # the one pass that streams every candidate (once per plan): timed by the library with HIP events
    # bound to the kernel's begin and end on the planner's stream.
    launches = len(runs)
    avg_ms = sum(x.score_full_ms for x in runs) / launches
    cands_per_launch = float(r.score_full_cands)
    def rate(bytes_per_cand):
        return cands_per_launch * bytes_per_cand / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
    loop_ms = sum(x.loop_ms for x in runs) / launches
    passes = max(int(r.n_iterations), 1)
    kpasses = max(int(r.loop_passes), 1)
    # bytes the loop kernel moves per plan: 40-byte candidate records re-scored (+ 8 gathers of 16 bytes for the
    # live ones, here counted for all), chunk jobs of 256 slots (two 8-byte timelines read, one written, prefix words)
    loop_bytes = r.loop_cands_scored * (40.0 + 8 * 16.0) + r.loop_chunk_jobs * 256 * 32.0
    loop_gbps = loop_bytes / (loop_ms * 1e-3) / 1e9 if loop_ms > 0 else 0.0
    listing_bytes = 32.0 * r.n_cand_evals + 72.0 * tr.K * passes       # what Algorithm 1 as listed would stream
    scored = float(r.score_full_cands + r.loop_cands_scored + r.retile_cands)

    out = {
        "metric": "migration candidates scored/sec (whole step: vitality analysis + eviction plan)",
        "value": r.n_cand_evals / dt_s,
        "unit": "candidates/s",
        "value_definition": "Algorithm 1's count: the sum over its ranking passes of the candidates live in the pass "
                            "(what the listing ranks and the CPU oracle does rank), divided by the step time.  The GPU "
                            "planner reaches the same decisions looking at far fewer: see candidates_actually_scored_per_s",
        "candidates_actually_scored_per_s": scored / dt_s,
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt_s * 1e3,
        "plan_ms": sum(x.plan_ms for x in runs) / launches,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": f"config {a.config}: {tr.name}", "K": tr.K, "N": tr.N, "P": tr.P,
                   "periods": h.C, "passes": int(r.n_iterations), "migrations": int(r.n_migrations),
                   "dropped": int(r.n_dropped), "status": int(r.status), "cap_frac": w.cap_frac,
                   "bw_out_Bpus": list(w.bw_out_Bpus), "bw_in_Bpus": list(w.bw_in_Bpus)},
        "roofline": {"bound": "hbm", "kernel": "k_loop", "achieved": loop_gbps, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": loop_gbps / HBM_PEAK_GBS, "traffic": loop_traffic_per_launch(a.config),
                     "traffic_unit": "bytes per launch",
                     "traffic_source": "stored: two rocprofv3 --pmc runs on this kernel (profiles/loop_stress_hbm_counters.md); "
                                       "null when the kernel's sources have changed since, or for another workload",
                     "achieved_bytes_per_launch": loop_bytes / max(int(r.loop_launches), 1),
                     "ms": loop_ms, "share_of_step": loop_ms / (dt_s * 1e3), "launches": int(r.loop_launches),
                     "bytes_per_plan": loop_bytes,
                     "listing_equivalent_GBps": listing_bytes / (loop_ms * 1e-3) / 1e9 if loop_ms > 0 else 0.0,
                     "us_per_algorithm_pass": 1e3 * loop_ms / passes, "kernel_passes": int(r.loop_passes),
                     "more_commit_rounds_from_the_same_list": int(r.loop_more_rounds),
                     "us_per_commit_round": 1e3 * loop_ms / max(int(r.loop_passes + r.loop_more_rounds), 1),
                     "migrations_per_kernel_pass": passes / kpasses, "us_per_kernel_pass": 1e3 * loop_ms / kpasses,
                     "retiles": int(r.loop_retiles), "cands_rescored_per_kernel_pass": r.loop_cands_scored / kpasses,
                     "second_rounds": int(r.loop_second_rounds), "chunk_jobs_per_kernel_pass": r.loop_chunk_jobs / kpasses,
                     "note": "the dominant kernel: one persistent workgroup, a serial chain of dependent small steps per "
                             "pass, bound by instruction and memory latency, not by bandwidth: achieved = the bytes it "
                             "really reads and writes (its own counters) / its time.  listing_equivalent_GBps is what "
                             "Algorithm 1 as listed would have to stream to do the same passes: not a bandwidth this "
                             "kernel reaches, only a measure of the work it avoids.  There is no streaming "
                             "timeline-update kernel to put on the roofline: updates touch a few chunks per migration"},
        "roofline_scoring_pass": {"bound": "hbm", "kernel": "k_score_full", "achieved": rate(BYTES_PER_CAND), "peak": HBM_PEAK_GBS,
                                  "unit": "GB/s", "frac": rate(BYTES_PER_CAND) / HBM_PEAK_GBS,
                                  "frac_at_32B": rate(BYTES_PER_CAND_READ_ONLY) / HBM_PEAK_GBS,
                                  "frac_moved_20B": rate(BYTES_PER_CAND_MOVED) / HBM_PEAK_GBS,
                                  "traffic": None, "traffic_source": "none in this run; counters of an earlier build: "
                                  "profiles/score_full_stress_hbm_counters.md",
                                  "launches": launches, "avg_launch_us": avg_ms * 1e3,
                                  "share_of_step": avg_ms / (dt_s * 1e3),
                                  "cands_per_launch": cands_per_launch, "bytes_per_cand": BYTES_PER_CAND,
                                  "algorithmic_bytes_per_launch": cands_per_launch * BYTES_PER_CAND,
                                  "note": "the one pass that streams every candidate, once per plan.  frac: 36 B per "
                                          "candidate (32 B read + the 4-byte key it writes); frac_at_32B: the read side "
                                          "alone; frac_moved_20B: the bytes the kernel itself streams (16-byte packed "
                                          "copy + key), its gathers staying in L2"},
    }

    # smart prefetching (Section 4.4) on the finished plan: a further row of the path, timed on its own
    hp = binding.g10_vitality(dt)
    cap, hcap = traces.resolve_caps(w, hp.peak)
    hp.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus)
    pf = [hp.prefetch() for _ in range(3)][-1]
    out["smart_prefetch"] = {"kernel": "k_eager", "ms": pf.ms, "migrations": pf.n_migrations, "moved": pf.n_moved,
                             "slots_gained": pf.slots_gained, "us_per_migration": 1e3 * pf.ms / max(pf.n_migrations, 1)}

    # slot-level replay of that plan (one first-in-first-out channel per destination and direction):
    # stall time as planned and with +-20 % kernel-time noise, each with the prefetches at their latest
    # safe time and where smart prefetching moved them
    noisy = torch.from_numpy(traces.noisy_durations(tr, 20.0, seed=2020).view(np.int64)).to(dev)
    out["replay"] = {}
    for name, d, eager in (("as_planned", None, False), ("as_planned_smart_prefetch", None, True),
                           ("noise_20_percent", noisy, False), ("noise_20_percent_smart_prefetch", noisy, True)):
        hp.replay(d, eager)
        rr = hp.replay(d, eager)
        out["replay"][name] = {"ms": rr.ms, "iter_ms": rr.iter_ns / 1e6, "stall_ms": rr.stall_ns / 1e6,
                               "stalled_kernels": rr.n_stalled, "late_migrations": int((rr.late > 0).sum()),
                               "GB_to_flash_host": [x / 1e9 for x in rr.bytes]}
    hp.close()

    # a capacity sweep planned in one call (g10_plan_batch): the loops of the plans run side by side
    nb = a.batch
    if nb > 1:
        hb = binding.g10_vitality(dt)
        base = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
        sweep = [dict(base, gpu_cap=int(hb.peak * (0.20 + 0.15 * i / (nb - 1)))) for i in range(nb)]
        hb.plan_batch(sweep)                                    # warm-up (allocates the workspaces)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rs = hb.plan_batch(sweep)
        tb = time.perf_counter() - t0
        out["batch"] = {"plans": nb, "sweep": "gpu_cap 20..35 % of the peak footprint", "ms": tb * 1e3,
                        "library_ms": rs[0].plan_ms, "prepare_ms": rs[0].batch_prepare_ms, "loops_ms": rs[0].batch_loops_ms,
                        "retile_ms": rs[0].batch_retile_ms, "results_ms": rs[0].batch_results_ms,
                        "binding_ms": tb * 1e3 - rs[0].plan_ms,
                        "ms_per_plan": tb * 1e3 / nb, "passes": int(sum(x.n_iterations for x in rs)),
                        "candidates_per_s": sum(x.n_cand_evals for x in rs) / tb,
                        "speedup_over_one_by_one": (r.plan_ms * 1e-3 * nb) / tb}
        # the flash-bandwidth sweep of Section 7 (6.4 to 32 GB/s): no two plans share their candidate windows
        sweep = []
        for i in range(nb):
            f = 6400 + (32000 - 6400) * i // (nb - 1)
            sweep.append(dict(base, bw_out=(f, w.bw_out_Bpus[1]), bw_in=(f, w.bw_in_Bpus[1])))
        hb.plan_batch(sweep)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rs = hb.plan_batch(sweep)
        tb = time.perf_counter() - t0
        hb.close()
        out["batch_bandwidth_sweep"] = {"plans": nb, "sweep": "flash bandwidth 6.4..32 GB/s", "ms": tb * 1e3,
                                        "prepare_ms": rs[0].batch_prepare_ms, "loops_ms": rs[0].batch_loops_ms,
                                        "retile_ms": rs[0].batch_retile_ms, "results_ms": rs[0].batch_results_ms,
                                        "ms_per_plan": tb * 1e3 / nb, "passes": int(sum(x.n_iterations for x in rs)),
                                        "candidates_per_s": sum(x.n_cand_evals for x in rs) / tb}

    # re-planning under kernel-time noise (the profiling-error study): the same batch call, every
    # plan on durations of its own; how much of the exact plan survives is reported beside the time
    if nb > 1:
        hn = binding.g10_vitality(dt)
        pcts = [0.0, 5.0, 10.0, 15.0, 20.0, 25.0]
        durs = [torch.from_numpy(traces.noisy_durations(tr, pc, seed=1000 + int(pc)).view(np.int64)).to(dev)
                for pc in pcts]
        sweep = [dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus,
                      dur=(None if pc == 0.0 else d)) for pc, d in zip(pcts, durs)]
        hn.plan_batch(sweep)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rn = hn.plan_batch(sweep)
        tn = time.perf_counter() - t0
        exact = set(zip(rn[0].records["cand"].tolist(), rn[0].records["dest"].tolist()))
        kept = [len(exact & set(zip(x.records["cand"].tolist(), x.records["dest"].tolist()))) / max(len(exact), 1)
                for x in rn]
        hn.close()
        out["noise_sweep"] = {"plans": len(pcts), "noise_percent": pcts, "ms": tn * 1e3,
                              "migrations": [int(x.n_migrations) for x in rn],
                              "share_of_exact_plan_kept": kept}

    # the two alternative readings of Section 4.3 on the same trace (outside the timed step):
    # the clipped-area benefit for the whole plan, the ratio key for its first 1000 passes (that
    # key prefers small tensors, so its plan on this trace has 20x the migrations)
    if nb > 1:
        hv = binding.g10_vitality(dt)
        base_args = dict(gpu_cap=cap, host_cap=hcap, bw_out=w.bw_out_Bpus, bw_in=w.bw_in_Bpus)
        b0 = hv.plan(**base_args)
        out["readings"] = {}
        for name, va in (("clipped_area", dict(area=1)), ("ratio_key_first_1000_passes", dict(rank=1, max_iters=1000))):
            hv.plan(**base_args, **va)
            rv = hv.plan(**base_args, **va)
            k = min(len(b0.records), len(rv.records))
            same = b0.records["cand"][:k] == rv.records["cand"][:k]
            common = len(set(b0.records["cand"].tolist()) & set(rv.records["cand"].tolist()))
            out["readings"][name] = {"ms": rv.plan_ms, "passes": int(rv.n_iterations), "migrations": int(rv.n_migrations),
                                     "us_per_pass": 1e3 * rv.loop_ms / max(int(rv.n_iterations), 1),
                                     "cands_rescored_per_pass": rv.loop_cands_scored / max(int(rv.n_iterations), 1),
                                     "areas_summed": int(rv.loop_area_evals), "areas_below_bound": int(rv.loop_area_refused),
                                     "rounds_scored_by_k_wide_score": int(rv.loop_wide_rounds),
                                     "first_record_that_differs_from_default": int((~same).argmax()) if not same.all() else k,
                                     "migrations_shared_with_default": common}
        hv.close()

    # the other workloads (milliseconds each): the step on the GPU beside the oracle's complete plan on one core
    if a.config == 5 and a.configs:
        out["configs"] = [one_config(binding, traces, c, dev, max(a.steps, 3), not a.no_cpu) for c in (1, 2, 3, 4)]

    if not a.no_cpu:
        from oracle import oracle as O

        def run():
            t0 = time.perf_counter()
            v = O.Vitality(tr, O.PREFIX)
            t_vit = time.perf_counter() - t0
            cap, hcap = traces.resolve_caps(w, v.peak)
            passes = a.cpu_passes
            if passes <= 0:                         # ~15 s of single-thread work at ~10 ns per evaluation
                passes = max(1, min(int(r.n_iterations), int(1.5e9 / max(v.C, 1))))
            t0 = time.perf_counter()
            p = v.plan(cap, hcap, w.bw_out_Bpus, w.bw_in_Bpus, max_iters=passes)
            return p, t_vit, time.perf_counter() - t0
        (p, t_vit, t_plan), core = oracle_pinned(run)
        n = len(p.records)
        same = all((r.records[f][:n] == p.records[f]).all() for f in p.records.dtype.names)
        out["cpu_baseline"] = {"value": p.n_cand_evals / (t_vit + t_plan), "unit": "candidates/s", "cores": 1,
                               "kind": "oracle", "threads_used": 1, "nproc": os.cpu_count(),
                               "cpu_model": cpu_model(), "pinned_to_core": core,
                               "sample": f"vitality analysis + the first {p.n_iterations} of {int(r.n_iterations)} "
                                         f"ranking passes of the same trace ({t_vit + t_plan:.1f} s)",
                               "matches_gpu_prefix": bool(same)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
