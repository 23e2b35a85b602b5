#!/usr/bin/env python3
"""Benchmark of the MMEE hot path on one MI355X.

A step is one complete search of the BERT-base-like configuration (B=1, H=12,
N=512, d=64, fp16; 16x16 PEs, 256 KB buffer, 256 B register files) for its two
objectives, energy-driven and latency-driven, in one pass: tiling tables are
built, every candidate that denotes a dataflow is decoded and costed (buffer
size, DRAM access, buffer<->RF traffic, cycles, energy, latency), masked by the
capacity constraint, and reduced on the device to the two optimal mappings.
Nothing is pruned in the timed steps, so candidates/s counts costs really formed;
the pruned search (the paper's method) is timed next to it as time-to-optimum.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# VALU issue peak of the chip: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second.
# (The published 78.6 TFLOP/s fp64 vector peak is this number times two for fused multiply-add;
# the model's additions, multiplications, maxima and comparisons round one by one, so each
# lane-operation is one operation.)
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# fp64-width operations the model needs.  Shared by the nine candidates of a (row, tiling) pair:
# 4 additions + max + compare for the buffer size and capacity, 2 additions for DRAM access,
# 2 products, 2 masks = 12.  Per candidate, with the energy regrouped (whole-number energies:
# every term exact, see MMEE_SEARCH_ORDERED_SUM): one addition, the latency max and one running
# minimum for each of the two objectives = 4; with the sum taken term by term: buffer words,
# e_gb product, three energy additions, latency max, two minima = 8.
OPS_PER_CANDIDATE = {True: 4 + 12 / 9, False: 8 + 12 / 9}
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/*.md), scaled by what the
# same counters read for a 1 GiB device-to-device copy (x2.0 and x1.0).  Valid only for the kernel
# sources they were taken with: any change to the sources turns "traffic" into null.
COUNTERS_TAKEN_WITH = "b0b8c5fa694cfc05fb8c67ef961c34def2104c105b0c8ee023167c3e0c6ea0f6"
SEARCH_TRAFFIC_BYTES = 28572.4 * 1024 * 2.0 + 325.1 * 1024 * 1.0
EVAL_TRAFFIC_BYTES = 22346.9 * 1024 * 2.0 + 4197505.2 * 1024 * 1.0


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    for f in ("layout.h", "kernels.h", "mmee.hip"):
        with open(os.path.join(ROOT, "paper_2604_03446_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-only", action="store_true",
                    help="run the timed steps only (for rocprofv3): no oracle, no extra legs")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on one GPU; --gpus %d is not supported "
                 "(the index space would shard by contiguous index ranges, one final min)" % args.gpus)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    import paper_2604_03446_amd as M
    from inputs import CONFIGS

    stream = torch.cuda.current_stream()
    M.mmee_set_stream(stream.cuda_stream)
    t0 = time.perf_counter()
    stats = M.mmee_offline_stats()            # offline stage: row encoding + pruning, once per process
    torch.cuda.synchronize()
    offline_ms = (time.perf_counter() - t0) * 1e3

    cfg = CONFIGS["bert"]
    w, h = M.workload(cfg["workload"]), M.hw(cfg["hw"])      # C structs once, not per call
    objectives = [M.OBJ_ENERGY, M.OBJ_LATENCY]
    regrouped = M.mmee_energy_regrouped(w, h, M.SEARCH_EXHAUSTIVE)
    ops = OPS_PER_CANDIDATE[regrouped]

    for _ in range(args.warmup):
        M.mmee_search_multi(w, h, objectives, M.SEARCH_EXHAUSTIVE)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kernel_s = 0.0
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        res = M.mmee_search_multi(w, h, objectives, M.SEARCH_EXHAUSTIVE)
        kernel_s += res[0].kernel_seconds
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    stream_ms = ev0.elapsed_time(ev1)
    evaluated = res[0].evaluated
    ms_per_step = wall / args.steps * 1e3
    kernel_ms = kernel_s / args.steps * 1e3
    value = evaluated / (wall / args.steps)

    out = {
        "metric": "candidate mappings evaluated/sec (every dataflow costed, energy- and latency-driven optimum in one pass)",
        "value": value, "unit": "candidates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": "bert: B=1 H=12 N=512 d=64 fp16 words; 16x16 PE array, 256 KiB GB, 256 B RF; "
                               "DRAM 200 / GB 6 / RF 1 / MAC 1 pJ; power-of-two tilings, 24 orders, 5^4 levels, "
                               "recompute, 3x3 stationary modes, fused/unfused",
                   "space": res[0].space, "candidates_costed_per_step": evaluated,
                   "objectives": ["energy", "latency"], "search": "exhaustive"},
        "best": {"energy": {"idx": res[0].best.idx, "energy_pj": res[0].cost.energy_pj,
                            "latency_cycles": res[0].cost.latency_cycles},
                 "latency": {"idx": res[1].best.idx, "energy_pj": res[1].cost.energy_pj,
                             "latency_cycles": res[1].cost.latency_cycles}},
        "search_kernel_ms": kernel_ms, "stream_ms_per_step": stream_ms / args.steps,
        "roofline": {"bound": "alu", "achieved": ops * evaluated / (kernel_ms * 1e-3) / 1e12,
                     "peak": ALU_PEAK_TOPS, "unit": "Tlane-op/s", "traffic": None,
                     "kernel": "k_search<energy+latency%s>" % (", regrouped energy sum" if regrouped else ""),
                     "ops_per_candidate": ops,
                     "kernel_candidates_per_s": evaluated / (kernel_ms * 1e-3)},
    }
    out["roofline"]["frac"] = out["roofline"]["achieved"] / out["roofline"]["peak"]
    counters_valid = kernel_sources_digest() == COUNTERS_TAKEN_WITH
    if counters_valid:
        out["roofline"]["traffic"] = SEARCH_TRAFFIC_BYTES

    if not args.profile_only:
        # the same step with the energy summed term by term (what a workload with fractional
        # energies per access gets)
        flags = M.SEARCH_EXHAUSTIVE | M.SEARCH_ORDERED_SUM
        for _ in range(5):
            M.mmee_search_multi(w, h, objectives, flags)
        n, ks = 50, 0.0
        t1 = time.perf_counter()
        for _ in range(n):
            ks += M.mmee_search_multi(w, h, objectives, flags)[0].kernel_seconds
        wall_o = (time.perf_counter() - t1) / n
        ach = OPS_PER_CANDIDATE[False] * evaluated / (ks / n) / 1e12
        out["ordered_sum"] = {"value": evaluated / wall_o, "unit": "candidates/s", "search_kernel_ms": ks / n * 1e3,
                              "roofline": {"bound": "alu", "achieved": ach, "peak": ALU_PEAK_TOPS,
                                           "unit": "Tlane-op/s", "frac": ach / ALU_PEAK_TOPS,
                                           "ops_per_candidate": OPS_PER_CANDIDATE[False]}}

        # time-to-optimum of the paper's method (pruned rows), host wall time per call
        tto = {}
        for name, c in CONFIGS.items():
            objs = c["objectives"]
            cw, ch = M.workload(c["workload"]), M.hw(c["hw"])
            for _ in range(5):
                M.mmee_search_multi(cw, ch, objs, M.SEARCH_PRUNED)
            n = 50
            t1 = time.perf_counter()
            for _ in range(n):
                r = M.mmee_search_multi(cw, ch, objs, M.SEARCH_PRUNED)
            dt_p = (time.perf_counter() - t1) / n
            for _ in range(2):
                M.mmee_search_multi(cw, ch, objs, M.SEARCH_EXHAUSTIVE)
            n = 10
            t1 = time.perf_counter()
            for _ in range(n):
                rx = M.mmee_search_multi(cw, ch, objs, M.SEARCH_EXHAUSTIVE)
            dt_x = (time.perf_counter() - t1) / n
            assert [a.best.idx for a in r] == [a.best.idx for a in rx]
            tto[name] = {"pruned_ms": dt_p * 1e3, "pruned_candidates": r[0].evaluated,
                         "exhaustive_ms": dt_x * 1e3, "exhaustive_candidates": rx[0].evaluated,
                         "exhaustive_kernel_ms": rx[0].kernel_seconds * 1e3,
                         "exhaustive_candidates_per_s": rx[0].evaluated / dt_x}
        out["time_to_optimum"] = tto
        out["offline_stage"] = {"ms_first_call": offline_ms, "rows_valid": list(stats.rows_valid),
                                "rows_kept": list(stats.rows_kept)}

        # per-candidate records: HBM-write bound, 64 bytes each
        n_rec = 1 << 26
        buf = torch.empty(n_rec * 8, dtype=torch.int64, device="cuda")
        first = 1_000_000_007
        for _ in range(3):
            M.mmee_eval_batch(w, h, first, n_rec, out=buf.data_ptr())
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record(stream)
        for _ in range(reps):
            M.mmee_eval_batch(w, h, first, n_rec, out=buf.data_ptr())
        e1.record(stream)
        torch.cuda.synchronize()
        eval_ms = e0.elapsed_time(e1) / reps
        gbs = n_rec * 64 / (eval_ms * 1e-3) / 1e9
        out["roofline_eval_batch"] = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": gbs / HBM_PEAK_GBS, "traffic": None, "kernel": "k_eval_batch",
                                      "records": n_rec, "ms": eval_ms,
                                      "candidates_per_s": n_rec / (eval_ms * 1e-3)}
        if counters_valid:
            out["roofline_eval_batch"]["traffic"] = EVAL_TRAFFIC_BYTES
        # a plain device-to-device copy of known size (1 GiB read + 1 GiB written): the reference
        # reading for the FETCH_SIZE / WRITE_SIZE counters when the run is profiled
        src = torch.zeros(1 << 27, dtype=torch.int64, device="cuda")
        buf[: src.numel()].copy_(src)
        torch.cuda.synchronize()
        del buf, src

    if not args.no_cpu_baseline and not args.profile_only:
        import oracle as O
        ow, oh = O.workload(cfg["workload"]), O.hw(cfg["hw"])
        t1 = time.perf_counter()
        rc, idx, cost, n_valid, threads = O.search_all(ow, oh)
        dt = time.perf_counter() - t1
        assert rc == 0 and idx[0] == res[0].best.idx and idx[1] == res[1].best.idx, "GPU and oracle disagree"
        assert cost[0].energy_pj == res[0].cost.energy_pj and cost[1].latency_cycles == res[1].cost.latency_cycles
        out["cpu_baseline"] = {"value": evaluated / dt, "unit": "candidates/s", "cores": threads, "kind": "oracle",
                               "sample": "the whole bert space: all %d indices enumerated once, three objectives "
                                         "kept, %d of them denote a dataflow and are costed" % (res[0].space, evaluated),
                               "seconds": dt, "optimum_matches_gpu": True}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
