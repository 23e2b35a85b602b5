#!/usr/bin/env python3
"""Benchmark of the MMEE hot path on one MI355X.

A step is one complete exhaustive search of the long-context configuration (B=1, H=32,
N=8192, d=128, fp16; 128x128 PEs, 8 MiB buffer, 1 KiB register files; tilings over all
divisors: 6.77e9 candidate indices) for its objective, the energy: tiling tables are built,
every candidate that denotes a dataflow is decoded and costed (buffer size, DRAM access,
buffer<->RF traffic, cycles, energy), masked by the capacity constraint, and reduced on the
device to the optimal mapping.  Nothing is pruned in the timed steps, so candidates/s counts
costs really formed; the pruned search (the paper's method) is timed next to it as
time-to-optimum, and the 1024-search hardware sweep as its own leg.

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
# fp64-width operations the model needs per candidate.
# One key (energy) over the full row set, k_search_dense.  Shared by the nine candidates of a
# (row, tiling) pair: one addition each for Eq. (1) and Eq. (2) (pair sums come from the tables),
# max + compare for Eq. (4) and the capacity, one addition for Eq. (7), one product, select + max for
# the mask = 8.  Per candidate, energy regrouped (every term an exact integer): one addition and the
# running minimum = 2; summed term by term: buffer words, e_gb product, three additions, minimum = 6.
OPS_DENSE_ENERGY = {True: 2 + 8 / 9, False: 6 + 8 / 9}
# Two keys (energy and latency) in one pass, k_search: 12 shared (as above plus the second addition of
# Eq. (1), (2), (7) that the row-per-lane kernel cannot fold, the latency product and its mask), and per
# candidate one addition, the latency max and two minima = 4 (8 term by term).
OPS_TWO_KEYS = {True: 4 + 12 / 9, False: 8 + 12 / 9}
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (summaries under profiles/), scaled by
# what the same counters read for a 1 GiB device-to-device copy (x2.0 and x1.0).  Valid only for the kernel
# sources they were taken with: any change to the sources turns "traffic" into null.
COUNTERS_TAKEN_WITH = "74cedcfbae3e9edf44926a0a0e7caf7f4cb45343d2735171fe7d2f1858ba838b"
TRAFFIC = {"k_search_dense_long": (2 * 58521.384 + 384.183) * 1024.0,      # FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, KiB per dispatch
           "k_search_bert": (2 * 26597.313 + 325.094) * 1024.0,
           "k_eval_batch": (2 * 20242.527 + 4194995.589) * 1024.0}
TRAFFIC_SOURCE = {"k_search_dense_long": "profiles/k_search_dense_long.md", "k_search_bert": "profiles/k_search_bert_exhaustive.md",
                  "k_eval_batch": "profiles/k_eval_batch_bert.md"}


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    for f in ("layout.h", "kernels.h", "batch.h", "mmee.hip"):
        with open(os.path.join(ROOT, "paper_2604_03446_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def traffic_of(kernel):
    """(bytes per launch or None, where the figure comes from)."""
    if kernel_sources_digest() != COUNTERS_TAKEN_WITH:
        return None, TRAFFIC_SOURCE[kernel] + " (kernel sources changed since the counters were taken)"
    return TRAFFIC[kernel], TRAFFIC_SOURCE[kernel]


def describe(cfg):
    w, h = cfg["workload"], cfg["hw"]
    return ("B=%d H=%d N=%d d=%d fp16 words; %dx%d PE array, %d KiB GB, %d B RF; DRAM %g / GB %g / RF %g / MAC %g pJ; "
            "%s tilings, 24 orders, 5^4 levels, recompute, 3x3 stationary modes, fused/unfused"
            % (w["B"], w["H"], w["N"], w["d"], h["pe_rows"], h["pe_cols"], h["gb_bytes"] // 1024, h["rf_bytes"],
               h["e_dram"], h["e_gb"], h["e_rf"], h["e_mac"], "all-divisor" if w["tiling_mode"] else "power-of-two"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-only", action="store_true",
                    help="run the timed steps only (for rocprofv3): no oracle, no extra legs")
    ap.add_argument("--profile-leg", choices=["long", "bert", "sweep", "eval"], default="long",
                    help="with --profile-only: which leg the timed steps run")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on one GPU; --gpus %d is not supported "
                 "(the index space would shard by contiguous index ranges, one final min)" % args.gpus)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    import paper_2604_03446_amd as M
    from inputs import CHAINS, CONFIGS, sweep_points

    stream = torch.cuda.current_stream()
    M.mmee_set_stream(stream.cuda_stream)
    t0 = time.perf_counter()
    stats = M.mmee_offline_stats()            # offline stage: row encoding + pruning, once per process
    torch.cuda.synchronize()
    offline_ms = (time.perf_counter() - t0) * 1e3

    def timed_search(cfg, objectives, flags, steps, warmup):
        """`steps` searches back to back: wall time per step, kernel time per step (HIP events inside the
        library, on the stream the kernels run on), stream time per step, last results."""
        w, h = M.workload(cfg["workload"]), M.hw(cfg["hw"])      # C structs once, not per call
        for _ in range(warmup):
            M.mmee_search_multi(w, h, objectives, flags)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        kernel_s = 0.0
        t1 = time.perf_counter()
        ev0.record(stream)
        for _ in range(steps):
            res = M.mmee_search_multi(w, h, objectives, flags)
            kernel_s += res[0].kernel_seconds
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t1
        return wall / steps, kernel_s / steps, ev0.elapsed_time(ev1) * 1e-3 / steps, res

    def sweep_leg(flags, reps, warmup):
        points = M.ManyPoints(sweep_points())       # marshalled once: the call is timed, not the dict conversion
        for _ in range(warmup):
            M.mmee_search_many(points, flags)
        t1 = time.perf_counter()
        for _ in range(reps):
            results, codes = M.mmee_search_many(points, flags)
        dt = (time.perf_counter() - t1) / reps
        # neighbouring entries (the two objectives of a problem) share one pass
        costed = sum(r.evaluated for r in results[::2])
        return {"searches": points.n, "problems": points.n // 2, "ms": dt * 1e3,
                "ms_inside_library": results[0].seconds * 1e3, "candidates_costed": costed,
                "candidates_per_s": costed / dt, "infeasible": sum(1 for c in codes if c != 0)}, results

    if args.profile_only:
        # the timed steps of one leg only, for rocprofv3, then a plain copy of known size (1 GiB read,
        # 1 GiB written) as the reference reading of the FETCH_SIZE / WRITE_SIZE counters
        if args.profile_leg == "long":
            timed_search(CONFIGS["long"], [M.OBJ_ENERGY], M.SEARCH_EXHAUSTIVE, args.steps, args.warmup)
        elif args.profile_leg == "bert":
            timed_search(CONFIGS["bert"], [M.OBJ_ENERGY, M.OBJ_LATENCY], M.SEARCH_EXHAUSTIVE, args.steps, args.warmup)
        elif args.profile_leg == "sweep":
            sweep_leg(M.SEARCH_PRUNED, max(1, args.steps), args.warmup)
        else:
            cfg = CONFIGS["bert"]
            buf = torch.empty((1 << 26) * 8, dtype=torch.int64, device="cuda")
            for _ in range(args.warmup + args.steps):
                M.mmee_eval_batch(cfg["workload"], cfg["hw"], 1_000_000_007, 1 << 26, out=buf.data_ptr())
            del buf
        src = torch.zeros(1 << 27, dtype=torch.int64, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"profile_leg": args.profile_leg}))
        return

    # ---- headline: the largest single-GPU configuration, exhaustive, its own objective ----
    cfg = CONFIGS["long"]
    objectives = [M.OBJ_ENERGY]
    # beyond the size bound of the a-priori proof the search still starts regrouped and checks the outcome
    whole = all(float(cfg["hw"][k]).is_integer() for k in ("e_dram", "e_gb", "e_rf", "e_mac"))
    regrouped = M.mmee_energy_regrouped(cfg["workload"], cfg["hw"], M.SEARCH_EXHAUSTIVE) or whole
    ops = OPS_DENSE_ENERGY[regrouped]
    step_s, kernel_s, stream_s, res = timed_search(cfg, objectives, M.SEARCH_EXHAUSTIVE, args.steps, args.warmup)
    evaluated = res[0].evaluated
    traffic, traffic_src = traffic_of("k_search_dense_long")
    out = {
        "metric": "candidate mappings evaluated/sec (every dataflow costed, energy-driven optimum)",
        "value": evaluated / step_s, "unit": "candidates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": step_s * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": "long: " + describe(cfg), "space": res[0].space, "candidates_costed_per_step": evaluated,
                   "objectives": ["energy"], "search": "exhaustive"},
        "best": {"energy": {"idx": res[0].best.idx, "energy_pj": res[0].cost.energy_pj,
                            "latency_cycles": res[0].cost.latency_cycles}},
        "search_kernel_ms": kernel_s * 1e3, "stream_ms_per_step": stream_s * 1e3,
        "roofline": {"bound": "alu", "achieved": ops * evaluated / kernel_s / 1e12, "peak": ALU_PEAK_TOPS,
                     "unit": "Tlane-op/s", "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": "k_search_dense<energy%s>" % (", regrouped energy sum" if regrouped else ""),
                     "ops_per_candidate": ops, "kernel_candidates_per_s": evaluated / kernel_s},
    }
    out["roofline"]["frac"] = out["roofline"]["achieved"] / out["roofline"]["peak"]

    if not args.profile_only:
        # the BERT-like configuration, its two objectives in one pass (k_search, lane = row)
        bert = CONFIGS["bert"]
        two = [M.OBJ_ENERGY, M.OBJ_LATENCY]
        legs = {}
        for name, flags in (("regrouped", M.SEARCH_EXHAUSTIVE), ("ordered_sum", M.SEARCH_EXHAUSTIVE | M.SEARCH_ORDERED_SUM)):
            s_, k_, _, r_ = timed_search(bert, two, flags, 50, 5)
            reg = name == "regrouped" and M.mmee_energy_regrouped(bert["workload"], bert["hw"], flags)
            ach = OPS_TWO_KEYS[reg] * r_[0].evaluated / k_ / 1e12
            legs[name] = {"value": r_[0].evaluated / s_, "unit": "candidates/s", "ms_per_step": s_ * 1e3,
                          "search_kernel_ms": k_ * 1e3, "candidates_costed_per_step": r_[0].evaluated,
                          "roofline": {"bound": "alu", "achieved": ach, "peak": ALU_PEAK_TOPS, "unit": "Tlane-op/s",
                                       "frac": ach / ALU_PEAK_TOPS, "ops_per_candidate": OPS_TWO_KEYS[reg],
                                       "kernel": "k_search<energy+latency%s>" % (", regrouped energy sum" if reg else "")}}
        t_, src_ = traffic_of("k_search_bert")
        legs["regrouped"]["roofline"].update(traffic=t_, traffic_source=src_)
        out["bert"] = {"workload": "bert: " + describe(bert), **legs}

        # the hardware sweep: 64 accelerators x 8 workloads x 2 objectives through mmee_search_many,
        # one launch stream, one synchronisation
        pruned_leg, pruned_res = sweep_leg(M.SEARCH_PRUNED, 5, 2)
        full_leg, full_res = sweep_leg(M.SEARCH_EXHAUSTIVE, 2, 1)
        assert [r.best.idx for r in pruned_res] == [r.best.idx for r in full_res]
        out["sweep"] = {"pruned": pruned_leg, "exhaustive": full_leg, "pruned_equals_exhaustive": True}

        # time-to-optimum of the paper's method (pruned rows), host wall time per call
        tto = {}
        for name, c in CONFIGS.items():
            objs = c["objectives"]
            dt_p, _, _, r = timed_search(c, objs, M.SEARCH_PRUNED, 50, 5)
            dt_x, kx, _, rx = timed_search(c, objs, M.SEARCH_EXHAUSTIVE, 10, 2)
            assert [a.best.idx for a in r] == [a.best.idx for a in rx]
            tto[name] = {"pruned_ms": dt_p * 1e3, "pruned_candidates": r[0].evaluated,
                         "exhaustive_ms": dt_x * 1e3, "exhaustive_candidates": rx[0].evaluated,
                         "exhaustive_kernel_ms": kx * 1e3,
                         "exhaustive_candidates_per_s": rx[0].evaluated / dt_x}
        out["time_to_optimum"] = tto

        # the rows built beyond the core path, timed the same way (host wall time per call)
        def wall(fn, reps, warm=2):
            for _ in range(warm):
                fn()
            t1 = time.perf_counter()
            for _ in range(reps):
                r = fn()
            return (time.perf_counter() - t1) / reps, r
        beyond = {}
        # free two-GEMM / convolution-chain shapes (Sec. VII-J, Table V), energy key
        chains = {}
        for name, c in CHAINS.items():
            dt_p, rp = wall(lambda: M.mmee_chain_search_multi(c["workload"], c["hw"], [M.OBJ_ENERGY], M.SEARCH_PRUNED), 20)
            dt_x, rx = wall(lambda: M.mmee_chain_search_multi(c["workload"], c["hw"], [M.OBJ_ENERGY], M.SEARCH_EXHAUSTIVE), 5)
            assert rp[0].best.idx == rx[0].best.idx
            chains[name] = {"pruned_ms": dt_p * 1e3, "exhaustive_ms": dt_x * 1e3, "exhaustive_candidates": rx[0].evaluated,
                            "exhaustive_candidates_per_s": rx[0].evaluated / dt_x}
        beyond["chains_energy"] = chains
        # both fronts of bert (Sec. VII-E, VII-C): one pass per front point
        for key, fn in (("front_energy_latency", M.mmee_pareto), ("front_bs_da", M.mmee_front_bs_da)):
            dt_p, (code_p, pts_p) = wall(lambda: fn(bert["workload"], bert["hw"], M.SEARCH_PRUNED), 5)
            dt_x, (code_x, pts_x) = wall(lambda: fn(bert["workload"], bert["hw"], M.SEARCH_EXHAUSTIVE), 2, 1)
            assert code_p == 0 and code_x == 0 and [r.best.idx for r in pts_p] == [r.best.idx for r in pts_x]
            beyond[key] = {"points": len(pts_p), "pruned_ms": dt_p * 1e3, "exhaustive_ms": dt_x * 1e3}
        # the energy-delay product (Sec. VII-K) on bert
        dt_p, rp = wall(lambda: M.mmee_search_multi(bert["workload"], bert["hw"], [M.OBJ_EDP], M.SEARCH_PRUNED), 20)
        dt_x, rx = wall(lambda: M.mmee_search_multi(bert["workload"], bert["hw"], [M.OBJ_EDP], M.SEARCH_EXHAUSTIVE), 10)
        assert rp[0].best.idx == rx[0].best.idx
        beyond["edp_bert"] = {"pruned_ms": dt_p * 1e3, "exhaustive_ms": dt_x * 1e3,
                              "exhaustive_candidates_per_s": rx[0].evaluated / dt_x}
        out["beyond_the_core_path"] = beyond
        out["offline_stage"] = {"ms_first_call": offline_ms, "rows_valid": list(stats.rows_valid),
                                "rows_kept": list(stats.rows_kept)}

        # per-candidate records: HBM-write bound, 64 bytes each
        w, h = M.workload(bert["workload"]), M.hw(bert["hw"])
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
        t_, src_ = traffic_of("k_eval_batch")
        out["roofline_eval_batch"] = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": gbs / HBM_PEAK_GBS, "traffic": t_, "traffic_source": src_,
                                      "kernel": "k_eval_batch", "records": n_rec, "ms": eval_ms,
                                      "candidates_per_s": n_rec / (eval_ms * 1e-3)}
        del buf

    if not args.no_cpu_baseline and not args.profile_only:
        import oracle as O
        ow, oh = O.workload(cfg["workload"]), O.hw(cfg["hw"])
        t1 = time.perf_counter()
        rc, idx, cost, n_valid, threads = O.search_all(ow, oh)
        dt = time.perf_counter() - t1
        assert rc == 0 and idx[0] == res[0].best.idx, "GPU and oracle disagree"
        assert cost[0].energy_pj == res[0].cost.energy_pj and cost[0].latency_cycles == res[0].cost.latency_cycles
        out["cpu_baseline"] = {"value": evaluated / dt, "unit": "candidates/s", "cores": threads,
                               "host_cpus": os.cpu_count(), "kind": "oracle",
                               "sample": "the whole long space: all %d indices enumerated once, four objectives "
                                         "kept, %d of them denote a dataflow and are costed" % (res[0].space, evaluated),
                               "seconds": dt, "optimum_matches_gpu": True}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
