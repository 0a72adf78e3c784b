"""Benchmark: candidates evaluated per second of the exhaustive allocation search on one MI355X.

A step is one pass of the whole hot path (per-task tables, the kernel that visits
every plan, the final merge) over one benchmark configuration; inputs are resident
in device memory except the O(KB) constant block each call stages itself.
Prints one JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz = one 32- or 64-bit vector ALU
# operation per lane per clock (fp64 FMA counted as two gives the published 78.6 TFLOP/s).
VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def algorithmic_lane_ops(n_tasks: int, n_paths: int, per_lane: bool, pipeline) -> float:
    """Vector-ALU operations (one lane, one 32- or 64-bit operation) a plan needs in the
    kernel that visits every plan.

    Tabulated kernel: one fp64 multiply (prefix product times the last task's accuracy), one
    fp64 add (the other paths' sum) when the tree has several leaves, and one fp64 max/compare
    against the lane's best.  The two feasibility compares of eq. (3) and eq. (7) are taken
    once per run of first-task choices with equal replicas and latency and are not counted.
    Per-lane kernel: the last task is scored per plan, and what that needs is counted, not what the kernel
    executes (about twice as much: table addresses, the step to the next choice level by level, mask
    bookkeeping) -- per variant 8: the replicas' byte, capacity `x * q`, `min` with the demand left, the
    subtraction, the multiply-add into the accuracy sum, the in-use test, max and select of the latency;
    per plan 12: next choice (2), sum of replicas, workers add and compare, latency add and compare, the
    unserved and empty tests, index and range test (3).  The fp64 division and the comparison with the
    best plan run for feasible plans only and are not counted.  The other tasks are scored once per strip
    of 64 plans (8 per variant + 32 with their division)."""
    if not per_lane:
        return (1 if n_tasks >= 2 else 0) + (1 if n_paths > 1 else 0) + 1
    ks = list(pipeline.n_variants)
    # (with profiled path accuracies the walk over the variant paths runs for feasible plans only and is
    # not counted)
    return 8 * ks[-1] + 12 + sum(8 * k + 32 for k in ks[:-1]) / 64.0


# HBM bytes per launch of the dominant kernel: rocprofv3 FETCH_SIZE + WRITE_SIZE per dispatch (KiB, scale
# factor 1.0 against a plain copy; profiles/combine_kernel_cfg5.md, profiles/per_lane_search_kernel_cfg5.md).
# They hold for the kernel sources they were taken with; with other sources `traffic` is null.
MEASURED_TRAFFIC_BYTES = {("cfg5_tree4_k4", "tabulated"): (2175 + 7216) * 1024,
                          ("cfg5_tree4_k4", "per_lane"): (4853 + 449660) * 1024}
TRAFFIC_SOURCES = ("loki_device.h", "loki_launch.h", "loki_kernels.hip", "loki_api.cpp")
TRAFFIC_SOURCES_SHA256 = "6bda9c9677b168721864393e01c5c06e6794650b56d34edc804f754cca2b17f7"


def measured_traffic(workload: str, kernel: str):
    if kernel_sources_digest() != TRAFFIC_SOURCES_SHA256:
        return None
    return MEASURED_TRAFFIC_BYTES.get((workload, kernel))


def kernel_sources_digest():
    """SHA-256 over the kernel and launch sources with comments and white space removed (a changed
    comment does not change the machine code the counters were taken with)."""
    import re
    h = hashlib.sha256()
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2407_03583_amd", "csrc")
    try:
        for f in TRAFFIC_SOURCES:
            with open(os.path.join(csrc, f), "r") as fh:
                text = fh.read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            text = re.sub(r"//[^\n]*", "", text)
            h.update("".join(text.split()).encode())
    except OSError:
        return None
    return h.hexdigest()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration 1..5 (default: the largest)")
    ap.add_argument("--per-lane", action="store_true", help="time the kernel that scores whole plans per lane")
    ap.add_argument("--variant-factors", action="store_true",
                    help="per-variant multiplicative factors r(i,k), 0.75 .. 1.5 rising with accuracy "
                         "(searched class by class by the tabulated kernels; with --per-lane whole plans per lane)")
    ap.add_argument("--per-variant-batch", action="store_true", help="a batch size per hosted variant")
    ap.add_argument("--path-tables", action="store_true",
                    help="objective from seeded profiled path accuracies (feasibility from the per-task tables; "
                         "one value per leaf on trees, a walk over the variant paths of feasible plans on chains)")
    ap.add_argument("--latency-per-path", action="store_true",
                    help="eq. (7) on every variant path with traffic instead of the per-task bound (tabulated, "
                         "with a second kernel for the plans only this rule admits; with --variant-factors or "
                         "--path-tables whole plans per lane)")
    ap.add_argument("--demand-qps", type=float, default=None,
                    help="replace the configuration's demand points by this one demand (queries/s)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the other configurations and the instruction-rate probes (profiling runs: "
                         "only the timed workload's kernels are launched)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (more GPUs would each take an index range); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch

    from paper_2407_03583_amd import binding, workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    w = wl.config(args.config)
    variant = []
    if args.variant_factors:
        w.pipeline.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in w.pipeline.acc_ppm]
        variant.append("variant_factors")
    if args.per_variant_batch:
        w.pipeline.per_variant_batch = True
        variant.append("per_variant_batch")
    if args.path_tables:
        w.pipeline.path_acc_ppm = wl.draw_path_tables(w.pipeline, wl.SplitMix64(w.seed + 1))
        variant.append("path_tables")
    if args.latency_per_path:
        w.pipeline.latency_per_path = True
        variant.append("latency_per_path")
    if args.demand_qps is not None:
        w.demand_mqps = [int(round(args.demand_qps * 1000))]
        variant.append(f"demand{args.demand_qps:g}qps")
    if variant:
        w.name += "+" + "+".join(variant)
    # what the library does anyway: per-variant factors are searched class by class by the tabulated kernels
    # (two or more tasks); profiled path accuracies with the feasibility part tabulated and the variant paths
    # walked for feasible plans only
    # (the per-path latency rule: on the tables with a second kernel for the plans only that rule admits, unless
    # per-variant factors or path tables are present as well, where the library scores whole plans per lane)
    args.per_lane = args.per_lane or (args.latency_per_path and (args.variant_factors or args.path_tables))
    by_class = args.variant_factors and w.pipeline.n_tasks >= 2 and not args.per_lane
    args.per_lane = args.per_lane or (args.variant_factors and not by_class)
    P = binding.Problem(w.pipeline)
    n = P.num_candidates()
    m = len(w.demand_mqps)
    flags = binding.LOKI_SEARCH_PER_LANE if args.per_lane else 0
    end = n
    if args.per_lane and n * m > (1 << 36):  # keep a step to seconds: a prefix of the index space
        end = (1 << 36) // m
    if not args.per_lane and n * m > (1 << 45):
        end = (1 << 45) // m
    evaluations = end * m

    results = torch.empty(32 * m, dtype=torch.uint8, device="cuda")
    for _ in range(args.warmup):
        P.alloc_search_enqueue(w.demand_mqps, w.workers, w.slo_us, w.comm_us, flags=flags, end=end, results=results)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        P.alloc_search_enqueue(w.demand_mqps, w.workers, w.slo_us, w.comm_us, flags=flags, end=end, results=results)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)
    ms_per_step = max(gpu_ms, wall_ms) / args.steps
    first = binding.results_from_bytes(results.cpu().numpy().tobytes())

    # duration of the dominant kernel alone (HIP events inside the library, on the same stream)
    kernel_ms = []
    for _ in range(max(1, min(args.steps, 5))):
        chk = P.alloc_search(w.demand_mqps, w.workers, w.slo_us, w.comm_us, flags=flags, end=end)
        kernel_ms.append(P.last_search_ms())
    assert [r.as_tuple() for r in chk] == [r.as_tuple() for r in first]
    main_ms = sum(k[1] for k in kernel_ms) / len(kernel_ms)
    n_paths = sum(1 for i in range(w.pipeline.n_tasks) if i not in w.pipeline.parent)
    ops = algorithmic_lane_ops(w.pipeline.n_tasks, n_paths, args.per_lane, w.pipeline)
    # profiled path accuracies on a tree with several leaves (at most 64 variant combinations above every
    # leaf): the library forms one value per leaf and the plans are combined as in the product form, with one
    # add and one max/compare per plan (the sums over the variant paths, one per tile entry and per lane slot,
    # are not counted)
    par = w.pipeline.parent
    above = [1] * w.pipeline.n_tasks   # variant combinations of the tasks above task i
    for i in range(1, w.pipeline.n_tasks):
        above[i] = above[par[i]] * w.pipeline.n_variants[par[i]]
    by_leaf = (args.path_tables and not args.per_lane and w.pipeline.n_tasks >= 3 and n_paths >= 2
               and max(above[i] for i in range(w.pipeline.n_tasks) if i not in par) <= 64)
    if by_leaf:
        ops = 2
    # profiled path accuracies on a single task path (at most 64 variant combinations above the last task): the
    # library bounds the objective of every feasible plan from above and walks the variant paths only of
    # those that can still reach the best seen; priced like the product form (what a search over these plans
    # costs at the least), the bound and the walks are overhead
    pruned = (args.path_tables and not args.per_lane and not args.variant_factors and n_paths == 1
              and above[w.pipeline.n_tasks - 1] <= 64)
    no_count = args.path_tables and not args.per_lane and not by_leaf and not pruned   # see the roofline note
    # work the kernels did: every plan of the range, except class by class, where plans whose first-task
    # choice cannot serve the demand are settled per choice on the host and never reach the kernels
    scored = P.last_search_plans_scored()
    achieved = None if no_count else ops * scored / (main_ms * 1e-3) / 1e12

    out = {
        "metric": "allocation candidates evaluated/sec (1 GPU)",
        # (class by class: the plans the kernels scored; plans settled per choice on the host are left out of
        # both this figure and the roofline fraction)
        "value": (scored if by_class else evaluations) / (ms_per_step * 1e-3),
        "unit": "candidates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int64+f64",
        "data": "synthetic",
        "config": {"workload": w.name, "seed": w.seed, "candidates": n, "demand_points": m,
                   "index_end": end, "evaluations_per_step": evaluations, "plans_scored_by_kernels": scored,
                   "kernel": ("per_lane_paths" if args.path_tables else "per_lane") if args.per_lane
                   else (("tabulated_by_class_paths" if args.path_tables else "tabulated_by_class") if by_class
                         else ("tabulated_paths" if args.path_tables else "tabulated")) + ("_by_leaf" if by_leaf else ""),
                   "feasible_fraction_point0": first[0].n_feasible / end},
        "kernel_ms": {"task_tables": sum(k[0] for k in kernel_ms) / len(kernel_ms), "search": main_ms,
                      "final_merge": sum(k[2] for k in kernel_ms) / len(kernel_ms)},
        "roofline": {"bound": "alu", "achieved": achieved, "peak": VALU_PEAK_TLANEOPS, "unit": "Tlane-op/s",
                     "frac": None if no_count else achieved / VALU_PEAK_TLANEOPS,
                     "traffic": measured_traffic(w.name, "per_lane" if args.per_lane else "tabulated"),
                     "lane_ops_per_candidate": None if no_count else ops},
    }
    if by_leaf:
        out["roofline"]["note"] = ("profiled path accuracies leaf by leaf: 2 operations per visited plan (add, "
                                   "max/compare); the sums over the variant paths, one per tile entry and per "
                                   "lane slot, are not counted")
    if pruned:
        out["roofline"]["note"] = ("profiled path accuracies on one task path: priced like the product form "
                                   f"({ops} operations per visited plan); the upper bound taken for every feasible "
                                   "plan and the walks over the variant paths of the plans it does not rule out "
                                   "are not counted")
    if no_count:
        out["roofline"]["note"] = ("profiled path accuracies: feasibility is taken per run of first-task choices "
                                   "and the walk over the variant paths runs for feasible plans only, so no "
                                   "per-plan operation count applies")
    # the other benchmark configurations and two dense demand points of this one (many feasible plans, many
    # ties at the top accuracy), a few timed blocking calls each: context for `value`, each with the roofline
    # fraction of its own search kernel priced like the headline one
    if not args.per_lane and not variant and not args.no_context:
        def context_entry(wc, demands):
            Pc = binding.Problem(wc.pipeline)
            Pc.alloc_search(demands, wc.workers, wc.slo_us, wc.comm_us)
            best_call, best_kernel = None, None
            for _ in range(3):
                t0 = time.perf_counter()
                rc = Pc.alloc_search(demands, wc.workers, wc.slo_us, wc.comm_us)
                dt = time.perf_counter() - t0
                km = Pc.last_search_ms()[1]
                best_call = dt if best_call is None else min(best_call, dt)
                best_kernel = km if best_kernel is None else min(best_kernel, km)
            ev = Pc.num_candidates() * len(demands)
            leaves = sum(1 for i in range(wc.pipeline.n_tasks) if i not in wc.pipeline.parent)
            ops_c = algorithmic_lane_ops(wc.pipeline.n_tasks, leaves, False, wc.pipeline)
            return {"evaluations": ev, "demand_points": len(demands), "ms_call": best_call * 1e3,
                    "ms_search_kernel": best_kernel, "candidates_per_s": ev / best_call,
                    "lane_ops_per_candidate": ops_c,
                    "frac": ops_c * ev / (best_kernel * 1e-3) / 1e12 / VALU_PEAK_TLANEOPS,
                    "feasible_points": sum(1 for r in rc if r.status == binding.LOKI_FOUND),
                    "feasible_fraction": sum(r.n_feasible for r in rc) / ev}
        others = {}
        for c in (1, 2, 3, 4, 5):
            if c == args.config:
                continue
            wc = wl.config(c)
            others[wc.name] = context_entry(wc, wc.demand_mqps)
        for qps in (300, 0):
            others[f"{w.name}+demand{qps}qps"] = context_entry(w, [qps * 1000])
        out["other_configs"] = others
    # what a dependency-free stream of the search's own instructions sustains on this GPU
    if not args.no_context:
        mix = binding.measure_valu_rate("search_mix")
        out["roofline"]["sustained_mix_Tlane_op_s"] = mix * 64 / 1e12
        out["roofline"]["frac_of_sustained_mix"] = None if no_count else achieved / (mix * 64 / 1e12)
        out["roofline"]["sustained_u32_Tlane_op_s"] = binding.measure_valu_rate("v_add_u32") * 64 / 1e12
    if not args.no_cpu_baseline:
        import oracle
        O = oracle.Problem(w.pipeline)
        sample = min(n, 1 << 30)
        stride = max(1, n // sample)
        if stride > 1 and stride % 2 == 0:
            stride -= 1  # odd stride: every digit of the index varies over the sample
        threads = oracle.max_threads()
        t0 = time.perf_counter()
        b = O.search(w.demand_mqps[0], w.workers, w.slo_us, w.comm_us, begin=0, end=min(n, sample * stride),
                     stride=stride, threads=threads)
        dt = time.perf_counter() - t0
        done = (min(n, sample * stride) + stride - 1) // stride
        t1 = time.perf_counter()
        one = min(done, 1 << 23)
        O.search(w.demand_mqps[0], w.workers, w.slo_us, w.comm_us, begin=0, end=one * stride, stride=stride, threads=1)
        single = one / (time.perf_counter() - t1)
        out["cpu_baseline"] = {"value": done / dt, "unit": "candidates/s", "cores": threads, "kind": "oracle",
                               "single_thread_value": single,
                               "sample": f"{done} candidates of demand point 0, every {stride}th index from 0, "
                                         f"plain per-index search, {dt:.1f} s",
                               "feasible_in_sample": int(b.n_feasible)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
