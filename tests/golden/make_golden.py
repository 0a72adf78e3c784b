"""Write tests/golden/cfg<N>.json: full-space search results of the benchmark
configurations, computed by the CPU checker only.  Every file says in `written_by`
which of the checker's two searches produced it:
  --plain   oracle.Problem.search: lo_eval on every index, the definition itself
            (configs 1 and 2: seconds to a minute on 8 cores);
  default   oracle.Problem.search_tabulated: the same two functions composed through a
            per-task table while an odometer walks the indices -- what makes 2^38 .. 2^40
            evaluations affordable (configs 3 - 5).  tests/test_oracle_pins.py checks it
            against the plain search in full on small problems and on slices of every
            config, and tests/test_oracle_pins.py::test_config5_golden_from_single_plan_
            evaluations re-derives config 5's stored result from lo_eval alone.

Usage: python tests/golden/make_golden.py [--threads T] [--plain] cfg [cfg ...]
Runtime on 8 cores: cfg 1-2 seconds (--plain: cfg 2 about half a minute), cfg 3 about
3 minutes, cfg 4 about 25 minutes, cfg 5 about 1.6 hours (5,829 s measured).

       python tests/golden/make_golden.py --variants
writes tests/golden/variants.json: the optional parts of the model on the 2^30-plan
configurations (per-variant factors on config 2's chain and config 4's tree, profiled
path accuracies on config 2, both together on config 2), each by the plain per-index
search; about 4 minutes.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2407_03583_amd import workloads as wl  # noqa: E402

# demand points also searched under the index-only tie rule
INDEX_ONLY_POINTS = {1: 1, 2: 1, 3: 64, 4: 8, 5: 0}


def record(b, demand):
    return dict(demand_mqps=int(demand), found=int(b.found), index=int(b.index),
                accuracy_hex=float(b.accuracy).hex(), accuracy=float(b.accuracy),
                workers=int(b.workers), n_feasible=int(b.n_feasible))


def factors_rising_with_accuracy(p):
    """Per-variant multiplicative factors 0.75 .. 1.5, larger for more accurate variants (Section 4.2)."""
    return [3 + (a - 600000) // 90000 for a in p.acc_ppm]


VARIANT_CASES = [  # name, config, what to add, demand points (milli-QPS; None: the configuration's first)
    ("cfg2_variant_factors", 2, "variant_factors", [50_000, 150_000, 400_000]),
    ("cfg4_variant_factors", 4, "variant_factors", [150_000, 600_000]),
    ("cfg2_path_tables", 2, "path_tables", None),
    ("cfg2_factors_and_path_tables", 2, "both", [150_000, 400_000]),
    ("cfg4_path_tables", 4, "path_tables", [150_000, 600_000]),
    ("cfg4_factors_and_path_tables", 4, "both", [600_000]),
]


def variants(threads):
    doc = dict(written_by="tests/golden/make_golden.py --variants (oracle.Problem.search, every index)", cases={})
    for name, cfg, what, demands in VARIANT_CASES:
        w = wl.config(cfg)
        p = w.pipeline
        if what in ("variant_factors", "both"):
            p.variant_factor_q4 = factors_rising_with_accuracy(p)
        if what in ("path_tables", "both"):
            p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(w.seed + 1))
        prob = oracle.Problem(p)
        t0 = time.time()
        results = []
        for d in demands or w.demand_mqps[:1]:
            results.append(record(prob.search(d, w.workers, w.slo_us, w.comm_us, threads=threads), d))
            print(f"{name} demand {d} {time.time() - t0:.0f}s", flush=True)
        doc["cases"][name] = dict(config=cfg, what=what, workload_digest=w.digest(), n_candidates=prob.num_candidates(),
                                  workers=w.workers, slo_us=w.slo_us, comm_us=w.comm_us, results=results,
                                  seconds=round(time.time() - t0, 1))
    with open(os.path.join(HERE, "variants.json"), "w") as f:
        json.dump(doc, f, indent=1)
        f.write("\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--threads", type=int, default=None)
    ap.add_argument("--variants", action="store_true")
    ap.add_argument("--plain", action="store_true", help="lo_eval on every index instead of the tabulated walk")
    ap.add_argument("cfgs", type=int, nargs="*")
    args = ap.parse_args()
    if args.variants:
        variants(args.threads)
    for cfg in args.cfgs:
        w = wl.config(cfg)
        prob = oracle.Problem(w.pipeline)
        search = prob.search if args.plain else prob.search_tabulated
        doc = dict(config=cfg, name=w.name, seed=w.seed, workload_digest=w.digest(),
                   n_candidates=prob.num_candidates(), workers=w.workers, slo_us=w.slo_us, comm_us=w.comm_us,
                   written_by="tests/golden/make_golden.py --plain (oracle.Problem.search: lo_eval on every index)"
                   if args.plain else "tests/golden/make_golden.py (oracle.Problem.search_tabulated)",
                   results=[], results_index_only=[])
        t0 = time.time()
        for m, d in enumerate(w.demand_mqps):
            b = search(d, w.workers, w.slo_us, w.comm_us, threads=args.threads)
            doc["results"].append(record(b, d))
            if m < INDEX_ONLY_POINTS[cfg]:
                b = search(d, w.workers, w.slo_us, w.comm_us, tie_index_only=True,
                           threads=args.threads)
                doc["results_index_only"].append(record(b, d))
            print(f"cfg {cfg} point {m + 1}/{len(w.demand_mqps)} {time.time() - t0:.0f}s", flush=True)
        doc["seconds"] = round(time.time() - t0, 1)
        doc["threads"] = args.threads or oracle.max_threads()
        with open(os.path.join(HERE, f"cfg{cfg}.json"), "w") as f:
            json.dump(doc, f, indent=1)
            f.write("\n")


if __name__ == "__main__":
    main()
