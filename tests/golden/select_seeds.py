"""Re-derive the workload seeds in paper_2407_03583_amd/workloads.py (SEEDS).

Rule: for each benchmark configuration c, the smallest seed >= 1000*c for which
the CPU checker finds at least one feasible candidate (single demand point) or
at least a quarter of the demand points feasible (sweeps).  Calls only the
generator and oracle/.  Usage:  python tests/golden/select_seeds.py [cfg ...]

Shortcuts that keep this affordable, none of which changes the outcome:
* a seed whose per-task capacity ceiling (every replica of every variant at its
  best batch size) is below the task's demand cannot be feasible and is
  skipped before the checker runs;
* feasibility is monotone non-increasing in demand, so for sweeps the number
  of feasible demand points is found by bisection over the sorted demands;
* when the worker budget can never bind (sum of all replica limits <= S) a
  feasible candidate exists iff per-task choices exist that serve the demand
  and keep every root-to-leaf latency sum within its budget; the per-task
  quantities are read from the checker's per-candidate evaluation.
"""
from __future__ import annotations

import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2407_03583_amd import workloads as wl  # noqa: E402


def ceiling_ok(w: wl.Workload, demand: int) -> bool:
    p = w.pipeline
    dn, sc = [demand], [1]
    for i in range(1, p.n_tasks):
        dn.append(dn[p.parent[i]] * p.fanout_q4[i])
        sc.append(sc[p.parent[i]] * 4)
    t = v = 0
    for i in range(p.n_tasks):
        k_i, nb = p.n_variants[i], p.n_batches[i]
        cap = sum(p.max_replicas[v + k] * max(p.thr_mqps[t + k * nb: t + (k + 1) * nb]) * sc[i]
                  for k in range(k_i))
        if cap < dn[i]:
            return False
        t += k_i * nb
        v += k_i
    return True


def exists_feasible_unbudgeted(w: wl.Workload, prob: oracle.Problem, demand: int) -> bool:
    """Exact when sum of replica limits <= workers."""
    p = w.pipeline
    assert sum(p.max_replicas) <= w.workers
    choices = p.choices_per_task()
    stride, lats, v = 1, [], 0
    for i in range(p.n_tasks):
        replica_combos = 1
        for k in range(p.n_variants[i]):
            replica_combos *= p.max_replicas[v + k] + 1
        v += p.n_variants[i]
        ok = set()
        for c in range(choices[i]):
            if c % replica_combos == 0:
                continue  # hosts nothing
            e = prob.eval(c * stride, demand, w.workers, w.slo_us, w.comm_us)
            if e.task_unserved[i] == 0:
                ok.add(int(e.task_maxlat[i]))
        if not ok:
            return False
        lats.append(min(ok))
        stride *= choices[i]
    leaves = [i for i in range(p.n_tasks) if i not in p.parent]
    for leaf in leaves:
        total, length, i = 0, 0, leaf
        while i >= 0:
            total += lats[i]
            length += 1
            i = p.parent[i]
        room = w.slo_us - w.comm_us * length
        if room < 0 or total > room // 2:
            return False
    return True


def feasible_points(w: wl.Workload, prob: oracle.Problem) -> int:
    """Number of feasible demand points, by bisection over the sorted demands."""
    ds = sorted(w.demand_mqps)

    def feas(d):
        if not ceiling_ok(w, d):
            return False
        return prob.search_tabulated(d, w.workers, w.slo_us, w.comm_us).found == 1

    lo, hi = 0, len(ds)  # ds[:lo] feasible, ds[hi:] infeasible
    while lo < hi:
        mid = (lo + hi) // 2
        if feas(ds[mid]):
            lo = mid + 1
        else:
            hi = mid
    return lo


def select(cfg: int, limit: int = 10_000_000) -> int:
    for seed in range(1000 * cfg, 1000 * cfg + limit):
        w = wl.config(cfg, seed)
        if len(w.demand_mqps) == 1:
            d = w.demand_mqps[0]
            if not ceiling_ok(w, d):
                continue
            prob = oracle.Problem(w.pipeline)
            if sum(w.pipeline.max_replicas) <= w.workers:
                good = exists_feasible_unbudgeted(w, prob, d)
            else:
                good = prob.search_tabulated(d, w.workers, w.slo_us, w.comm_us).found == 1
            if good:
                return seed
        else:
            need = (len(w.demand_mqps) + 3) // 4
            if not ceiling_ok(w, sorted(w.demand_mqps)[need - 1]):
                continue
            prob = oracle.Problem(w.pipeline)
            if feasible_points(w, prob) >= need:
                return seed
    raise RuntimeError("no seed found")


if __name__ == "__main__":
    cfgs = [int(a) for a in sys.argv[1:]] or [1, 2, 3, 4, 5]
    for c in cfgs:
        print(f"config {c}: seed {select(c)} (in workloads.py: {wl.SEEDS[c]})", flush=True)
