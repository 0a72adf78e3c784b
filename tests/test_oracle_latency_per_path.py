"""Pins for the CPU checker's eq. (7) as the paper states it: the latency of every variant path with
traffic (Table 1's I(p)), against a hand-derived example, an exact-rational second implementation that
finds the paths with traffic from interval overlaps, relations to the per-task bound, and the paper's
own formulation as a linear program over the path ratios.  No GPU."""
import copy
import json
import os
import random
from fractions import Fraction
from types import SimpleNamespace

import numpy as np
import pytest
from scipy.optimize import linprog

import oracle
import pyref
from paper_2407_03583_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
LAT = oracle.BAD_LATENCY


def with_rule(p, per_path):
    q = copy.copy(p)
    q.latency_per_path = bool(per_path)
    return q


def split_traffic_problem(rng, parent, monotone=False):
    """Replicas that serve 30 - 70 % of their task's demand each (up to two per variant on two tasks, one on
    longer trees: 81 to 4,096 plans), so that plans split traffic over several variants; latencies independent
    of accuracy (monotone: growing with it)."""
    n = len(parent)
    replicas = 2 if n == 2 else 1
    demand = rng.randint(60_000, 200_000)
    p = wl.Pipeline(n_tasks=n, parent=parent, fanout_q4=[4] + [rng.randint(3, 8) for _ in range(n - 1)],
                    n_variants=[], n_batches=[], batch_size=[], max_replicas=[], acc_ppm=[], latency_us=[], thr_mqps=[])
    level = [demand]
    for i in range(1, n):
        level.append(level[parent[i]] * p.fanout_q4[i] // 4)
    for i in range(n):
        k = rng.randint(2, 3)
        p.n_variants.append(k)
        p.n_batches.append(1)
        p.batch_size.append(1)
        accs, lats = rng.sample(range(600, 951), k), rng.sample(range(4, 40), k)
        if monotone:
            accs.sort()
            lats.sort()
        for a, l in zip(accs, lats):
            p.max_replicas.append(replicas)
            p.acc_ppm.append(a * 1000)
            p.latency_us.append(l * 1000)
            p.thr_mqps.append(level[i] * rng.randint(30, 70) // (100 if replicas == 2 else 70))
    slowest = max(sum(max(p.latency_us[sum(p.n_variants[:i]):sum(p.n_variants[:i + 1])]) for i in path)
                  for path in p.leaf_paths())
    return p, demand, [slowest * 2 * 7 // 10, slowest * 2 * 85 // 100]


def test_hand_example():
    with open(os.path.join(HERE, "golden", "latency_per_path_example.json")) as f:
        doc = json.load(f)
    names = [["B", "A"], ["D", "C"]]
    for case in doc["cases"]:
        p = SimpleNamespace(**dict(doc["pipeline"], thr_mqps=case["thr_mqps"]))
        for per_path, key in ((False, "per_task_infeasible"), (True, "per_path_infeasible")):
            q = with_rule(p, per_path)
            e = oracle.Problem(q).eval(doc["plan_index"], case["demand_mqps"], doc["workers"], case["slo_us"])
            assert e.infeasible == case[key], (case["what"], per_path)
            if not e.infeasible:
                a = [float(Fraction(*f)) for f in case["task_acc"]]
                assert e.accuracy == (a[0] * a[1]) / 1.0, case["what"]
        found = pyref.variant_paths_with_traffic(with_rule(p, True), doc["plan_index"], case["demand_mqps"])
        assert len(found) == 1 and found[0][0] == [0, 1]
        assert sorted(names[0][a] + names[1][b] for a, b in found[0][1]) == case["traffic_paths"], case["what"]


@pytest.mark.parametrize("seed", range(8))
def test_every_plan_matches_the_interval_reading(seed):
    """Every plan of a small problem under both rules against tests/pyref.py, where the per-path rule
    cuts the request streams into intervals instead of replaying the routing."""
    rng = random.Random(1000 + seed)
    parent = [[-1, 0], [-1, 0, 1], [-1, 0, 0], [-1, 0, 1, 1]][seed % 4]
    p, demand, slos = split_traffic_problem(rng, parent)
    for slo in slos[:1]:
        for per_path in (False, True):
            q = with_rule(p, per_path)
            O = oracle.Problem(q)
            for idx in range(O.num_candidates()):
                e = O.eval(idx, demand, 99, slo)
                r = pyref.evaluate(q, idx, demand, 99, slo)
                assert e.infeasible == r["infeasible"], (idx, slo, per_path)
                if not e.infeasible:
                    assert e.accuracy == r["accuracy"], (idx, slo, per_path)


def test_the_two_rules_differ_on_these_problems():
    """The comparison above is not vacuous: on a good share of the problems the per-path rule admits plans
    the per-task bound rejects (and never the other way round)."""
    differ = total = 0
    for seed in range(40):
        rng = random.Random(1000 + seed)
        p, demand, slos = split_traffic_problem(rng, [[-1, 0], [-1, 0, 1], [-1, 0, 0], [-1, 0, 1, 1]][seed % 4])
        for slo in slos:
            a = oracle.Problem(with_rule(p, False)).search(demand, 99, slo)
            b = oracle.Problem(with_rule(p, True)).search(demand, 99, slo)
            assert b.n_feasible >= a.n_feasible
            if a.found:
                assert b.found and b.accuracy >= a.accuracy
            differ += b.n_feasible > a.n_feasible
            total += 1
    assert differ >= total // 5, (differ, total)


def test_rules_agree_where_latency_grows_with_accuracy():
    """Most-accurate-first pairs the most accurate variants in use of consecutive tasks (the first requests
    of the stream go to both), so where a task's latency grows with its accuracy the slowest in-use variants
    share a path with traffic and the per-task bound is exact."""
    for seed in range(30):
        rng = random.Random(2000 + seed)
        p, demand, slos = split_traffic_problem(rng, [[-1, 0], [-1, 0, 1], [-1, 0, 0]][seed % 3], monotone=True)
        for slo in slos:
            a = oracle.Problem(with_rule(p, False)).search(demand, 99, slo)
            b = oracle.Problem(with_rule(p, True)).search(demand, 99, slo)
            assert a.as_tuple() == b.as_tuple(), (seed, slo)


def test_first_and_last_variants_in_use_always_share_a_path():
    """When all demand is served, the head of every task's request stream goes from the first variant in use
    of a task (route order) to the first one of its child, and the tail from the last to the last: both
    variant paths carry requests whatever the capacities, so their latency bounds the per-path rule from
    below, as the per-task sum bounds it from above.  Checked on the checker's routing tables."""
    seen = gap = 0
    for seed in range(12):
        rng = random.Random(1000 + seed)
        parent = [[-1, 0], [-1, 0, 1], [-1, 0, 0], [-1, 0, 1, 1]][seed % 4]
        p, demand, slos = split_traffic_problem(rng, parent)
        O = oracle.Problem(with_rule(p, True))
        voff = [sum(p.n_variants[:i]) for i in range(p.n_tasks)]
        for idx in range(O.num_candidates()):
            r = O.route_table(idx, demand)
            x, _ = O.decode(idx)
            if any(r.unserved[i] > 0 or not any(x[voff[i]:voff[i] + p.n_variants[i]]) for i in range(p.n_tasks)):
                continue
            order = [sorted(range(p.n_variants[i]), key=lambda k: (-p.acc_ppm[voff[i] + k], k)) for i in range(p.n_tasks)]
            used = [[k for k in order[i] if r.routed[i][k] > 0] for i in range(p.n_tasks)]
            for pick in (0, -1):
                for i in range(1, p.n_tasks):
                    up, down = used[parent[i]][pick], used[i][pick]
                    assert r.prob[i][up][down] > 0.0, (seed, idx, i, pick)
                assert r.prob[0][0][used[0][pick]] > 0.0
            # and the bounds: lower <= worst path with traffic <= upper, the budget placed on each in turn
            lat = [[p.latency_us[voff[i] + k] for k in range(p.n_variants[i])] for i in range(p.n_tasks)]
            for path in p.leaf_paths():
                low = max(sum(lat[i][used[i][pick]] for i in path) for pick in (0, -1))
                high = sum(max(lat[i][k] for k in used[i]) for i in path)
                assert low <= high
                gap += low < high
            seen += 1
            e_low = O.eval(idx, demand, 99, 2 * max(max(sum(lat[i][used[i][pick]] for i in path) for pick in (0, -1))
                                                    for path in p.leaf_paths()) - 1)
            assert e_low.infeasible & LAT, (seed, idx)
    assert seen > 500 and gap > 100, (seen, gap)


def test_one_variant_in_use_per_task_makes_the_rules_agree():
    """With a single variant per task there is one variant path, and both rules are its latency."""
    for seed in range(10):
        w = wl.random_small(seed, max_tasks=4, max_variants=1, max_replicas=3, max_candidates=5000)
        for slo in (w.slo_us, w.slo_us // 2, w.slo_us // 4):
            a = oracle.Problem(with_rule(w.pipeline, False)).search(w.demand_mqps[0], w.workers, slo, w.comm_us)
            b = oracle.Problem(with_rule(w.pipeline, True)).search(w.demand_mqps[0], w.workers, slo, w.comm_us)
            assert a.as_tuple() == b.as_tuple()


def test_search_and_range_split_under_the_per_path_rule():
    rng = random.Random(7)
    p, demand, slos = split_traffic_problem(rng, [-1, 0, 1])
    O = oracle.Problem(with_rule(p, True))
    n = O.num_candidates()
    whole = O.search(demand, 99, slos[0])
    tab = O.search_tabulated(demand, 99, slos[0])      # falls back to the plain search under this rule
    assert whole.as_tuple() == tab.as_tuple()
    cut = n // 3 + 5
    lo, hi = O.search(demand, 99, slos[0], end=cut), O.search(demand, 99, slos[0], begin=cut)
    assert lo.n_feasible + hi.n_feasible == whole.n_feasible
    count = sum(1 for idx in range(n) if not O.eval(idx, demand, 99, slos[0]).infeasible)
    assert count == whole.n_feasible


# ---- the paper's formulation for a fixed allocation: a linear program over the path ratios ---------

def lp_with_slow_paths_closed(p, demand, xs, budget):
    """Two-task chain.  Variables c(k0, k1) >= 0, sum 1 (every request takes a variant path); capacity of
    every variant (eq. (2)); a path slower than the budget must carry nothing (eq. (7): I(p) = 0).
    Returns the largest sum c(p) * A(k0) * A(k1), or None when no routing satisfies the constraints."""
    K0, K1 = p.n_variants
    fan = Fraction(p.fanout_q4[1], 4)
    nvar = K0 * K1
    cost = np.zeros(nvar)
    bounds = []
    for k0 in range(K0):
        for k1 in range(K1):
            v = k0 * K1 + k1
            cost[v] = -(p.acc_ppm[k0] / 1e6) * (p.acc_ppm[K0 + k1] / 1e6)
            slow = p.latency_us[k0] + p.latency_us[K0 + k1] > budget
            bounds.append((0, 0) if slow else (0, None))
    A_ub, b_ub = [], []
    for k0 in range(K0):
        row = np.zeros(nvar)
        row[k0 * K1:(k0 + 1) * K1] = 1.0
        A_ub.append(row)
        b_ub.append(xs[0][k0] * p.thr_mqps[k0] / demand)
    for k1 in range(K1):
        row = np.zeros(nvar)
        row[k1::K1] = 1.0
        A_ub.append(row)
        b_ub.append(xs[1][k1] * p.thr_mqps[K0 + k1] / float(demand * fan))
    r = linprog(cost, A_ub=np.array(A_ub), b_ub=np.array(b_ub), A_eq=np.ones((1, nvar)), b_eq=[1.0], bounds=bounds,
                method="highs", options={"primal_feasibility_tolerance": 1e-10, "dual_feasibility_tolerance": 1e-10})
    return -r.fun if r.status == 0 else None


def test_feasible_plans_are_feasible_in_the_papers_formulation():
    """For a fixed allocation of a two-task chain the paper's constraints on the path ratios are linear.
    A plan the checker accepts under the per-path rule comes with a routing (Algorithm 1's) that satisfies
    them, so the program must be feasible and its optimum at least the checker's accuracy; a plan for which
    no routing at all satisfies them must be rejected by the checker.  The per-task bound, being an upper
    bound on every path's latency, must reject whatever the program rejects too."""
    accepted = rejected_by_lp = only_per_path = 0
    for seed in range(12):
        rng = random.Random(3000 + seed)
        p, demand, slos = split_traffic_problem(rng, [-1, 0])
        O1, O0 = oracle.Problem(with_rule(p, True)), oracle.Problem(with_rule(p, False))
        for slo in slos:
            for idx in range(O1.num_candidates()):
                e1, e0 = O1.eval(idx, demand, 99, slo), O0.eval(idx, demand, 99, slo)
                if e1.infeasible & ~LAT:
                    continue
                x, _ = O1.decode(idx)
                xs = [x[:p.n_variants[0]], x[p.n_variants[0]:]]
                best = lp_with_slow_paths_closed(p, demand, xs, slo // 2)
                if best is None:
                    rejected_by_lp += 1
                    assert e1.infeasible & LAT and e0.infeasible & LAT, (seed, slo, idx)
                elif not e1.infeasible:
                    accepted += 1
                    assert best >= e1.accuracy - 1e-8, (seed, slo, idx, best, e1.accuracy)
                    only_per_path += bool(e0.infeasible)
    assert accepted > 500 and rejected_by_lp > 100 and only_per_path > 20, (accepted, rejected_by_lp, only_per_path)
