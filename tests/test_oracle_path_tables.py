"""Pins for the CPU checker's objective with profiled path accuracies, sum_p c(p) * A-hat(p)
(Section 4.1 "Accuracy"), c(p) from Algorithm 1's routing (Section 5.1).  None of these re-types the
checker's own walk: they use a hand-derived example, closed forms that follow from the definition
(marginals, constants, single-variant plans, the product form when nothing is coupled), and an
exact-rational second implementation that gets the flows from interval overlaps instead of
Algorithm 1's sequential bookkeeping."""
import json
import os
import random
from fractions import Fraction
from types import SimpleNamespace

import pytest

import oracle
import pyref
from paper_2407_03583_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TOL = 4e-16 * 40    # a few dozen roundings of values below 1


def load_example():
    g = json.load(open(os.path.join(GOLDEN, "path_table_example.json")))
    return g, SimpleNamespace(**g["pipeline"])


def test_hand_derived_example():
    g, p = load_example()
    O = oracle.Problem(p)
    idx = O.encode(g["plan_x"], [0, 0])
    e = O.eval(idx, g["demand_mqps"], g["workers"], g["slo_us"])
    assert e.infeasible == 0 and e.workers == 4
    num, den = g["objective_exact"]
    assert abs(Fraction(e.accuracy) - Fraction(num, den)) < TOL
    # the shares the derivation uses are the routing table's
    r = O.route_table(idx, g["demand_mqps"])
    assert abs(Fraction(r.prob[0][0][1]) * Fraction(r.prob[1][1][0]) - Fraction(*g["shares"]["AX"])) < TOL
    assert abs(Fraction(r.prob[0][0][1]) * Fraction(r.prob[1][1][1]) - Fraction(*g["shares"]["AY"])) < TOL
    assert abs(Fraction(r.prob[0][0][0]) * Fraction(r.prob[1][0][1]) - Fraction(*g["shares"]["BY"])) < TOL
    assert r.prob[1][0][0] == 0.0
    # and it differs from what the product of task accuracies would give
    p2 = SimpleNamespace(**{**g["pipeline"], "path_acc_ppm": None})
    assert abs(oracle.Problem(p2).eval(idx, g["demand_mqps"], g["workers"], g["slo_us"]).accuracy - 0.774) < 1e-12


def test_search_on_the_example_prefers_what_the_table_says():
    """With the table of the example, hosting only A and X cannot serve 100 QPS; the best plan is the
    one that maximises the table-weighted sum, which the exact reference finds too."""
    g, p = load_example()
    O = oracle.Problem(p)
    best = O.search(g["demand_mqps"], g["workers"], g["slo_us"])
    ref = pyref.search(p, g["demand_mqps"], g["workers"], g["slo_us"])
    assert best.found == 1 and best.index == ref["index"] and best.n_feasible == ref["n_feasible"]
    assert abs(best.accuracy - ref["accuracy"]) < TOL


def feasible_samples(w, O, limit=200):
    n = O.num_candidates()
    step = max(1, n // 400)
    out = []
    for idx in range(0, n, step):
        e = O.eval(idx, w.demand_mqps[0], w.workers, w.slo_us, w.comm_us)
        if not e.infeasible:
            out.append((idx, e))
            if len(out) >= limit:
                break
    return out


def tight_problem(rng, variant_factors=False, per_variant_batch=False):
    """A small tree in which one replica serves about a third of a task's demand, so that feasible
    plans spread every task's traffic over several variants (inputs only)."""
    n = rng.randint(2, 3)
    parent = [-1] + [rng.randint(0, i - 1) for i in range(1, n)]
    demand = rng.randint(60_000, 300_000)
    p = wl.Pipeline(n_tasks=n, parent=parent, fanout_q4=[4] + [rng.randint(2, 10) for _ in range(n - 1)],
                    n_variants=[], n_batches=[], batch_size=[], max_replicas=[], acc_ppm=[], latency_us=[],
                    thr_mqps=[], per_variant_batch=per_variant_batch)
    level = [demand]
    for i in range(1, n):
        level.append(level[parent[i]] * p.fanout_q4[i] // 4)
    for i in range(n):
        k_i = rng.randint(2, 3)
        batches = [1, 4] if per_variant_batch else [2]
        p.n_variants.append(k_i)
        p.n_batches.append(len(batches))
        p.batch_size.extend(batches)
        for _ in range(k_i):
            p.max_replicas.append(2)
            p.acc_ppm.append(rng.randint(60, 95) * 10000)
            per_replica = max(1000, level[i] * rng.randint(20, 60) // 100)
            for b in batches:
                p.latency_us.append(rng.randint(2000, 6000) * b)
                p.thr_mqps.append(per_replica * (3 + b) // 4)
    if variant_factors:
        p.variant_factor_q4 = [rng.randint(2, 8) for _ in p.acc_ppm]
    p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(rng.randint(0, 1 << 30)))
    return p, demand


@pytest.mark.parametrize("variant_factors", [False, True])
@pytest.mark.parametrize("per_variant_batch", [False, True])
def test_against_the_exact_rational_reference(variant_factors, per_variant_batch):
    rng = random.Random(100 + 2 * variant_factors + per_variant_batch)
    checked = coupled = 0
    for _ in range(12):
        p, demand = tight_problem(rng, variant_factors, per_variant_batch)
        O = oracle.Problem(p)
        n = O.num_candidates()
        for idx in rng.sample(range(n), min(n, 1500)):
            e = O.eval(idx, demand, 99, 1_000_000)
            if e.infeasible:
                continue
            r = pyref.evaluate(p, idx, demand, 99, 1_000_000)
            assert r["infeasible"] == 0
            assert abs(Fraction(e.accuracy) - r["exact"]) < TOL, idx
            checked += 1
            route = O.route_table(idx, demand)
            if all(sum(1 for k in range(8) if route.routed[i][k] > 0) > 1 for i in range(p.n_tasks)):
                coupled += 1
            if checked >= 60 * (_ + 1):
                break
    assert checked > 200 and coupled > 50   # plans in which every task really splits its traffic


def test_brute_force_search_agrees_with_the_exact_reference():
    done = 0
    for seed in range(80):
        w = wl.random_small(seed, path_tables=True, max_candidates=600)
        O = oracle.Problem(w.pipeline)
        best = O.search(w.demand_mqps[0], w.workers, w.slo_us, w.comm_us)
        exact_best, n_feasible = None, 0
        for idx in range(O.num_candidates()):
            r = pyref.evaluate(w.pipeline, idx, w.demand_mqps[0], w.workers, w.slo_us, w.comm_us)
            if r["infeasible"]:
                continue
            n_feasible += 1
            if exact_best is None or r["exact"] > exact_best:
                exact_best = r["exact"]
        assert best.n_feasible == n_feasible, seed
        if n_feasible:
            done += 1
            # the winner's exact value is the maximum up to fp64 rounding of near ties
            won = pyref.evaluate(w.pipeline, best.index, w.demand_mqps[0], w.workers, w.slo_us, w.comm_us)
            assert won["exact"] >= exact_best - Fraction(1, 10**13), seed
            assert abs(Fraction(best.accuracy) - won["exact"]) < TOL
    assert done >= 15


def additive_table(p, g):
    """A-hat(p) = sum over the path's tasks of g[task][variant] (ppm)."""
    out = []
    for path in p.leaf_paths():
        size = 1
        for i in path:
            size *= p.n_variants[i]
        for e in range(size):
            rest, v = e, 0
            for i in path:
                v += g[i][rest % p.n_variants[i]]
                rest //= p.n_variants[i]
            out.append(v)
    return out


def test_additive_tables_depend_on_the_marginals_only():
    """If A-hat(p) is a sum of per-task terms, sum_p c(p) A-hat(p) = sum over tasks of the task's
    traffic shares times its terms, whatever the coupling between tasks: the shares of a task's
    variants are routed/demand from the routing table.  (One factor per edge: with per-variant factors
    the requests of a task are no longer in proportion to the root requests they stem from, and c(p)
    follows a root request's lineage, not the downstream request counts.)"""
    rng = random.Random(11)
    checked = 0
    for trial in range(16):
        p, demand = tight_problem(rng)
        g = [[rng.randint(0, 1_000_000 // p.n_tasks) for _ in range(p.n_variants[i])] for i in range(p.n_tasks)]
        p.path_acc_ppm = additive_table(p, g)
        O = oracle.Problem(p)
        paths = p.leaf_paths()
        n = O.num_candidates()
        found = 0
        for idx in rng.sample(range(n), min(n, 1500)):
            e = O.eval(idx, demand, 99, 1_000_000)
            if e.infeasible:
                continue
            r = O.route_table(idx, demand)
            want = Fraction(0)
            for path in paths:
                for i in path:
                    for k in range(p.n_variants[i]):
                        want += Fraction(r.routed[i][k], r.demand[i]) * Fraction(g[i][k], 1_000_000)
            want /= len(paths)
            assert abs(Fraction(e.accuracy) - want) < TOL, (trial, idx)
            checked += 1
            found += 1
            if found >= 30:
                break
    assert checked > 200


def test_constant_table_and_single_variant_plans():
    for seed in range(30):
        w = wl.random_small(seed, max_candidates=4000)
        p = w.pipeline
        sizes = p.path_table_sizes()
        p.path_acc_ppm = [640000] * sum(sizes)
        O = oracle.Problem(p)
        for idx, e in feasible_samples(w, O, 20):
            assert abs(e.accuracy - 0.64) < TOL          # the shares of every task path sum to one
        # distinct entries: a plan hosting one variant per task scores exactly its own entry
        p.path_acc_ppm = [100000 + 37 * j for j in range(sum(sizes))]
        O = oracle.Problem(p)
        paths = p.leaf_paths()
        for idx, e in feasible_samples(w, O, 400):
            x, _ = O.decode(idx)
            voff, per_task = 0, []
            for i in range(p.n_tasks):
                per_task.append([k for k in range(p.n_variants[i]) if x[voff + k] > 0])
                voff += p.n_variants[i]
            if any(len(h) != 1 for h in per_task):
                continue
            want, off = Fraction(0), 0
            for path, size in zip(paths, sizes):
                entry, stride = 0, 1
                for i in path:
                    entry += per_task[i][0] * stride
                    stride *= p.n_variants[i]
                want += Fraction(p.path_acc_ppm[off + entry], 1_000_000)
                off += size
            assert abs(Fraction(e.accuracy) - want / len(paths)) < TOL
            if len(paths) == 1:
                assert e.accuracy == p.path_acc_ppm[entry] / 1000000.0   # mass 1.0: not even a rounding


def test_product_tables_match_the_product_objective_when_nothing_is_coupled():
    """Two-task chain whose root has a single variant: c(p) is the leaf's traffic share, so with
    A-hat(p) = A(root) * A(leaf variant) the sum is the product of the two task accuracies, the
    objective that the other pins hold in place.  Accuracies in whole thousandths keep the products
    integral in ppm."""
    rng = random.Random(5)
    checked = 0
    for _ in range(30):
        k1 = rng.randint(2, 4)
        acc0 = [rng.randint(600, 950) * 1000]
        acc1 = [rng.randint(600, 950) * 1000 for _ in range(k1)]
        lat = [rng.randint(2000, 9000) for _ in range(1 + k1)]
        p = SimpleNamespace(n_tasks=2, parent=[-1, 0], fanout_q4=[4, rng.randint(2, 9)], n_variants=[1, k1],
                            n_batches=[1, 1], batch_size=[2, 4], max_replicas=[3] + [2] * k1, acc_ppm=acc0 + acc1,
                            latency_us=lat, thr_mqps=[2 * 10**9 // lat[0]] + [4 * 10**9 // v for v in lat[1:]],
                            path_acc_ppm=[acc0[0] * a // 1_000_000 for a in acc1])
        plain = SimpleNamespace(**{**vars(p), "path_acc_ppm": None})
        O, Q = oracle.Problem(p), oracle.Problem(plain)
        demand = rng.randint(100_000, 900_000)
        for idx in range(O.num_candidates()):
            e, q = O.eval(idx, demand, 9, 100_000), Q.eval(idx, demand, 9, 100_000)
            assert e.infeasible == q.infeasible
            if not e.infeasible:
                assert abs(e.accuracy - q.accuracy) < TOL
                checked += 1
    assert checked > 200


def test_no_demand_scores_the_first_hosted_variants():
    g, p = load_example()
    O = oracle.Problem(p)
    # hosting everything: the most accurate variants A (index 1) and X (index 0) -> entry 1 + 2*0
    e = O.eval(O.encode([1, 1, 1, 1], [0, 0]), 0, 4, g["slo_us"])
    assert e.infeasible == 0 and e.accuracy == 880000 / 1000000.0
    e = O.eval(O.encode([1, 0, 0, 1], [0, 0]), 0, 4, g["slo_us"])       # only B and Y hosted
    assert e.infeasible == 0 and e.accuracy == 660000 / 1000000.0


def test_tabulated_search_falls_back_and_agrees():
    w = wl.random_small(12, path_tables=True, max_candidates=4000)
    O = oracle.Problem(w.pipeline)
    a = O.search(w.demand_mqps[0], w.workers, w.slo_us, w.comm_us)
    b = O.search_tabulated(w.demand_mqps[0], w.workers, w.slo_us, w.comm_us)
    assert a.as_tuple() == b.as_tuple()
