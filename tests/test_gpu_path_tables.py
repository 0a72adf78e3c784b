"""GPU parity for the objective from profiled path accuracies (sum_p c(p) * A-hat(p), Section 4.1
"Accuracy"; c(p) from Algorithm 1's routing, Section 5.1): search results and per-plan objectives
against the CPU checker, bit for bit."""
import json
import os
import random
import struct
from types import SimpleNamespace

import pytest

import oracle
from paper_2407_03583_amd import binding, workloads as wl
from test_oracle_path_tables import tight_problem

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TIE = binding.LOKI_TIE_INDEX_ONLY
LANE = binding.LOKI_SEARCH_PER_LANE   # the kernel that scores whole plans per lane (else: the tabulated walk
                                      # over the plan space with the variant paths walked for feasible plans)


def bits(x):
    return struct.unpack("<Q", struct.pack("<d", x))[0]


def agree(res, ref):
    got, want = res.as_tuple(), ref.as_tuple()
    return got[0] == want[0] and bits(got[1]) == bits(want[1]) and got[2:] == want[2:]


def check_plans(P, O, indices, demand, workers, slo, comm=0):
    out = P.alloc_eval(indices, demand, workers, slo, comm)
    feasible = 0
    for idx, got in zip(indices, out):
        e = O.eval(idx, demand, workers, slo, comm)
        assert got.infeasible == e.infeasible and got.workers == e.workers, idx
        assert bits(got.accuracy) == bits(e.accuracy), (idx, got.accuracy, e.accuracy)
        feasible += e.infeasible == 0
    return feasible


def test_hand_derived_example():
    g = json.load(open(os.path.join(GOLDEN, "path_table_example.json")))
    p = SimpleNamespace(**g["pipeline"])
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    assert check_plans(P, O, list(range(n)), g["demand_mqps"], g["workers"], g["slo_us"]) > 0
    idx = O.encode(g["plan_x"], [0, 0])
    got = P.alloc_eval([idx], g["demand_mqps"], g["workers"], g["slo_us"])[0]
    assert abs(got.accuracy - 0.779) < 1e-15
    for demand in (g["demand_mqps"], 0, 30_000, 160_000, 10**7):
        for flags in (0, TIE):
            res = P.alloc_search([demand], g["workers"], g["slo_us"], flags=flags)[0]
            assert agree(res, O.search(demand, g["workers"], g["slo_us"], tie_index_only=bool(flags))), demand


@pytest.mark.parametrize("variant_factors", [False, True])
@pytest.mark.parametrize("per_variant_batch", [False, True])
def test_small_random_problems(variant_factors, per_variant_batch):
    found = 0
    for seed in range(48):
        w = wl.random_small(seed, path_tables=True, variant_factors=variant_factors,
                            per_variant_batch=per_variant_batch, max_candidates=6000)
        P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
        n = P.num_candidates()
        d = w.demand_mqps[0]
        for flags in (0, TIE, LANE, LANE | TIE):
            res = P.alloc_search([d], w.workers, w.slo_us, w.comm_us, flags=flags)[0]
            ref = O.search(d, w.workers, w.slo_us, w.comm_us, tie_index_only=bool(flags & TIE))
            assert agree(res, ref), (seed, flags, res.as_tuple(), ref.as_tuple())
        found += res.status == 0
        check_plans(P, O, list(range(0, n, max(1, n // 300))), d, w.workers, w.slo_us, w.comm_us)
        # a split range merges to the same answer as the checker on the same range
        a, b = n // 3, n - n // 5
        for flags in (0, LANE):
            res = P.alloc_search([d], w.workers, w.slo_us, w.comm_us, begin=a, end=b, flags=flags)[0]
            assert agree(res, O.search(d, w.workers, w.slo_us, w.comm_us, begin=a, end=b)), (seed, flags)
    assert found >= 8


@pytest.mark.parametrize("variant_factors", [False, True])
@pytest.mark.parametrize("per_variant_batch", [False, True])
def test_plans_that_split_traffic_at_every_task(variant_factors, per_variant_batch):
    rng = random.Random(500 + 2 * variant_factors + per_variant_batch)
    feasible = 0
    for _ in range(10):
        p, demand = tight_problem(rng, variant_factors, per_variant_batch)
        P, O = binding.Problem(p), oracle.Problem(p)
        n = P.num_candidates()
        feasible += check_plans(P, O, rng.sample(range(n), min(n, 3000)), demand, 99, 1_000_000)
        if n <= 300_000:
            for flags in (0, TIE, LANE):
                res = P.alloc_search([demand, demand // 2, 2 * demand], 99, 1_000_000, flags=flags)
                for d, r in zip([demand, demand // 2, 2 * demand], res):
                    assert agree(r, O.search(d, 99, 1_000_000, tie_index_only=bool(flags & TIE))), (d, flags)
    assert feasible > 300


@pytest.mark.parametrize("n_tasks,k,replicas", [(2, 5, 2), (2, 5, 3), (3, 4, 1), (3, 3, 2), (1, 6, 2)])
def test_chains_with_many_feasible_plans(n_tasks, k, replicas):
    """Single task paths, where the tabulated search skips the walk for plans whose upper bound on the objective
    cannot reach the best one seen: dense demand points (many feasible plans, many of them near the top),
    several points per call, ties on and off, split ranges, against the checker's plain search."""
    rng = wl.SplitMix64(300 + 10 * n_tasks + k)
    p = wl.make_pipeline([-1] + list(range(n_tasks - 1)), k, replicas, (1, 4), rng)
    p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(301 + k))
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    demands = [0, 20_000, 60_000, 120_000, 200_000, 350_000]
    dense = 0
    for flags in (0, TIE):
        out = P.alloc_search(demands, 24, 400_000, flags=flags)
        for d, res in zip(demands, out):
            ref = O.search(d, 24, 400_000, tie_index_only=bool(flags & TIE))
            assert agree(res, ref), (d, flags, res.as_tuple(), ref.as_tuple())
            dense += ref.n_feasible * 20 > n
    assert dense >= 2
    a, b = n // 3 + 7, n - n // 4
    for lo, hi in ((0, a), (a, b), (b, n)):
        res = P.alloc_search([60_000], 24, 400_000, begin=lo, end=hi)[0]
        assert agree(res, O.search(60_000, 24, 400_000, begin=lo, end=hi)), (lo, hi)
    # a table that rises with the first task's variant only, and one that is constant: bounds that are tight
    # for every plan (nothing can be skipped on the strength of the bound alone)
    for table in ([600_000 + 40_000 * (e % k) for e in range(k ** n_tasks)], [777_000] * (k ** n_tasks)):
        p.path_acc_ppm = table
        P, O = binding.Problem(p), oracle.Problem(p)
        for d in (60_000, 200_000):
            res, ref = P.alloc_search([d], 24, 400_000)[0], O.search(d, 24, 400_000)
            assert agree(res, ref), (d, res.as_tuple(), ref.as_tuple())


def test_four_task_tree_with_three_variants():
    """Tree 0 -> 1 -> 2, 0 -> 3: two task paths of different length, tables of 27 and 9 entries, 8.5
    million plans, searched in one call for several demand points and in two halves."""
    rng = wl.SplitMix64(80)
    p = wl.make_pipeline([-1, 0, 1, 0], 3, 2, (1, 4), rng)
    p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(78))
    assert p.path_table_sizes() == [27, 9]
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    assert n == (27 * 2) ** 4
    demands = [20_000, 60_000, 150_000, 300_000]
    out = P.alloc_search(demands, 20, 600_000)
    per_lane = P.alloc_search(demands, 20, 600_000, flags=LANE)
    found = 0
    for d, res, res_lane in zip(demands, out, per_lane):
        ref = O.search(d, 20, 600_000)
        assert agree(res, ref), (d, res.as_tuple(), ref.as_tuple())
        assert agree(res_lane, ref), (d, res_lane.as_tuple(), ref.as_tuple())
        found += ref.found
    assert found == 3
    half = n // 2 + 12345
    lo = P.alloc_search([60_000], 20, 600_000, begin=0, end=half)[0]
    hi = P.alloc_search([60_000], 20, 600_000, begin=half, end=n)[0]
    assert agree(lo, O.search(60_000, 20, 600_000, begin=0, end=half))
    assert agree(hi, O.search(60_000, 20, 600_000, begin=half, end=n))
    assert lo.n_feasible + hi.n_feasible == out[1].n_feasible


def test_deep_chain_reaches_the_last_level():
    """Eight tasks in a chain with two variants each: one table of 256 entries, eight levels of the walk."""
    rng = random.Random(3)
    acc, lat, thr = [], [], []
    for i in range(8):
        for k in range(2):
            acc.append(rng.randint(70, 95) * 10000)
            l = rng.randint(1500, 3000)
            lat.append(l)
            thr.append(rng.randint(60_000, 140_000))
    p = wl.Pipeline(n_tasks=8, parent=[-1, 0, 1, 2, 3, 4, 5, 6], fanout_q4=[4] * 8, n_variants=[2] * 8,
                    n_batches=[1] * 8, batch_size=[2] * 8, max_replicas=[1, 2] * 8, acc_ppm=acc, latency_us=lat,
                    thr_mqps=thr)
    p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(5))
    assert p.path_table_sizes() == [256]
    P, O = binding.Problem(p), oracle.Problem(p)
    assert P.num_candidates() == 6 ** 8
    for demand, W in ((150_000, 24), (0, 8), (100_000, 12)):
        ref = O.search(demand, W, 100_000)
        for flags in (0, LANE):
            res = P.alloc_search([demand], W, 100_000, flags=flags)[0]
            assert agree(res, ref), (demand, flags, res.as_tuple(), ref.as_tuple())


def test_plan_trace_with_path_tables():
    """The demand-trace planner on config 1 with profiled path accuracies: every step's plan against the
    checker, and the phase against the entry of the most accurate variants."""
    w = wl.config(1)
    p = w.pipeline
    p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(9))
    P, O = binding.Problem(p), oracle.Problem(p)
    ramp = [7_000 * t for t in range(60)]
    steps = P.plan_trace(ramp, 500_000, w.workers, w.slo_us)
    top_entry = (p.n_variants[0] - 1) + p.n_variants[0] * (p.n_variants[1] - 1)   # accuracies are sorted ascending
    top = p.path_acc_ppm[top_entry] / 1000000.0
    phases = set()
    for t, s in enumerate(steps):
        ref = O.search(s.estimate_mqps, w.workers, w.slo_us)
        assert agree(s.plan, ref), (t, s.plan.as_tuple(), ref.as_tuple())
        want = binding.LOKI_PHASE_OVERLOAD if not ref.found else (
            binding.LOKI_PHASE_HARDWARE if ref.accuracy >= top else binding.LOKI_PHASE_ACCURACY)
        assert s.phase == want, t
        phases.add(s.phase)
    assert phases == {0, 1, 2}


def test_config_sizes_with_path_tables_tabulated_against_per_lane():
    """Config 2 (2^30 plans) with profiled path accuracies: the tabulated walk over the plan space against the
    kernel that scores whole plans per lane, full space and a ragged index range; config 5 (2^40 plans,
    out of the per-lane kernel's reach): the winner through the checker, the feasible count against the
    stored result of the plain model (feasibility does not depend on the objective)."""
    w = wl.config(2)
    p = w.pipeline
    p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(w.seed + 1))
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    for begin, end in ((0, n), (n // 7 + 3, n - n // 11)):
        a = P.alloc_search(w.demand_mqps, w.workers, w.slo_us, begin=begin, end=end)[0]
        b = P.alloc_search(w.demand_mqps, w.workers, w.slo_us, begin=begin, end=end, flags=LANE)[0]
        assert agree(a, b), (begin, end, a.as_tuple(), b.as_tuple())
        assert a.status == 0 and a.n_feasible > 100_000
        e = O.eval(a.index, w.demand_mqps[0], w.workers, w.slo_us)
        assert e.infeasible == 0 and bits(e.accuracy) == bits(a.accuracy) and e.workers == a.workers_used
    w5 = wl.config(5)
    p5 = w5.pipeline
    p5.path_acc_ppm = wl.draw_path_tables(p5, wl.SplitMix64(w5.seed + 1))
    P5, O5 = binding.Problem(p5), oracle.Problem(p5)
    r = P5.alloc_search(w5.demand_mqps, w5.workers, w5.slo_us)[0]
    doc = json.load(open(os.path.join(GOLDEN, "cfg5.json")))
    assert r.status == 0 and r.n_feasible == doc["results"][0]["n_feasible"] == 108
    e = O5.eval(r.index, w5.demand_mqps[0], w5.workers, w5.slo_us)
    assert e.infeasible == 0 and bits(e.accuracy) == bits(r.accuracy) and e.workers == r.workers_used


TREES_WITH_SEVERAL_LEAVES = [   # parents, what the case is for, variants per task
    ([-1, 0, 0], "star, two leaves", 2),
    ([-1, 0, 0, 0], "star, three leaves: the path count is no power of two, one leaf belongs to the work item", 2),
    ([-1, 0, 1, 0], "paths of three and two tasks", 2),
    ([-1, 0, 1, 1], "both leaves under task 1: the last task has two ancestors", 2),
    ([-1, 0, 0, 1, 2], "two chains of three tasks", 2),
    ([-1, 0, 1, 2, 3, 0], "a path of five tasks", 2),
    ([-1, 0, 1, 2, 3, 0], "a path of five tasks with 81 branches above its leaf: more than are taken leaf by leaf", 3),
]


# (with per-variant factors the fixed-point range check leaves no demand worth testing at five levels)
@pytest.mark.parametrize("parent,what,n_variants,variant_factors",
                         [(t, w, k, vf) for t, w, k in TREES_WITH_SEVERAL_LEAVES for vf in (False, True)
                          if not (vf and len(t) == 6)])
def test_trees_with_several_leaves_leaf_by_leaf(parent, what, n_variants, variant_factors):
    """With two or more leaves the objective is a sum of one value per leaf, each a function of the choices
    along that leaf's task path (Section 4.1 "Accuracy": the system accuracy averages over the task paths);
    the search forms each value once for all the plans that share those choices.  Whole space, both tie
    rules, several demand points, and index ranges, against the checker's plan-by-plan search."""
    n = len(parent)
    rng = wl.SplitMix64(900 + 7 * n + sum(parent))
    p = wl.make_pipeline(parent, n_variants, 2 if n <= 5 else 1, (1, 4) if n_variants == 2 else (2,), rng)
    p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(901 + n))
    if variant_factors:
        p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]
    by_leaf = n_variants ** (n - 2) <= 64   # (holds for these trees: the deepest leaf has n - 2 ancestors)
    P, O = binding.Problem(p), oracle.Problem(p)
    N = P.num_candidates()
    assert N <= 2_000_000
    workers, slo = 3 * n, 500_000
    demands = {3: [15_000, 40_000, 90_000, 200_000], 4: [15_000, 40_000, 90_000, 200_000],
               5: [1_000, 4_000, 10_000, 25_000], 6: [500, 1_000, 2_000, 4_000]}[n]
    if n_variants == 3:
        demands = [2_000, 8_000, 20_000, 50_000]
    found = 0
    for flags in (0, TIE):
        out = P.alloc_search(demands, workers, slo, flags=flags)
        for d, res in zip(demands, out):
            ref = O.search(d, workers, slo, tie_index_only=bool(flags))
            assert agree(res, ref), (what, d, flags, res.as_tuple(), ref.as_tuple())
            found += ref.found
    assert found >= 4, what
    # which way the search went shows in the number of plans its kernels visited: leaf by leaf the work
    # items hold only usable choices of the tasks with children; the walk over the whole space visits all
    if not variant_factors:
        if by_leaf:
            assert 0 < P.last_search_plans_scored() < N * len(demands), what
        else:
            assert P.last_search_plans_scored() == N * len(demands), what
    d = demands[1]
    cuts = [0, N // 7, N // 2 + 3, N - N // 5, N]
    total = 0
    for a, b in zip(cuts, cuts[1:]):
        res = P.alloc_search([d], workers, slo, begin=a, end=b)[0]
        assert agree(res, O.search(d, workers, slo, begin=a, end=b)), (what, a, b)
        total += res.n_feasible
    assert total == P.alloc_search([d], workers, slo)[0].n_feasible > 0
    # a tight worker budget and a tight latency limit
    for w_, s_ in ((n + 2, slo), (workers, 160_000 if n <= 5 else 260_000)):
        res = P.alloc_search([d], w_, s_)[0]
        assert agree(res, O.search(d, w_, s_)), (what, w_, s_)
    # no demand at all: no variant has traffic, every hop hands on to the first hosted variant
    res = P.alloc_search([0, 1], workers, slo)
    for d0, r in zip([0, 1], res):
        assert agree(r, O.search(d0, workers, slo)), (what, "demand", d0)
