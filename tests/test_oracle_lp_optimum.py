"""Pin for the CPU checker's objective with profiled path accuracies against a linear program.

The paper's optimisation model lets the solver choose the path ratios c(p) freely, subject to the
capacity of every variant (Section 4.1: objective sum_p c(p) A-hat(p), eq. (1)-(2)); its Resource
Manager then routes most-accurate-first (Algorithm 1, Section 5.1) and the paper remarks that this
routing is optimal.  For a fixed allocation the best c(p) is a linear program, solved here with
scipy's HiGHS.  When A-hat is the product of per-variant accuracies and every task path has at most two
tasks, the optimum is known in closed form from the rearrangement inequality: fill the most accurate
variants first at every task and pair the most accurate upstream requests with the most accurate
downstream variants, which is what Algorithm 1's sequential bookkeeping does.  So:

  * product tables, paths of two tasks: LP optimum == the checker's objective for the same allocation;
  * any table, any tree: LP optimum >= the checker's objective (the LP may route better, never worse).

Nothing here calls the checker's formulas: the LP only knows capacities, demands and the table."""
import random

import numpy as np
import pytest
from scipy.optimize import linprog

import oracle
from paper_2407_03583_amd import workloads as wl

LP_TOL = 1e-8   # HiGHS is run with tolerances of 1e-10; a wrong coupling moves the objective by 1e-3 and more


def small_tree(rng, parent, product_tables):
    """One batch size per task, accuracies on a 0.001 grid so that products are exact in parts per million."""
    n = len(parent)
    demand = rng.randint(60_000, 300_000)
    p = wl.Pipeline(n_tasks=n, parent=parent, fanout_q4=[4] + [rng.randint(2, 10) for _ in range(n - 1)],
                    n_variants=[], n_batches=[], batch_size=[], max_replicas=[], acc_ppm=[], latency_us=[],
                    thr_mqps=[])
    level = [float(demand)]          # eq. (1): requests/s per task, in milli-QPS (quarters are exact in binary)
    for i in range(1, n):
        level.append(level[parent[i]] * p.fanout_q4[i] / 4)
    for i in range(n):
        k_i = rng.randint(2, 3)
        p.n_variants.append(k_i)
        p.n_batches.append(1)
        p.batch_size.append(2)
        for acc in rng.sample(range(600, 951), k_i):     # distinct, so the order of accuracy is strict
            p.max_replicas.append(2)
            p.acc_ppm.append(acc * 1000)
            p.latency_us.append(rng.randint(2000, 6000))
            p.thr_mqps.append(max(1000, int(level[i]) * rng.randint(20, 60) // 100))
    offs = np.concatenate([[0], np.cumsum(p.n_variants)])
    table = []
    for path in p.leaf_paths():
        sizes = [p.n_variants[i] for i in path]
        for e in range(int(np.prod(sizes))):
            ks, rest = [], e
            for s in sizes:          # the root's variant is the least significant digit
                ks.append(rest % s)
                rest //= s
            if product_tables:
                num = 1
                for i, k in zip(path, ks):
                    num *= p.acc_ppm[offs[i] + k]
                assert num % 10 ** (6 * (len(path) - 1)) == 0 or len(path) > 2
                table.append(num // 10 ** (6 * (len(path) - 1)))
            else:
                table.append(rng.randint(300_000, 990_000))
    p.path_acc_ppm = table
    return p, demand, level


def lp_optimum(p, demand_levels, xs):
    """max over the path ratios of every root-to-leaf task path, root marginal shared between the paths."""
    offs = np.concatenate([[0], np.cumsum(p.n_variants)])
    paths = p.leaf_paths()
    # variables: per task path, one per combination of variants (same order as the table)
    sizes = [[p.n_variants[i] for i in path] for path in paths]
    counts = [int(np.prod(s)) for s in sizes]
    start = np.concatenate([[0], np.cumsum(counts)])
    nvar = int(start[-1])
    cost = -np.array(p.path_acc_ppm, dtype=float) / 1e6 / len(paths)

    def digits(j, e):
        ks = []
        for s in sizes[j]:
            ks.append(e % s)
            e //= s
        return ks

    A_ub, b_ub, A_eq, b_eq = [], [], [], []
    for j, path in enumerate(paths):
        row = np.zeros(nvar)
        row[start[j]:start[j + 1]] = 1.0
        A_eq.append(row)
        b_eq.append(1.0)           # every request of the root takes some variant path
        for depth, i in enumerate(path):
            if depth == 0 and j > 0:
                continue           # the root's capacity is stated once; marginals are tied below
            for k in range(p.n_variants[i]):
                row = np.zeros(nvar)
                for e in range(counts[j]):
                    if digits(j, e)[depth] == k:
                        row[start[j] + e] = 1.0     # share of task i's requests that reaches its variant k
                A_ub.append(row)
                b_ub.append(xs[i][k] * p.thr_mqps[offs[i] + k] / demand_levels[i])   # eq. (2): capacity of its replicas over the task's demand
    # tasks shared by several task paths see one and the same split of their requests
    for j in range(1, len(paths)):
        shared = [d for d, i in enumerate(paths[j]) if d < len(paths[0]) and paths[0][d] == i]
        for d in shared:
            i = paths[j][d]
            for k in range(p.n_variants[i]):
                row = np.zeros(nvar)
                for e in range(counts[0]):
                    if digits(0, e)[d] == k:
                        row[start[0] + e] += 1.0
                for e in range(counts[j]):
                    if digits(j, e)[d] == k:
                        row[start[j] + e] -= 1.0
                A_eq.append(row)
                b_eq.append(0.0)
    r = linprog(cost, A_ub=np.array(A_ub), b_ub=np.array(b_ub, dtype=float), A_eq=np.array(A_eq), b_eq=np.array(b_eq),
                bounds=(0, None), method="highs",
                options={"primal_feasibility_tolerance": 1e-10, "dual_feasibility_tolerance": 1e-10})
    return -r.fun if r.status == 0 else None


def sampled_plans(rng, p, demand, limit):
    O = oracle.Problem(p)
    n = O.num_candidates()
    out = []
    for idx in rng.sample(range(n), min(n, 4000)):
        e = O.eval(idx, demand, 99, 10_000_000)
        if e.infeasible:
            continue
        x, _ = O.decode(idx)
        xs, at = [], 0
        for k_i in p.n_variants:
            xs.append(list(x[at:at + k_i]))
            at += k_i
        out.append((idx, e.accuracy, xs))
        if len(out) >= limit:
            break
    return out


@pytest.mark.parametrize("parent", [[-1, 0], [-1, 0, 0]])
def test_product_tables_on_short_paths_reach_the_lp_optimum(parent):
    rng = random.Random(7 + len(parent))
    checked = split = 0
    for _ in range(10):
        p, demand, level = small_tree(rng, parent, product_tables=True)
        for idx, acc, xs in sampled_plans(rng, p, demand, 25):
            best = lp_optimum(p, level, xs)
            assert best is not None, idx
            assert abs(best - acc) < LP_TOL, (idx, best, acc)
            checked += 1
            split += all(sum(1 for v in task if v > 0) > 1 for task in xs)
    assert checked > 100 and split > 30     # plans that host several variants of every task among them


@pytest.mark.parametrize("parent,product", [([-1, 0, 1], True), ([-1, 0, 1], False), ([-1, 0, 0], False),
                                            ([-1, 0, 1, 0], False)])
def test_no_routing_scores_above_the_lp_optimum(parent, product):
    """Longer paths or arbitrary tables: hop-by-hop most-accurate-first routing need not be the best
    choice of path ratios, but it is one of the choices the LP ranges over."""
    rng = random.Random(70 + len(parent) + product)
    checked = below = 0
    for _ in range(6):
        p, demand, level = small_tree(rng, parent, product_tables=product)
        for idx, acc, xs in sampled_plans(rng, p, demand, 20):
            best = lp_optimum(p, level, xs)
            assert best is not None, idx
            assert acc <= best + LP_TOL, (idx, best, acc)
            checked += 1
            below += acc < best - 1e-5
    assert checked > 60
    if not product:
        assert below > 0        # with arbitrary tables the LP does find better routings somewhere


def milp_optimum(p, demand_levels, workers, slack=0.0):
    """The paper's optimisation model with the latency limit out of the way (Section 4.1, Step 2): integer
    replica counts x(i,k) within their bounds, free path ratios, eq. (2) per variant, eq. (3) on the total;
    maximise sum_p c(p) A-hat(p) averaged over the task paths.  slack: relative change of every capacity
    (the solver accepts violations of about 1e-6, so the caller brackets the exact answer)."""
    from scipy.optimize import milp, LinearConstraint, Bounds
    offs = np.concatenate([[0], np.cumsum(p.n_variants)])
    paths = p.leaf_paths()
    sizes = [[p.n_variants[i] for i in path] for path in paths]
    counts = [int(np.prod(s)) for s in sizes]
    start = np.concatenate([[0], np.cumsum(counts)])
    nf = int(start[-1])
    nx = int(offs[-1])
    nvar = nf + nx                      # path ratios first, then the replica counts
    cost = np.concatenate([-np.array(p.path_acc_ppm, dtype=float) / 1e6 / len(paths), np.zeros(nx)])

    def digit(j, e, depth):
        for s in sizes[j][:depth]:
            e //= s
        return e % sizes[j][depth]

    rows, lo, hi = [], [], []
    for j, path in enumerate(paths):
        row = np.zeros(nvar)
        row[start[j]:start[j + 1]] = 1.0
        rows.append(row), lo.append(1.0), hi.append(1.0)
        for depth, i in enumerate(path):
            for k in range(p.n_variants[i]):
                share = np.zeros(nvar)
                for e in range(counts[j]):
                    if digit(j, e, depth) == k:
                        share[start[j] + e] = 1.0
                if depth == 0 and j > 0:        # the root splits its requests one way for all task paths
                    first = np.zeros(nvar)
                    for e in range(counts[0]):
                        if digit(0, e, 0) == k:
                            first[start[0] + e] = 1.0
                    rows.append(share - first), lo.append(0.0), hi.append(0.0)
                    continue
                share[nf + offs[i] + k] = -p.thr_mqps[offs[i] + k] * (1.0 + slack) / demand_levels[i]    # eq. (2)
                rows.append(share), lo.append(-np.inf), hi.append(0.0)
    total = np.zeros(nvar)
    total[nf:] = 1.0
    rows.append(total), lo.append(0.0), hi.append(float(workers))                            # eq. (3)
    integrality = np.concatenate([np.zeros(nf), np.ones(nx)])
    bounds = Bounds(np.zeros(nvar), np.concatenate([np.ones(nf), np.array(p.max_replicas, dtype=float)]))
    r = milp(cost, constraints=LinearConstraint(np.array(rows), np.array(lo), np.array(hi)), integrality=integrality,
             bounds=bounds, options={"mip_rel_gap": 0.0})
    return -r.fun if r.status == 0 else None


@pytest.mark.parametrize("parent", [[-1, 0], [-1, 0, 0]])
def test_search_optimum_equals_the_milp_optimum_when_latency_does_not_bind(parent):
    """The exhaustive search over bounded replica counts with most-accurate-first routing against the
    paper's own formulation (solver-chosen path ratios) on pipelines where the two must agree: product
    tables, task paths of two tasks, a service-level objective no plan can miss."""
    rng = random.Random(300 + len(parent))
    solved = budget_binds = 0
    for _ in range(30):
        p, demand, level = small_tree(rng, parent, product_tables=True)
        O = oracle.Problem(p)
        unlimited = O.search(demand, 99, 10_000_000)
        if not unlimited.found:
            continue
        workers = max(len(parent), unlimited.workers - rng.randint(0, 3))
        best = O.search(demand, workers, 10_000_000)
        # the solver tolerates constraint violations of about 1e-6 (a capacity 0.25 milli-QPS short of the
        # demand passes), so bracket the exact optimum between slightly smaller and slightly larger capacities
        below = milp_optimum(p, level, workers, -1e-5)
        above = milp_optimum(p, level, workers, +1e-5)
        if not best.found:
            assert below is None
            continue
        assert above is not None
        assert best.accuracy <= above + 2e-6, (above, best.accuracy)     # HiGHS stops branching at an absolute gap of 1e-6
        if below is None or above - below > 1e-4:
            continue            # a capacity sits within 1e-5 of a demand: the bracket says nothing there
        assert below - 2e-6 <= best.accuracy, (below, best.accuracy)
        solved += 1
        budget_binds += best.accuracy < unlimited.accuracy
    assert solved >= 12 and budget_binds >= 4, (solved, budget_binds)
