"""A second, independent reading of the candidate evaluation, used only to pin
the C checker in oracle/ on small problems.

Written in exact rational arithmetic in *real units* (queries/second, not the
checker's scaled integers): demand at a task is D * prod(fan-out) as a
Fraction, capacity is x * q as a Fraction, the task accuracy is a Fraction that
is rounded to a double exactly once.  The fp64 steps (path products root
first, path sum in leaf order, division by the number of paths) then follow in
Python floats, which are IEEE doubles with no contraction.

Citations: eq. (1)-(3), (6), (7), (12) and Algorithm 1 of the Loki paper
(HPDC'24), Sections 4.1, 4.2 and 5.1.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Dict, List, Tuple

BAD_WORKERS, BAD_DEMAND, BAD_EMPTY, BAD_LATENCY = 1, 2, 4, 8


def _tables(p):
    """Nested dicts: task -> variant -> {replica_limit, acc, lat{b}, thr{b}} plus batch lists."""
    tasks = []
    v = b = t = 0
    for i in range(p.n_tasks):
        batches = list(p.batch_size[b:b + p.n_batches[i]])
        variants = []
        for k in range(p.n_variants[i]):
            lat = {bi: p.latency_us[t + k * len(batches) + bi] for bi in range(len(batches))}
            thr = {bi: p.thr_mqps[t + k * len(batches) + bi] for bi in range(len(batches))}
            vf = getattr(p, "variant_factor_q4", None)
            variants.append(dict(limit=p.max_replicas[v + k], acc=p.acc_ppm[v + k], lat=lat, thr=thr,
                                 factor=None if vf is None else Fraction(vf[v + k], 4)))
        tasks.append(dict(batches=batches, variants=variants, parent=p.parent[i],
                          fan=Fraction(p.fanout_q4[i], 4)))
        v += p.n_variants[i]
        b += p.n_batches[i]
        t += p.n_variants[i] * len(batches)
    return tasks


def decode(p, index: int) -> List[Tuple[List[int], List[int]]]:
    """index -> per task (replica counts, batch position per variant); task 0 and variant 0 least
    significant.  One batch size per task: the batch digit is the most significant digit of the
    task's group.  Per-variant batch sizes: a variant's digit is 0 (not hosted) or
    1 + (replicas - 1) * |B| + batch position."""
    pv = bool(getattr(p, "per_variant_batch", False))
    plan = []
    for task in _tables(p):
        nb = len(task["batches"])
        xs, betas = [], []
        for var in task["variants"]:
            if pv:
                radix = 1 + var["limit"] * nb
                g = index % radix
                index //= radix
                xs.append(0 if g == 0 else (g - 1) // nb + 1)
                betas.append(0 if g == 0 else (g - 1) % nb)
            else:
                xs.append(index % (var["limit"] + 1))
                index //= var["limit"] + 1
        if not pv:
            beta = index % nb
            index //= nb
            betas = [beta] * len(xs)
        plan.append((xs, betas))
    return plan


def num_candidates(p) -> int:
    pv = bool(getattr(p, "per_variant_batch", False))
    n = 1
    for task in _tables(p):
        nb = len(task["batches"])
        if not pv:
            n *= nb
        for var in task["variants"]:
            n *= 1 + var["limit"] * nb if pv else var["limit"] + 1
    return n


def evaluate(p, index: int, demand_mqps: int, workers: int, slo_us: int, comm_us: int = 0) -> Dict:
    tasks = _tables(p)
    plan = decode(p, index)
    # demand per task in QPS (eq. (1)): with one factor per edge it is fixed up front; with
    # per-variant factors a child's demand is what the parent's variants create (filled in below)
    per_variant = tasks[0]["variants"][0]["factor"] is not None
    demand = []
    for i, task in enumerate(tasks):
        demand.append(Fraction(demand_mqps, 1000) if i == 0 else
                      (None if per_variant else demand[task["parent"]] * task["fan"]))
    created = [Fraction(0)] * len(tasks)  # requests per second a task creates per unit of child fan-out
    mask = 0
    used_workers = sum(sum(xs) for xs, _ in plan)
    if used_workers > workers:
        mask |= BAD_WORKERS
    acc_task, lat_task = [], []
    for i, task in enumerate(tasks):
        xs, betas = plan[i]
        if per_variant and i > 0:
            demand[i] = created[task["parent"]] * task["fan"]
        hosted = [k for k in range(len(xs)) if xs[k] > 0]
        hosted.sort(key=lambda k: (-task["variants"][k]["acc"], k))
        if not hosted:
            mask |= BAD_EMPTY
        left = demand[i]
        gained = Fraction(0)
        in_use = []
        for pos, k in enumerate(hosted):
            var = task["variants"][k]
            capacity = xs[k] * Fraction(var["thr"][betas[k]], 1000)
            take = min(left, capacity)
            if take > 0 or pos == 0:
                in_use.append(var["lat"][betas[k]])
            gained += take * Fraction(var["acc"], 1_000_000)
            if per_variant:
                created[i] += take * var["factor"]
            left -= take
        if left > 0:
            mask |= BAD_DEMAND
        lat_task.append(max(in_use) if in_use else 0)
        if demand[i] > 0:
            acc_task.append(gained / demand[i])
        elif hosted:
            acc_task.append(Fraction(task["variants"][hosted[0]]["acc"], 1_000_000))
        else:
            acc_task.append(Fraction(0))
    leaves = [i for i in range(len(tasks)) if all(t["parent"] != i for t in tasks)]
    paths = []
    for leaf in leaves:
        path, i = [], leaf
        while i >= 0:
            path.append(i)
            i = tasks[i]["parent"]
        paths.append(path[::-1])
    if getattr(p, "latency_per_path", False):
        # eq. (7) itself: every variant path that carries traffic, for plans that serve all demand
        if not mask & (BAD_DEMAND | BAD_EMPTY) and slow_path_with_traffic(p, index, demand_mqps, slo_us, comm_us):
            mask |= BAD_LATENCY
    else:
        for path in paths:
            room = slo_us - comm_us * len(path)
            if room < 0 or sum(lat_task[i] for i in path) > room // 2:
                mask |= BAD_LATENCY
    out = dict(infeasible=mask, workers=used_workers, accuracy=0.0, task_lat=lat_task)
    if mask == 0 and getattr(p, "path_acc_ppm", None) is not None:
        out["exact"] = path_objective_exact(p, index, demand_mqps)
        out["accuracy"] = float(out["exact"])   # within a few ulps of the checker's step-by-step fp64 value
        return out
    if mask == 0:
        a = [float(f) for f in acc_task]  # one correct rounding each
        total = None
        for path in paths:
            prod = a[path[0]]
            for i in path[1:]:
                prod = prod * a[i]
            total = prod if total is None else total + prod
        out["accuracy"] = total / float(len(paths))
        # exact value of the objective, for error-bound checks
        exact = Fraction(0)
        for path in paths:
            pr = Fraction(1)
            for i in path:
                pr *= acc_task[i]
            exact += pr
        out["exact"] = exact / len(paths)
    return out


def search(p, demand_mqps: int, workers: int, slo_us: int, comm_us: int = 0, tie_index_only: bool = False):
    best = None
    n_feasible = 0
    for index in range(num_candidates(p)):
        e = evaluate(p, index, demand_mqps, workers, slo_us, comm_us)
        if e["infeasible"]:
            continue
        n_feasible += 1
        key = (-e["accuracy"], 0 if tie_index_only else e["workers"], index)
        if best is None or key < best[0]:
            best = (key, index, e["accuracy"], e["workers"])
    if best is None:
        return dict(found=0, index=(1 << 64) - 1, accuracy=0.0, workers=-1, n_feasible=0)
    return dict(found=1, index=best[1], accuracy=best[2], workers=best[3], n_feasible=n_feasible)


def placement(p, index: int, demand_mqps: int):
    """Where every task's requests sit, as intervals of the task's request stream in QPS: the stream is
    handed to the hosted variants in order of accuracy (ties: lower index first), each taking what its
    capacity allows (Algorithm 1).  Returns per task: demand, {variant: (start, end)} and, per variant,
    the requests it creates per unit of child fan-out."""
    tasks = _tables(p)
    plan = decode(p, index)
    per_variant = tasks[0]["variants"][0]["factor"] is not None
    demand, spans, created = [], [], []
    for i, task in enumerate(tasks):
        xs, betas = plan[i]
        if i == 0:
            d = Fraction(demand_mqps, 1000)
        else:
            d = sum(created[task["parent"]].values(), Fraction(0)) * task["fan"]
        hosted = sorted((k for k in range(len(xs)) if xs[k] > 0), key=lambda k: (-task["variants"][k]["acc"], k))
        at, span, made = Fraction(0), {}, {}
        for k in hosted:
            var = task["variants"][k]
            take = min(d - at, xs[k] * Fraction(var["thr"][betas[k]], 1000))
            span[k] = (at, at + take)
            made[k] = take * (var["factor"] if per_variant else 1)
            at += take
        demand.append(d)
        spans.append(span)
        created.append(made)
    return tasks, plan, demand, spans, created


def path_objective_exact(p, index: int, demand_mqps: int) -> Fraction:
    """sum_p c(p) * A-hat(p), averaged over the root-to-leaf task paths, in exact arithmetic.

    The requests a variant creates for a child occupy one interval of the child's request stream, the
    upstream variants lined up by accuracy like the child's own variants; the share of an upstream
    variant's requests that a downstream variant serves is the overlap of the two intervals over the
    upstream interval's length.  (The checker instead replays Algorithm 1's sequential bookkeeping.)"""
    tasks, plan, demand, spans, created = placement(p, index, demand_mqps)
    leaves = [i for i in range(len(tasks)) if all(t["parent"] != i for t in tasks)]
    table = list(p.path_acc_ppm)
    offset = 0
    total = Fraction(0)

    def first_hosted(i):
        xs = plan[i][0]
        hosted = sorted((k for k in range(len(xs)) if xs[k] > 0), key=lambda k: (-tasks[i]["variants"][k]["acc"], k))
        return hosted[0]

    def split(i, upstream):
        """Shares over task i's variants of the requests coming from `upstream` = (parent task, variant),
        or from the frontend when upstream is None."""
        if upstream is None:
            lo, hi = Fraction(0), demand[0]
        else:
            par, kp = upstream
            order = sorted(created[par], key=lambda k: (-tasks[par]["variants"][k]["acc"], k))
            lo = sum((created[par][k] for k in order[:order.index(kp)]), Fraction(0)) * tasks[i]["fan"]
            hi = lo + created[par][kp] * tasks[i]["fan"]
        if hi == lo:
            return {first_hosted(i): Fraction(1)}
        shares = {}
        for k, (a, b) in spans[i].items():
            overlap = min(b, hi) - max(a, lo)
            if overlap > 0:
                shares[k] = overlap / (hi - lo)
        return shares

    for leaf in leaves:
        path, i = [], leaf
        while i >= 0:
            path.append(i)
            i = tasks[i]["parent"]
        path = path[::-1]
        sizes = [len(tasks[i]["variants"]) for i in path]

        def walk(depth, upstream, mass, entry, stride):
            i = path[depth]
            acc = Fraction(0)
            for k, share in split(i, upstream).items():
                e = entry + k * stride
                if depth == len(path) - 1:
                    acc += mass * share * Fraction(table[offset + e], 1_000_000)
                else:
                    acc += walk(depth + 1, (i, k), mass * share, e, stride * sizes[depth])
            return acc

        total += walk(0, None, Fraction(1), 0, 1)
        n = 1
        for s_ in sizes:
            n *= s_
        offset += n
    return total / len(leaves)


def variant_paths_with_traffic(p, index: int, demand_mqps: int):
    """Per root-to-leaf task path: the variant paths (one variant per task) every hop of which carries
    requests -- I(p) = 1 in the paper's Table 1.  Taken from the intervals of placement(): a downstream
    variant gets requests from an upstream one exactly when their intervals of the downstream task's request
    stream overlap in more than a point.  At zero demand the path of the first hosted variants."""
    tasks, plan, demand, spans, created = placement(p, index, demand_mqps)
    leaves = [i for i in range(len(tasks)) if all(t["parent"] != i for t in tasks)]

    def by_accuracy(i, ks):
        return sorted(ks, key=lambda k: (-tasks[i]["variants"][k]["acc"], k))

    def upstream_span(i, par, kp):
        order = by_accuracy(par, created[par])
        lo = sum((created[par][k] for k in order[:order.index(kp)]), Fraction(0)) * tasks[i]["fan"]
        return lo, lo + created[par][kp] * tasks[i]["fan"]

    out = []
    for leaf in leaves:
        path, i = [], leaf
        while i >= 0:
            path.append(i)
            i = tasks[i]["parent"]
        path = path[::-1]
        found = []

        def walk(depth, chosen):
            i = path[depth]
            if depth == 0:
                lo, hi = Fraction(0), demand[0]
            else:
                lo, hi = upstream_span(i, path[depth - 1], chosen[-1])
            if hi == lo:
                hosted = by_accuracy(i, [k for k in range(len(plan[i][0])) if plan[i][0][k] > 0])
                nxt = hosted[:1]
            else:
                nxt = [k for k, (a, b) in spans[i].items() if min(b, hi) - max(a, lo) > 0]
            for k in nxt:
                if depth == len(path) - 1:
                    found.append(tuple(chosen + [k]))
                else:
                    walk(depth + 1, chosen + [k])

        walk(0, [])
        out.append((path, found))
    return out


def slow_path_with_traffic(p, index: int, demand_mqps: int, slo_us: int, comm_us: int) -> bool:
    tasks = _tables(p)
    plan = decode(p, index)
    for path, found in variant_paths_with_traffic(p, index, demand_mqps):
        room = slo_us - comm_us * len(path)
        if room < 0:
            return True
        for ks in found:
            if sum(tasks[i]["variants"][k]["lat"][plan[i][1][k]] for i, k in zip(path, ks)) > room // 2:
                return True
    return False
