"""The host side of the library (validation, layouts, batching, the class walk, staging) built for the CPU
with AddressSanitizer and UndefinedBehaviorSanitizer and driven through its C-ABI.

tests/host_sanitize/hip_stubs.cpp stands in for the HIP runtime and for the kernel launches (a launch writes
every array its kernel would write, so a layout that is too small is an ASan report); tests/host_sanitize/
driver.cpp reads one problem from a text file, runs every entry point over it and prints what the host
computes itself, which is compared with the CPU checker here.  No GPU."""
import itertools
import os
import random
import subprocess
from types import SimpleNamespace

import pytest

import oracle
from paper_2407_03583_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "host_sanitize")
CSRC = os.path.join(ROOT, "paper_2407_03583_amd", "csrc")


def build_driver(exe, *defines):
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-Wall", "-Wextra",
           "-Wno-unused-parameter", "-Wno-deprecated-declarations", *defines,
           os.path.join(CSRC, "loki_api.cpp"), os.path.join(SAN, "hip_stubs.cpp"), os.path.join(SAN, "driver.cpp"),
           "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    return exe


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    return build_driver(str(tmp_path_factory.mktemp("host_sanitize") / "driver"))


def write_problem(path, p, demands, workers, slo, comm, indices, ranges):
    vf = getattr(p, "variant_factor_q4", None)
    pt = getattr(p, "path_acc_ppm", None)
    lists = [[p.n_tasks, 1 if getattr(p, "per_variant_batch", False) else 0, 1 if vf is not None else 0,
              1 if pt is not None else 0, workers, slo, comm, 1 if getattr(p, "latency_per_path", False) else 0],
             p.parent, p.fanout_q4, p.n_variants, p.n_batches, p.batch_size, p.max_replicas, p.acc_ppm,
             p.latency_us, p.thr_mqps, vf or [], pt or [], demands, indices, ranges]
    with open(path, "w") as f:
        for lst in lists:
            f.write(" ".join(str(int(v)) for v in [len(lst)] + list(lst)) + "\n")


def run(driver, tmp_path, p, demands, workers, slo, comm=0, indices=(), ranges=()):
    spec = str(tmp_path / "problem.txt")
    write_problem(spec, p, list(demands), workers, slo, comm, list(indices), list(ranges))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)   # the sanitizer runtime has to come first in the process
    r = subprocess.run([driver, spec], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, (r.stdout[-1500:], r.stderr[-3000:])
    assert r.stdout.rstrip().endswith("done") or "create -" in r.stdout, r.stdout[-500:]
    return r.stdout.splitlines()


def check_host_outputs(lines, p, demand, indices):
    """Decoded plans and routing tables of the sanitized build against the CPU checker."""
    O = oracle.Problem(p)
    dec = [ln.split() for ln in lines if ln.startswith("decode 0 ")]
    routes = [ln.split() for ln in lines if ln.startswith("route 0")]
    assert len(dec) == len(indices) == len(routes)
    off_b, batches = [], p.batch_size
    for idx, d, r in zip(indices, dec, routes):
        x, beta = O.decode(idx)
        bar = d.index("|")
        assert [int(v) for v in d[3:bar]] == x
        got_b = [int(v) for v in d[bar + 1:]]
        if not getattr(p, "per_variant_batch", False):
            off = 0
            for i in range(p.n_tasks):
                assert got_b[i] == batches[off + beta[i]]
                off += p.n_batches[i]
        rt = O.route_table(idx, demand)
        want = []
        for i in range(p.n_tasks):
            for k in range(p.n_variants[i]):
                want.append(f"{rt.routed[i][k]}:{rt.leftover[i][k]}")
        assert r[2:] == want, (idx, r[2:], want)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_benchmark_configurations_run_clean(driver, tmp_path, cfg):
    w = wl.config(cfg)
    n = w.pipeline.num_candidates()
    rng = random.Random(cfg)
    indices = [0, 1, n - 1, n // 2, n // 3 + 7] + [rng.randrange(n) for _ in range(20)]
    c0 = w.pipeline.max_replicas and 1
    strideL = n // (w.pipeline.n_batches[-1] * (max(w.pipeline.max_replicas) + 1) ** w.pipeline.n_variants[-1])
    ranges = [0, 1, n - 1, n, n // 3, n // 3 + 12345, strideL - 5, strideL + 777, n // 2, n // 2, 17, 17 + strideL // 2]
    demands = w.demand_mqps[:70]
    lines = run(driver, tmp_path, w.pipeline, demands, w.workers, w.slo_us, w.comm_us, indices, ranges)
    assert f"candidates 0 {n}" in lines
    assert all("rc 0" in ln for ln in lines if ln.startswith(("search", "range")))
    assert {"too small -4", "misaligned -4", "reversed -6", "negative demand -3", "huge demand -3"} <= set(lines)
    assert "enqueue 0" in lines and "trace 0" in lines and "eval 0" in lines and "route batch 0" in lines
    check_host_outputs(lines, w.pipeline, demands[0], indices)


@pytest.mark.parametrize("what", ["variant_factors", "per_variant_batch", "path_tables", "complete_model",
                                  "latency_per_path", "latency_per_path_complete_model"])
@pytest.mark.parametrize("cfg", [2, 4, 5])
def test_model_variants_run_clean(driver, tmp_path, cfg, what):
    """Per-variant factors run class by class on the host: the walk over the classes, the batches of points,
    their descriptors and the merge arguments all go through the sanitizers."""
    w = wl.config(cfg)
    p = w.pipeline
    if what.startswith("latency_per_path"):   # on the tables with the second kernel, or whole plans per lane
        p.latency_per_path = True
        what = what[len("latency_per_path_"):]
    if what in ("variant_factors", "complete_model"):
        p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]
    if what == "per_variant_batch":
        p.per_variant_batch = True
        p.max_replicas = [1] * len(p.max_replicas)   # keeps the per-variant plan space of 5^4 choices per task small
    if what in ("path_tables", "complete_model"):
        p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(w.seed + 1))
    n = p.num_candidates()
    rng = random.Random(cfg)
    indices = [0, n - 1] + [rng.randrange(n) for _ in range(10)]
    demands = sorted(set(w.demand_mqps))[:40] if cfg == 4 else [w.demand_mqps[0], w.demand_mqps[0] // 3, 0]
    lines = run(driver, tmp_path, p, demands, w.workers, w.slo_us, w.comm_us, indices, [0, n // 2, n // 5, n // 5 + 99999])
    assert all("rc 0" in ln for ln in lines if ln.startswith(("search", "range")))
    check_host_outputs(lines, p, demands[0], indices)


def plans_with_usable_inner_choices(p, demand):
    """Plans in which every task that has children serves all the demand its ancestors' choices create for it
    (eq. (1) with per-variant factors, eq. (2) with most-accurate-first filling): what a class-by-class search
    hands to the kernels.  Plain enumeration over the choices, task by task, in exact integers."""
    n = p.n_tasks
    voff = [sum(p.n_variants[:i]) for i in range(n + 1)]
    boff = [0]
    for i in range(n):
        boff.append(boff[-1] + p.n_variants[i] * p.n_batches[i])
    depth = [0] * n
    for i in range(1, n):
        depth[i] = depth[p.parent[i]] + 1
    has_children = [i in p.parent for i in range(n)]
    pv = getattr(p, "per_variant_batch", False)

    def choices(i):
        """(replicas, batch position) per variant for every choice of task i."""
        K, nb = p.n_variants[i], p.n_batches[i]
        R = p.max_replicas[voff[i]:voff[i + 1]]
        per_variant = [[(0, 0)] + [(x, b) for x in range(1, R[k] + 1) for b in range(nb)] for k in range(K)] if pv else None
        if pv:
            return [list(c) for c in itertools.product(*per_variant)]
        return [[(x, b) for x in xs] for b in range(nb) for xs in itertools.product(*[range(R[k] + 1) for k in range(K)])]

    def created(i, choice, D):
        """None if the choice cannot serve D; else what it creates per unit of a child's fan-out."""
        K, nb = p.n_variants[i], p.n_batches[i]
        order = sorted(range(K), key=lambda k: (-p.acc_ppm[voff[i] + k], k))
        rem, out, any_hosted = D, 0, False
        for k in order:
            x, b = choice[k]
            if x == 0:
                continue
            any_hosted = True
            cap = x * p.thr_mqps[boff[i] + k * nb + b] * 16 ** depth[i]
            routed = min(rem, cap)
            out += routed * p.variant_factor_q4[voff[i] + k]
            rem -= routed
        return out if any_hosted and rem == 0 else None

    all_choices = [choices(i) for i in range(n)]

    def count(i, demand_of):
        if i == n:
            return 1
        D = demand_of[i]
        if not has_children[i]:
            return len(all_choices[i]) * count(i + 1, demand_of)
        by_amount = {}
        for c in all_choices[i]:
            out = created(i, c, D)
            if out is not None:
                by_amount[out] = by_amount.get(out, 0) + 1
        total = 0
        for out, members in by_amount.items():
            nxt = dict(demand_of)
            for j in range(i + 1, n):
                if p.parent[j] == i:
                    nxt[j] = out * p.fanout_q4[j]
            total += members * count(i + 1, nxt)
        return total

    return count(0, {0: demand})


def test_class_counts_against_plain_enumeration(driver, tmp_path):
    """The host finds the classes of a task from a walk over the tree of its variants' digits; the number of
    plans it hands to the kernels (loki_last_search_plans_scored) must be the number of plans whose tasks with
    children can all serve their demand, counted here choice by choice."""
    by_class = 0
    for seed in range(40):
        w = wl.random_small(seed, max_candidates=6000, variant_factors=True, per_variant_batch=seed % 3 == 2)
        p = w.pipeline
        n = p.num_candidates()
        demands = [w.demand_mqps[0], w.demand_mqps[0] // 2, 0]
        lines = run(driver, tmp_path, p, demands, w.workers, w.slo_us, w.comm_us)
        scored = [int(ln.split()[2]) for ln in lines if ln.startswith("scored 0 ")]
        assert len(scored) == 4
        want = sum(plans_with_usable_inner_choices(p, d) for d in demands)
        # flags 0 and 1: class by class where the problem allows it; 2 and 3: whole plans per lane
        assert scored[2] == scored[3] == n * len(demands)
        assert scored[0] == scored[1] and scored[0] in (want, n * len(demands)), (seed, scored, want, n)
        by_class += scored[0] == want and want != n * len(demands)
    assert by_class >= 10, by_class


def test_limit_cases_run_clean(driver, tmp_path):
    """The extremes the interface allows: 2^24 choices of one task, a plan space of 2^62, 65,535 demand
    points, 8 tasks of 8 variants, and a task whose choices do not fit the ordering kernel's buckets."""
    rng = random.Random(3)

    def prof(k, nb):
        lat, thr = [], []
        for _ in range(k):
            l0, l1 = rng.randint(2000, 10000), rng.randint(1000, 20000)
            for b in range(nb):
                lat.append(l0 + l1 * (b + 1))
                thr.append((b + 1) * 10 ** 9 // (l0 + l1 * (b + 1)))
        return lat, thr

    # one task with 2^24 choices (8 variants x radix 8), 65,535 demand points
    lat, thr = prof(8, 1)
    p = SimpleNamespace(n_tasks=1, parent=[-1], fanout_q4=[4], n_variants=[8], n_batches=[1], batch_size=[1],
                        max_replicas=[7] * 8, acc_ppm=[600000 + 1000 * k for k in range(8)], latency_us=lat, thr_mqps=thr)
    assert p.n_variants[0] == 8
    lines = run(driver, tmp_path, p, [30_000, 0], 30, 200_000, 0, [0, (1 << 24) - 1, 12345], [5, (1 << 24) - 3])
    assert "candidates 0 16777216" in lines and all("rc 0" in ln for ln in lines if ln.startswith(("search", "range")))
    # 65,535 demand points (the most a call takes) on config 1's 65,536 plans
    w = wl.config(1)
    lines = run(driver, tmp_path, w.pipeline, [1000 * (m % 977) for m in range(65535)], w.workers, w.slo_us, 0, [0], [3, 999])
    assert all("rc 0" in ln for ln in lines if ln.startswith(("search", "range")))
    # a plan space of 2^62: 8 tasks, 2 variants of up to 15 replicas and 2 batch sizes, 2^9 choices each -> 2^72 is
    # refused; 6 such tasks and two of 2^4 -> 2^62
    nv, nbs, bsz, rep, acc, lats, thrs = [], [], [], [], [], [], []
    for i in range(8):
        big = i < 6
        nv.append(2)
        nbs.append(2 if big else 1)
        bsz += [1, 4] if big else [2]
        rep += [15, 15] if big else [3, 3]
        acc += [700000, 900000]
        l, t = prof(2, 2 if big else 1)
        lats += l
        thrs += t
    p = SimpleNamespace(n_tasks=8, parent=[-1, 0, 1, 2, 3, 4, 5, 6], fanout_q4=[4] * 8, n_variants=nv, n_batches=nbs,
                        batch_size=bsz, max_replicas=rep, acc_ppm=acc, latency_us=lats, thr_mqps=thrs)
    n = p_candidates = (2 ** 9) ** 6 * 16 * 16
    assert n == 1 << 62
    lines = run(driver, tmp_path, p, [50_000, 0], 100, 10 ** 7, 0, [0, n - 1, n // 7],
                [n // 3, n // 3 + (1 << 17), n - (1 << 20), n])
    assert f"candidates 0 {n}" in lines
    assert all("rc 0" in ln for ln in lines if ln.startswith("range"))
    # a first task with 2 x 256 replica counts x 5 batch sizes: more (replicas, latency) classes than buckets
    lat, thr = prof(2, 5)
    l1, t1 = prof(1, 1)
    p = SimpleNamespace(n_tasks=2, parent=[-1, 0], fanout_q4=[4, 6], n_variants=[2, 1], n_batches=[5, 1],
                        batch_size=[1, 2, 4, 8, 16, 4], max_replicas=[255, 255, 1], acc_ppm=[700000, 800000, 900000],
                        latency_us=lat + l1, thr_mqps=thr + t1)
    lines = run(driver, tmp_path, p, [30_000], 300, 400_000, 0, [0, 327680 * 2 - 1], [7, 327680])
    assert "candidates 0 655360" in lines
    # refused at creation: 2^72 plans, 257 replicas, a throughput that would overflow once scaled to a deep task
    for change, rc in ((dict(n_tasks=1, parent=[-1], fanout_q4=[4], n_variants=[1], n_batches=[1], batch_size=[1],
                             max_replicas=[256], acc_ppm=[1], latency_us=[5], thr_mqps=[5]), -3),):
        lines = run(driver, tmp_path, SimpleNamespace(**change), [1], 1, 100, 0, [], [])
        assert lines[0] == f"create {rc}"
    deep = SimpleNamespace(n_tasks=8, parent=[-1, 0, 1, 2, 3, 4, 5, 6], fanout_q4=[4] * 8, n_variants=[1] * 8,
                           n_batches=[1] * 8, batch_size=[1] * 8, max_replicas=[1] * 8, acc_ppm=[900000] * 8,
                           latency_us=[1000] * 8, thr_mqps=[1 << 40] * 8)
    assert run(driver, tmp_path, deep, [1], 8, 10 ** 6, 0, [], [])[0] == "create 0"      # 2^40 * 4^7 = 2^54: the limit
    deep.variant_factor_q4 = [4] * 8                                                    # units of 1 / 16^depth: 2^68
    assert run(driver, tmp_path, deep, [1], 8, 10 ** 6, 0, [], [])[0] == "create -3"


def test_bad_demand_in_a_later_group_leaves_nothing_behind(driver, tmp_path):
    """Class-by-class searches take the demand points in groups; a demand that is out of range in a later
    group is found before the first group is enqueued (the call returns LOKI_E_RANGE)."""
    w = wl.config(4)
    p = w.pipeline
    p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]
    demands = sorted(set(w.demand_mqps))[:30]
    lines = run(driver, tmp_path, p, demands, w.workers, w.slo_us, 0, [0], [])
    assert "negative demand -3" in lines and "huge demand -3" in lines


def test_demand_point_with_more_points_than_the_descriptors_hold(tmp_path):
    """A build of the host side whose descriptor arrays hold 40 (demand point, classes) points instead of
    65,535.  Config 4's tree with factors has from a handful to more than 100 points per demand point: a call whose first demand
    point stays below 40 and whose second exceeds it takes the first class by class, then the second per
    lane into its own result slot, then goes on class by class; a call whose first point exceeds it falls
    back per lane as a whole.  (The stand-in for the final merge writes "nothing found", status 1, where the
    per-lane search's merge would write; the class-by-class merge's stand-in leaves 0x5a5a5a5a.)"""
    exe = build_driver(str(tmp_path / "driver_small"), "-DLOKI_CLASS_POINTS_LIMIT=40")
    w = wl.config(4)
    p = w.pipeline
    p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]
    n = p.num_candidates()
    few, many = 2_900_000, 500_000     # a handful of points at 2,900 QPS, more than 100 at 500 QPS
    untouched = str(0x5a5a5a5a)
    lines = run(exe, tmp_path, p, [few, many, few], w.workers, w.slo_us, 0, [0], [])
    first = [ln for ln in lines if ln.startswith("search flags 0 ")][0].split()
    assert first[4] == "0" and first[6:9] == [untouched, "1", untouched], first
    scored = [ln for ln in lines if ln.startswith("scored 0 ")][0].split()
    assert n <= int(scored[2]) < 3 * n         # one demand point per lane (n plans) plus the classes of the two others
    lines = run(exe, tmp_path, p, [many, few], w.workers, w.slo_us, 0, [0], [])
    first = [ln for ln in lines if ln.startswith("search flags 0 ")][0].split()
    assert first[4] == "0" and first[6:8] == ["1", "1"], first
    assert [ln for ln in lines if ln.startswith("scored 0 ")][0].split()[2] == str(2 * n)
