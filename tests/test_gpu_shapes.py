"""GPU parity on shapes that take the less travelled paths of the tabulated kernel."""
import os
import random
import struct
from types import SimpleNamespace

import pytest

import oracle
from paper_2407_03583_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

TIE, LANE = binding.LOKI_TIE_INDEX_ONLY, binding.LOKI_SEARCH_PER_LANE


def bits(x):
    return struct.unpack("<Q", struct.pack("<d", x))[0]


def agree(res, ref):
    got, want = res.as_tuple(), ref.as_tuple()
    return got[0] == want[0] and bits(got[1]) == bits(want[1]) and got[2:] == want[2:]


def profile(rng, k, batches):
    acc = [rng.randint(600000, 950000) for _ in range(k)]
    lat, thr = [], []
    for _ in range(k):
        l0, l1 = rng.randint(2000, 10000), rng.randint(1000, 20000)
        for b in batches:
            lat.append(l0 + l1 * b)
            thr.append(b * 10**9 // (l0 + l1 * b))
    return acc, lat, thr


def test_root_task_with_more_buckets_than_the_ordering_kernel_holds():
    """Root: 2 variants x 256 replica counts x 5 batch sizes = 327,680 choices and 511 x 10 + 1
    (replicas, latency) classes, which exceeds the ordering kernel's histogram: identity order."""
    rng = random.Random(5)
    a0, l0, t0 = profile(rng, 2, [1, 2, 4, 8, 16])
    a1, l1, t1 = profile(rng, 1, [4])
    p = SimpleNamespace(n_tasks=2, parent=[-1, 0], fanout_q4=[4, 6], n_variants=[2, 1], n_batches=[5, 1],
                        batch_size=[1, 2, 4, 8, 16, 4], max_replicas=[255, 255, 1], acc_ppm=a0 + a1,
                        latency_us=l0 + l1, thr_mqps=t0 + t1)
    P, O = binding.Problem(p), oracle.Problem(p)
    assert P.num_candidates() == 327680 * 2
    for demand, W in ((30_000, 20), (150_000, 300), (0, 511)):
        for flags in (0, TIE):
            res = P.alloc_search([demand], W, 400_000, flags=flags)[0]
            ref = O.search(demand, W, 400_000, tie_index_only=bool(flags & TIE))
            assert agree(res, ref), (demand, W, flags, res.as_tuple(), ref.as_tuple())


def test_seven_leaf_star_uses_the_true_division():
    """Root with 7 children: 7 paths (not a power of two), so the mean over paths is a real division."""
    rng = random.Random(9)
    n = 8
    acc, lat, thr, nv, nb, bs, rep = [], [], [], [], [], [], []
    for i in range(n):
        a, l, t = profile(rng, 2, [1, 4])
        acc += a
        lat += l
        thr += t
        nv.append(2)
        nb.append(2)
        bs += [1, 4]
        rep += [1, 1]
    p = SimpleNamespace(n_tasks=n, parent=[-1] + [0] * 7, fanout_q4=[4] + [rng.randint(2, 6) for _ in range(7)],
                        n_variants=nv, n_batches=nb, batch_size=bs, max_replicas=rep, acc_ppm=acc,
                        latency_us=lat, thr_mqps=thr)
    P, O = binding.Problem(p), oracle.Problem(p)
    assert P.num_candidates() == 8 ** 8  # 16.7M
    for demand in (0, 20_000, 45_000):
        ref = O.search(demand, 12, 300_000)
        for flags in (0, LANE):
            res = P.alloc_search([demand], 12, 300_000, flags=flags)[0]
            assert agree(res, ref), (demand, flags, res.as_tuple(), ref.as_tuple())
    # three leaves below a two-level tree, with ranges cutting through the last task's choices
    p3 = SimpleNamespace(n_tasks=5, parent=[-1, 0, 1, 1, 0], fanout_q4=[4, 5, 6, 4, 9],
                         n_variants=nv[:5], n_batches=nb[:5], batch_size=bs[:10], max_replicas=[2] * 10,
                         acc_ppm=acc[:10], latency_us=lat[:20], thr_mqps=thr[:20])
    P, O = binding.Problem(p3), oracle.Problem(p3)
    nn = P.num_candidates()
    assert nn == 18 ** 5
    for lo, hi in ((0, nn), (12345, 1_000_000), (nn - 700_001, nn - 1)):
        ref = O.search(25_000, 9, 250_000, begin=lo, end=hi)
        for flags in (0, LANE, TIE):
            if flags & TIE:
                ref = O.search(25_000, 9, 250_000, begin=lo, end=hi, tie_index_only=True)
            res = P.alloc_search([25_000], 9, 250_000, flags=flags, begin=lo, end=hi)[0]
            assert agree(res, ref), (lo, hi, flags, res.as_tuple(), ref.as_tuple())


def test_deep_chain_of_eight_tasks():
    rng = random.Random(21)
    acc, lat, thr = [], [], []
    for i in range(8):
        a, l, t = profile(rng, 2, [2])
        acc += a
        lat += [v // 4 for v in l]
        thr += [v * 40 for v in t]
    p = SimpleNamespace(n_tasks=8, parent=[-1, 0, 1, 2, 3, 4, 5, 6], fanout_q4=[4, 5, 4, 6, 4, 5, 4, 4],
                        n_variants=[2] * 8, n_batches=[1] * 8, batch_size=[2] * 8, max_replicas=[1, 2] * 8,
                        acc_ppm=acc, latency_us=lat, thr_mqps=thr)
    P, O = binding.Problem(p), oracle.Problem(p)
    assert P.num_candidates() == 6 ** 8
    for demand, W, comm in ((10_000, 12, 0), (200_000, 20, 500), (0, 8, 0)):
        ref = O.search(demand, W, 200_000, comm)
        for flags in (0, LANE):
            res = P.alloc_search([demand], W, 200_000, comm, flags=flags)[0]
            assert agree(res, ref), (demand, W, flags, res.as_tuple(), ref.as_tuple())


def test_every_tile_length_with_a_ragged_last_tile():
    """The launch shortens the tile of root-task choices when a call has few work items.  One chain,
    root with 7 x 10 x 9 x 3 = 1,890 choices, searched for 1, 10 and 24 demand points: the calls land on
    tiles of 256 entries (one point) and of 512 (the library's thresholds), each with several tiles and a
    last tile that is not full."""
    rng = random.Random(33)
    a0, l0, t0 = profile(rng, 3, [1, 2, 4])
    a1, l1, t1 = profile(rng, 2, [2, 8])
    a2, l2, t2 = profile(rng, 2, [4])
    p = SimpleNamespace(n_tasks=3, parent=[-1, 0, 1], fanout_q4=[4, 5, 6], n_variants=[3, 2, 2],
                        n_batches=[3, 2, 1], batch_size=[1, 2, 4, 2, 8, 4], max_replicas=[6, 9, 8, 11, 11, 5, 6],
                        acc_ppm=a0 + a1 + a2, latency_us=l0 + l1 + l2, thr_mqps=t0 + t1 + t2)
    P, O = binding.Problem(p), oracle.Problem(p)
    assert P.num_candidates() == (7 * 10 * 9 * 3) * (12 * 12 * 2) * (6 * 7)   # root: 1,890 choices
    for n_points in (1, 10, 24):
        demands = [rng.randint(5_000, 700_000) for _ in range(n_points)]
        for flags in (0, TIE):
            out = P.alloc_search(demands, 40, 300_000, flags=flags)
            for d, res in list(zip(demands, out))[:: max(1, n_points // 4)]:
                ref = O.search_tabulated(d, 40, 300_000, tie_index_only=bool(flags & TIE))
                assert agree(res, ref), (n_points, d, flags, res.as_tuple(), ref.as_tuple())


def test_many_demand_points_in_one_call():
    w = wl.config(1)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    rng = random.Random(2)
    demands = [rng.randint(0, 260_000) for _ in range(3000)]
    out = P.alloc_search(demands, w.workers, w.slo_us)
    for d, res in list(zip(demands, out))[::37]:
        assert agree(res, O.search(d, w.workers, w.slo_us)), d
    # monotone in demand across the whole sweep (a property that needs no checker)
    order = sorted(range(len(demands)), key=lambda i: demands[i])
    accs = [out[i].accuracy if out[i].status == 0 else -1.0 for i in order]
    assert all(a >= b for a, b in zip(accs, accs[1:]))


def test_plan_space_of_two_to_the_62_searched_by_ranges():
    """Three tasks with 2^20, 2^21 and 2^21 choices: 2^62 plans, just below the library's limit.  Ranges
    at the bottom, across a carry of the last task's choice, and at the very top, through both kernels;
    the 64-bit index arithmetic is what is being checked."""
    rng = random.Random(62)
    acc, lat, thr, bs = [], [], [], []
    for i, batches in enumerate(([2], [1, 4], [2, 8])):
        a, l, t = profile(rng, 5, batches)
        acc += a
        lat += [v // 8 for v in l]
        thr += [v * (30 if i else 10) for v in t]
        bs += batches
    p = SimpleNamespace(n_tasks=3, parent=[-1, 0, 0], fanout_q4=[4, 6, 9], n_variants=[5, 5, 5], n_batches=[1, 2, 2],
                        batch_size=bs, max_replicas=[15] * 15, acc_ppm=acc, latency_us=lat, thr_mqps=thr)
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    assert n == 1 << 62
    stride_last = 1 << 41
    span = 1 << 17
    found = 0
    for begin in (0, 5 * stride_last - span // 2, (1 << 61) + 987_654_321, n - span):
        for flags in (0, LANE):
            res = P.alloc_search([900_000], 400, 400_000, flags=flags, begin=begin, end=begin + span)[0]
            ref = O.search(900_000, 400, 400_000, begin=begin, end=begin + span)
            assert agree(res, ref), (begin, flags, res.as_tuple(), ref.as_tuple())
        found += ref.found
    assert found >= 2
    idxs = [0, 1, n - 1, n - 2, (1 << 61) + 1, 3 * stride_last - 1, 3 * stride_last]
    for got, idx in zip(P.alloc_eval(idxs, 900_000, 400, 400_000), idxs):
        e = O.eval(idx, 900_000, 400, 400_000)
        assert (got.infeasible, got.workers, bits(got.accuracy)) == (e.infeasible, e.workers, bits(e.accuracy)), idx


def test_the_most_choices_a_task_may_have():
    """2^24 choices in one task (six variants, up to 15 replicas each): alone, and as the first task of a
    chain, where the ordering kernel sorts all of them into runs."""
    rng = random.Random(24)
    a0, l0, t0 = profile(rng, 6, [4])
    a1, l1, t1 = profile(rng, 1, [1, 2])
    one = SimpleNamespace(n_tasks=1, parent=[-1], fanout_q4=[4], n_variants=[6], n_batches=[1], batch_size=[4],
                          max_replicas=[15] * 6, acc_ppm=a0, latency_us=l0, thr_mqps=t0)
    two = SimpleNamespace(n_tasks=2, parent=[-1, 0], fanout_q4=[4, 5], n_variants=[6, 1], n_batches=[1, 2],
                          batch_size=[4, 1, 2], max_replicas=[15] * 6 + [3], acc_ppm=a0 + a1, latency_us=l0 + l1,
                          thr_mqps=t0 + [40 * v for v in t1])
    for p, n in ((one, 1 << 24), (two, 1 << 27)):
        P, O = binding.Problem(p), oracle.Problem(p)
        assert P.num_candidates() == n
        for demand, W in ((2_500_000, 40), (400_000, 93)):
            for flags in (0, TIE):
                res = P.alloc_search([demand], W, 300_000, flags=flags)[0]
                ref = O.search_tabulated(demand, W, 300_000, tie_index_only=bool(flags & TIE))
                assert agree(res, ref), (n, demand, flags, res.as_tuple(), ref.as_tuple())
            assert ref.found


def test_the_largest_number_of_demand_points():
    """65,535 demand points (the limit of one call) on config 1."""
    w = wl.config(1)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    rng = random.Random(8)
    demands = [rng.randint(0, 300_000) for _ in range(65_535)]
    out = P.alloc_search(demands, w.workers, w.slo_us)
    assert len(out) == 65_535
    for j in list(range(0, 65_535, 1111)) + [65_534]:
        assert agree(out[j], O.search(demands[j], w.workers, w.slo_us)), j
    order = sorted(range(len(demands)), key=lambda i: demands[i])
    accs = [out[i].accuracy if out[i].status == 0 else -1.0 for i in order]
    assert all(a >= b for a, b in zip(accs, accs[1:]))
    with pytest.raises(binding.LokiError):
        P.alloc_search(demands + [1], w.workers, w.slo_us)


def test_valu_rate_measurement_is_plausible():
    nominal = 256 * 4 * 2.4e9 / 4          # wavefront instructions per second at one per SIMD per 4 cycles
    # classes that issue at the full rate; the 32-bit integer streams have been seen above the nominal figure
    full = {"v_mul_f64": 1.05, "v_add_f64": 1.05, "v_max_f64": 1.05, "search_mix": 1.05, "v_fma_f64": 1.05,
            "v_add_u32": 1.4, "v_min_u32": 1.4}
    for kind in binding.RATE_KINDS:
        rate = binding.measure_valu_rate(kind)
        print(kind, rate / nominal)
        if kind in full:
            assert 0.5 * nominal < rate < full[kind] * nominal, (kind, rate)
        else:   # 32-bit multiplies, the fp64 reciprocal, LDS reads: slower classes, never faster than the full rate
            assert 0.02 * nominal < rate < 1.05 * nominal, (kind, rate)


def test_objective_operation_order_on_the_gpu():
    """Cases where root-first and leaf-first products (and forward and reverse leaf sums) differ in the last bit."""
    def simple(parent, accs):
        n = len(accs)
        return SimpleNamespace(n_tasks=n, parent=parent, fanout_q4=[4] * n, n_variants=[1] * n, n_batches=[1] * n,
                               batch_size=[1] * n, max_replicas=[1] * n, acc_ppm=accs, latency_us=[1000] * n,
                               thr_mqps=[10**9] * n)
    for p in (simple([-1, 0, 1], [600000, 661725, 772830]), simple([-1, 0, 0, 0], [800000, 600000, 661725, 735795]),
              simple([-1, 0, 1, 1, 0], [800000, 600000, 661725, 735795, 772830])):
        P, O = binding.Problem(p), oracle.Problem(p)
        ref = O.search(1000, 8, 100_000)
        assert ref.found == 1
        for flags in (0, LANE):
            res = P.alloc_search([1000], 8, 100_000, flags=flags)[0]
            assert agree(res, ref), (flags, res.as_tuple(), ref.as_tuple())


def test_values_at_the_ends_of_their_ranges():
    """Eight variants and eight batch sizes in one task, 255 replicas of a single variant in another, a
    fan-out of 1024.00, the largest latency and throughputs that pass the range proof, accuracies 0 and 1."""
    rng = random.Random(99)
    # task 0: 8 variants x up to 3 replicas x 8 batch sizes = 524,288 choices
    acc0 = [0, 1_000_000] + [rng.randint(1, 999_999) for _ in range(6)]
    lat0, thr0 = [], []
    for k in range(8):
        for b in range(8):
            lat0.append(rng.randint(1, 40_000))
            thr0.append(rng.randint(0, 3_000_000))
    # task 1: one variant, 0..255 replicas, two batch sizes; fan-out 4096 quarters
    lat1 = [1 << 30, 1000]
    thr1 = [(1 << 40), 9_000_000]
    p = SimpleNamespace(n_tasks=2, parent=[-1, 0], fanout_q4=[4, 4096], n_variants=[8, 1], n_batches=[8, 2],
                        batch_size=[1, 2, 3, 5, 8, 13, 21, 34, 1, 64], max_replicas=[3] * 8 + [255],
                        acc_ppm=acc0 + [777_777], latency_us=lat0 + lat1, thr_mqps=thr0 + thr1)
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    assert n == (4 ** 8 * 8) * (256 * 2)
    idxs = [0, n - 1] + [rng.randrange(n) for _ in range(4000)]
    for demand, W, slo in ((2_000_000, 300, 2 * ((1 << 30) + 50_000)), (1_000, 20, 100_000), (0, 9, 90_000)):
        for got, idx in zip(P.alloc_eval(idxs, demand, W, slo), idxs):
            e = O.eval(idx, demand, W, slo)
            assert (got.infeasible, got.workers, bits(got.accuracy)) == (e.infeasible, e.workers, bits(e.accuracy)), idx
        for flags in (0, TIE, LANE):
            res = P.alloc_search([demand], W, slo, flags=flags)[0]
            ref = O.search_tabulated(demand, W, slo, tie_index_only=bool(flags & TIE))
            assert agree(res, ref), (demand, flags, res.as_tuple(), ref.as_tuple())


def test_handles_can_be_created_used_and_destroyed_many_times():
    """Every handle owns pinned staging memory and events: 200 handles, each used once and closed, and
    several handles used alternately on one stream, give the same answers throughout."""
    w1, w2 = wl.config(1), wl.random_small(5)
    ref1 = oracle.Problem(w1.pipeline).search(w1.demand_mqps[0], w1.workers, w1.slo_us)
    ref2 = oracle.Problem(w2.pipeline).search(w2.demand_mqps[0], w2.workers, w2.slo_us, w2.comm_us)
    for _ in range(200):
        P = binding.Problem(w1.pipeline)
        assert agree(P.alloc_search(w1.demand_mqps, w1.workers, w1.slo_us)[0], ref1)
        P.close()
    a, b, c = binding.Problem(w1.pipeline), binding.Problem(w2.pipeline), binding.Problem(w1.pipeline)
    for _ in range(20):
        assert agree(a.alloc_search(w1.demand_mqps, w1.workers, w1.slo_us)[0], ref1)
        assert agree(b.alloc_search(w2.demand_mqps, w2.workers, w2.slo_us, w2.comm_us)[0], ref2)
        assert agree(c.alloc_search(w1.demand_mqps, w1.workers, w1.slo_us, flags=LANE)[0], ref1)
    for h in (a, b, c):
        h.close()
        h.close()   # closing twice is harmless


def test_bench_prints_one_json_line_with_the_agreed_fields():
    """bench.py end to end on the smallest configuration, plain and with the optional parts of the model."""
    import json
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for extra, kernel in (([], "tabulated"), (["--variant-factors"], "tabulated_by_class"),
                          (["--path-tables"], "tabulated_paths"), (["--per-lane"], "per_lane"),
                          (["--variant-factors", "--path-tables"], "tabulated_by_class_paths")):
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--config", "1", "--steps", "2", "--warmup", "1",
                            "--no-cpu-baseline", "--no-context"] + extra, capture_output=True, text=True, timeout=300)
        assert r.returncode == 0, r.stderr[-2000:]
        lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
        assert len(lines) == 1
        d = json.loads(lines[0])
        for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                    "vs_baseline", "dtype", "data", "config", "roofline"):
            assert key in d, key
        assert d["n_gpus"] == 1 and d["steps"] == 2 and d["vs_baseline"] is None and d["data"] == "synthetic"
        assert d["config"]["kernel"] == kernel and d["config"]["workload"].startswith("cfg1_")
        assert d["value"] > 0 and d["ms_per_step"] > 0
        assert d["roofline"]["bound"] == "alu" and set(("achieved", "peak", "unit", "frac", "traffic")) <= set(d["roofline"])
