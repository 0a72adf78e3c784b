"""GPU parity: the HIP library (through its C-ABI) against the CPU checker on
the same seeded inputs.  Integer outputs and the fp64 objective must match bit
for bit (both sides take every decision in int64 / individually rounded fp64)."""
import json
import os
import random
import struct
from types import SimpleNamespace

import pytest

import oracle
from paper_2407_03583_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
TIE, LANE = binding.LOKI_TIE_INDEX_ONLY, binding.LOKI_SEARCH_PER_LANE
ALL_FLAGS = [0, TIE, LANE, LANE | TIE]


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: these tests must run on an MI355X")
    binding.lib()


def bits(x: float) -> int:
    return struct.unpack("<Q", struct.pack("<d", x))[0]


def same(res: binding.Result, ref) -> bool:
    """ref: oracle.Best or a golden record dict."""
    if isinstance(ref, dict):
        t = (ref["index"], float.fromhex(ref["accuracy_hex"]), ref["n_feasible"], ref["workers"], ref["found"])
    else:
        t = ref.as_tuple()
    got = res.as_tuple()
    return got[0] == t[0] and bits(got[1]) == bits(t[1]) and got[2:] == t[2:]


def check(res, ref, what):
    assert same(res, ref), f"{what}: gpu {res.as_tuple()} vs ref {ref if isinstance(ref, dict) else ref.as_tuple()}"


# ---- sizes the checker finishes in seconds: exhaustive comparison -----------------------------------------

def test_config1_full_space_all_modes():
    w = wl.config(1)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    d = w.demand_mqps[0]
    for flags in ALL_FLAGS:
        res = P.alloc_search([d], w.workers, w.slo_us, w.comm_us, flags=flags)[0]
        ref = O.search(d, w.workers, w.slo_us, w.comm_us, tie_index_only=bool(flags & TIE))
        check(res, ref, f"cfg1 flags={flags}")
    # a sweep of demand points in one call, from zero demand to beyond capacity
    demands = [0, 1, 50_000, 120_000, 200_000, 300_000, 10**7]
    for flags in ALL_FLAGS:
        out = P.alloc_search(demands, w.workers, w.slo_us, w.comm_us, flags=flags)
        for dd, res in zip(demands, out):
            check(res, O.search(dd, w.workers, w.slo_us, w.comm_us, tie_index_only=bool(flags & TIE)),
                  f"cfg1 sweep d={dd} flags={flags}")
    assert out[-1].status == binding.LOKI_NO_FEASIBLE and out[-1].index == binding.UINT64_MAX


def test_config1_every_candidate_eval():
    w = wl.config(1)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    n = P.num_candidates()
    for d in (0, w.demand_mqps[0]):
        got = P.alloc_eval(list(range(n)), d, w.workers, w.slo_us, w.comm_us)
        for idx in range(n):
            e = O.eval(idx, d, w.workers, w.slo_us, w.comm_us)
            g = got[idx]
            assert (g.infeasible, g.workers, bits(g.accuracy)) == (e.infeasible, e.workers, bits(e.accuracy)), idx


@pytest.mark.parametrize("seed", range(48))
def test_random_small_problems(seed):
    """Ragged K_i / R_ik / |B_i|, random trees with up to 4 tasks, duplicate accuracies,
    communication latency, zero demand now and then."""
    w = wl.random_small(seed, max_tasks=4, max_variants=3, max_replicas=3, max_candidates=60000)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    n = P.num_candidates()
    assert n == O.num_candidates()
    d = w.demand_mqps[0]
    for flags in ALL_FLAGS:
        res = P.alloc_search([d], w.workers, w.slo_us, w.comm_us, flags=flags)[0]
        ref = O.search(d, w.workers, w.slo_us, w.comm_us, tie_index_only=bool(flags & TIE))
        check(res, ref, f"{w.name} flags={flags}")
    rng = random.Random(seed)
    idxs = list(range(n)) if n <= 4096 else [rng.randrange(n) for _ in range(4096)]
    got = P.alloc_eval(idxs, d, w.workers, w.slo_us, w.comm_us)
    for g, idx in zip(got, idxs):
        e = O.eval(idx, d, w.workers, w.slo_us, w.comm_us)
        assert (g.infeasible, g.workers, bits(g.accuracy)) == (e.infeasible, e.workers, bits(e.accuracy)), idx
        assert P.decode(idx)[0] == O.decode(idx)[0]
    # a ragged sub-range
    if n > 10:
        lo = rng.randrange(0, n // 2)
        hi = rng.randrange(lo, n + 1)
        for flags in ALL_FLAGS:
            res = P.alloc_search([d], w.workers, w.slo_us, w.comm_us, flags=flags, begin=lo, end=hi)[0]
            ref = O.search(d, w.workers, w.slo_us, w.comm_us, tie_index_only=bool(flags & TIE), begin=lo, end=hi)
            check(res, ref, f"{w.name} range [{lo},{hi}) flags={flags}")


def test_degenerate_cases():
    w = wl.config(1)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    d = w.demand_mqps[0]
    n = P.num_candidates()
    for flags in ALL_FLAGS:
        # empty range
        r = P.alloc_search([d], w.workers, w.slo_us, flags=flags, begin=777, end=777)[0]
        assert r.as_tuple() == (binding.UINT64_MAX, 0.0, 0, -1, 0)
        # single candidate ranges (first, last, the winner)
        for idx in (0, n - 1, 29744):
            r = P.alloc_search([d], w.workers, w.slo_us, flags=flags, begin=idx, end=idx + 1)[0]
            check(r, O.search(d, w.workers, w.slo_us, begin=idx, end=idx + 1), f"single {idx}")
        # no workers, no time, negative room after communication latency
        for (W, slo, comm) in ((0, w.slo_us, 0), (w.workers, 0, 0), (w.workers, 5000, 4000)):
            r = P.alloc_search([d], W, slo, comm, flags=flags)[0]
            check(r, O.search(d, W, slo, comm), f"W={W} slo={slo} comm={comm}")
            assert r.status == binding.LOKI_NO_FEASIBLE
    # one task, one variant, one batch size: 2 candidates
    from types import SimpleNamespace
    tiny = SimpleNamespace(n_tasks=1, parent=[-1], fanout_q4=[4], n_variants=[1], n_batches=[1], batch_size=[4],
                           max_replicas=[1], acc_ppm=[1000000], latency_us=[9000], thr_mqps=[444444])
    Pt, Ot = binding.Problem(tiny), oracle.Problem(tiny)
    for flags in ALL_FLAGS:
        for dd in (0, 444444, 444445):
            check(Pt.alloc_search([dd], 1, 18000, flags=flags)[0], Ot.search(dd, 1, 18000), f"tiny d={dd}")


def test_error_paths_do_not_launch():
    import torch
    w = wl.config(1)
    P = binding.Problem(w.pipeline)
    ws = torch.empty(P.workspace_bytes(1) + 512, dtype=torch.uint8, device="cuda")
    L = binding.lib()
    import ctypes as C
    out = (binding.Result * 1)()
    dem = (C.c_int64 * 1)(120000)
    n = P.num_candidates()
    base = ws.data_ptr()
    assert base % 256 == 0

    def call(demand=dem, m=1, W=8, slo=200000, comm=0, flags=0, b=0, e=n, ptr=base, size=ws.numel(), o=out):
        return L.loki_alloc_search(P._h, demand, m, W, slo, comm, flags, b, e, ptr, size, 0, o)
    assert call(size=1024) == binding.LOKI_E_WORKSPACE
    assert call(ptr=base + 8) == binding.LOKI_E_WORKSPACE
    assert call(flags=64) == binding.LOKI_E_ARG
    assert call(b=5, e=4) == binding.LOKI_E_ARG
    assert call(e=n + 1) == binding.LOKI_E_ARG
    assert call(m=0) == binding.LOKI_E_ARG
    assert call(W=-1) == binding.LOKI_E_RANGE
    assert call(demand=(C.c_int64 * 1)(-5)) == binding.LOKI_E_RANGE
    assert call(demand=(C.c_int64 * 1)(1 << 40)) == binding.LOKI_E_RANGE
    assert call(demand=None) == binding.LOKI_E_NULL
    assert call() == binding.LOKI_OK


# ---- full benchmark sizes --------------------------------------------------------------------------------------

def golden(cfg):
    path = os.path.join(HERE, "golden", f"cfg{cfg}.json")
    if not os.path.exists(path):
        pytest.skip(f"{path} not generated yet (tests/golden/make_golden.py)")
    with open(path) as f:
        doc = json.load(f)
    w = wl.config(cfg)
    assert doc["workload_digest"] == w.digest(), "golden file is for different inputs"
    return doc, w


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_full_size_search_against_stored_checker_results(cfg):
    """The launch configuration the benchmark times: all demand points in one call, whole index space."""
    doc, w = golden(cfg)
    P = binding.Problem(w.pipeline)
    assert P.num_candidates() == doc["n_candidates"]
    out = P.alloc_search(w.demand_mqps, w.workers, w.slo_us, w.comm_us)
    assert len(out) == len(doc["results"])
    for m, (res, ref) in enumerate(zip(out, doc["results"])):
        check(res, ref, f"cfg{cfg} point {m}")
    k = len(doc["results_index_only"])
    if k:
        out = P.alloc_search(w.demand_mqps[:k], w.workers, w.slo_us, w.comm_us, flags=TIE)
        for m, (res, ref) in enumerate(zip(out, doc["results_index_only"])):
            check(res, ref, f"cfg{cfg} point {m} index-only")


def test_config2_full_space_per_lane_kernel():
    doc, w = golden(2)
    P = binding.Problem(w.pipeline)
    for flags in (LANE, LANE | TIE):
        res = P.alloc_search(w.demand_mqps, w.workers, w.slo_us, w.comm_us, flags=flags)[0]
        check(res, doc["results"][0] if not flags & TIE else doc["results_index_only"][0], f"cfg2 flags={flags}")


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_sampled_candidates_and_subranges(cfg):
    w = wl.config(cfg)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    n = P.num_candidates()
    rng = random.Random(100 + cfg)
    demands = [w.demand_mqps[0], w.demand_mqps[len(w.demand_mqps) // 2], min(w.demand_mqps)]
    # (i) sampled candidates one by one; half of them near the winner so that feasible ones are hit
    for d in demands[:2]:
        win = P.alloc_search([d], w.workers, w.slo_us, w.comm_us)[0]
        idxs = [rng.randrange(n) for _ in range(25000)]
        if win.status == binding.LOKI_FOUND:
            e = O.eval(win.index, d, w.workers, w.slo_us, w.comm_us)
            assert e.infeasible == 0 and bits(e.accuracy) == bits(win.accuracy) and e.workers == win.workers_used
            digits_span = min(n, 1 << 20)
            idxs += [(win.index // digits_span) * digits_span + rng.randrange(digits_span) for _ in range(25000)]
            idxs.append(win.index)
        got = P.alloc_eval(idxs, d, w.workers, w.slo_us, w.comm_us)
        n_feas = 0
        for g, idx in zip(got, idxs):
            e = O.eval(idx, d, w.workers, w.slo_us, w.comm_us)
            assert (g.infeasible, g.workers, bits(g.accuracy)) == (e.infeasible, e.workers, bits(e.accuracy)), idx
            if g.infeasible == 0:
                n_feas += 1
                # no sampled feasible plan beats the reported winner
                assert (g.accuracy, -g.workers, -idx) <= (win.accuracy, -win.workers_used, -win.index)
        print(f"cfg{cfg} d={d}: {n_feas} feasible among {len(idxs)} sampled")
    # (ii) sub-ranges the plain per-index checker can enumerate, in both kernels
    d = demands[2]
    for span in (1 << 18, (1 << 20) - 12345):
        lo = rng.randrange(0, n - span)
        win = P.alloc_search([d], w.workers, w.slo_us, w.comm_us)[0]
        spots = [lo]
        if win.status == binding.LOKI_FOUND:
            spots.append(max(0, min(n - span, win.index - span // 3)))
        for b in spots:
            ref = O.search(d, w.workers, w.slo_us, w.comm_us, begin=b, end=b + span)
            for flags in (0, LANE):
                res = P.alloc_search([d], w.workers, w.slo_us, w.comm_us, flags=flags, begin=b, end=b + span)[0]
                check(res, ref, f"cfg{cfg} range [{b},{b + span}) flags={flags}")


def test_range_partition_merges_to_full_result():
    doc, w = golden(2)
    P = binding.Problem(w.pipeline)
    n = P.num_candidates()
    cuts = [0, 123_456_789, 535_286_220, 535_286_221, 900_000_001, n]
    parts = [P.alloc_search(w.demand_mqps, w.workers, w.slo_us, begin=a, end=b)[0] for a, b in zip(cuts, cuts[1:])]
    ref = doc["results"][0]
    assert sum(p.n_feasible for p in parts) == ref["n_feasible"]
    best = min((p for p in parts if p.status == 0), key=lambda p: (-p.accuracy, p.workers_used, p.index))
    assert (best.index, best.accuracy.hex(), best.workers_used) == (ref["index"], ref["accuracy_hex"], ref["workers"])


def test_enqueue_variant_matches_blocking_call():
    import torch
    w = wl.config(1)
    P = binding.Problem(w.pipeline)
    blocking = P.alloc_search(w.demand_mqps, w.workers, w.slo_us)
    for flags in (0, LANE):
        buf = P.alloc_search_enqueue(w.demand_mqps, w.workers, w.slo_us, flags=flags)
        buf2 = P.alloc_search_enqueue(w.demand_mqps, w.workers, w.slo_us, flags=flags)  # back to back, same handle
        torch.cuda.synchronize()
        for b in (buf, buf2):
            got = binding.results_from_bytes(bytes(b.cpu().numpy().tobytes()))
            assert got[0].as_tuple() == blocking[0].as_tuple()
    assert P.last_search_ms()[1] > 0.0


def test_route_table_of_the_winner():
    for cfg in (1, 2):
        w = wl.config(cfg)
        P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
        d = w.demand_mqps[0]
        win = P.alloc_search([d], w.workers, w.slo_us)[0]
        assert win.status == binding.LOKI_FOUND
        r, ro = P.route_table(win.index, d), O.route_table(win.index, d)
        for i in range(w.pipeline.n_tasks):
            assert r.demand[i] == ro.demand[i] and r.scale[i] == ro.scale[i] and r.unserved[i] == ro.unserved[i] == 0
            for k in range(w.pipeline.n_variants[i]):
                assert (r.capacity[i][k], r.routed[i][k], r.leftover[i][k], r.budget_us[i][k]) == \
                    (ro.capacity[i][k], ro.routed[i][k], ro.leftover[i][k], ro.budget_us[i][k])
                for k2 in range(oracle.MAX_VARIANTS):
                    assert bits(r.prob[i][k][k2]) == bits(ro.prob[i][k][k2])


@pytest.mark.parametrize("seed", range(24))
def test_per_variant_multiplicative_factors(seed):
    """Child demand follows the parent's routing (eq. (1) with r(i,k)); the library takes the per-lane path."""
    w = wl.random_small(5000 + seed, max_tasks=4, max_variants=3, max_replicas=3, max_candidates=60000,
                        variant_factors=True)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    n = P.num_candidates()
    d = w.demand_mqps[0]
    for flags in ALL_FLAGS:
        res = P.alloc_search([d, d // 2], w.workers, w.slo_us, w.comm_us, flags=flags)
        for dd, r in zip((d, d // 2), res):
            check(r, O.search(dd, w.workers, w.slo_us, w.comm_us, tie_index_only=bool(flags & TIE)),
                  f"{w.name} d={dd} flags={flags}")
    rng = random.Random(seed)
    idxs = list(range(n)) if n <= 4096 else [rng.randrange(n) for _ in range(4096)]
    got = P.alloc_eval(idxs, d, w.workers, w.slo_us, w.comm_us)
    for g, idx in zip(got, idxs):
        e = O.eval(idx, d, w.workers, w.slo_us, w.comm_us)
        assert (g.infeasible, g.workers, bits(g.accuracy)) == (e.infeasible, e.workers, bits(e.accuracy)), idx
    win = P.alloc_search([d], w.workers, w.slo_us, w.comm_us)[0]
    if win.status == binding.LOKI_FOUND:
        r, ro = P.route_table(win.index, d), O.route_table(win.index, d)
        for i in range(w.pipeline.n_tasks):
            assert (r.demand[i], r.scale[i], r.unserved[i]) == (ro.demand[i], ro.scale[i], ro.unserved[i])
            for k in range(w.pipeline.n_variants[i]):
                assert (r.capacity[i][k], r.routed[i][k], r.leftover[i][k]) == \
                    (ro.capacity[i][k], ro.routed[i][k], ro.leftover[i][k])


@pytest.mark.parametrize("seed", range(24))
def test_per_variant_batch_sizes(seed):
    """y(i,k): every hosted variant with its own batch size; still separable per task, so both kernels apply."""
    w = wl.random_small(8000 + seed, max_tasks=3, max_variants=2, max_replicas=2, max_batches=3, max_candidates=200000,
                        per_variant_batch=True, variant_factors=seed % 4 == 3)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    n = P.num_candidates()
    d = w.demand_mqps[0]
    for flags in ALL_FLAGS:
        res = P.alloc_search([d], w.workers, w.slo_us, w.comm_us, flags=flags)[0]
        check(res, O.search(d, w.workers, w.slo_us, w.comm_us, tie_index_only=bool(flags & TIE)),
              f"{w.name} flags={flags}")
    rng = random.Random(seed)
    idxs = list(range(n)) if n <= 4096 else [rng.randrange(n) for _ in range(4096)]
    got = P.alloc_eval(idxs, d, w.workers, w.slo_us, w.comm_us)
    for g, idx in zip(got, idxs):
        e = O.eval(idx, d, w.workers, w.slo_us, w.comm_us)
        assert (g.infeasible, g.workers, bits(g.accuracy)) == (e.infeasible, e.workers, bits(e.accuracy)), idx


def test_per_variant_batch_sizes_at_scale():
    """Config-1 profiles with a batch size per variant: 13^3 choices per task, 4.8M plans, 2197 root choices."""
    w = wl.config(1)
    w.pipeline.per_variant_batch = True
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    assert P.num_candidates() == 13 ** 6
    for d in (0, w.demand_mqps[0], 2 * w.demand_mqps[0]):
        ref = O.search(d, w.workers, w.slo_us)
        for flags in (0, LANE):
            check(P.alloc_search([d], w.workers, w.slo_us, flags=flags)[0], ref, f"pv cfg1 d={d} flags={flags}")


def test_batched_route_tables_match_the_host_path_and_the_checker():
    import ctypes as C
    cases = [wl.config(1), wl.config(4)]
    cases += [wl.random_small(9000 + s, max_tasks=4, max_candidates=30000, variant_factors=s % 2 == 0,
                              per_variant_batch=s % 3 == 0) for s in range(8)]
    for w in cases:
        P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
        demands = w.demand_mqps if len(w.demand_mqps) > 1 else [w.demand_mqps[0] * f // 4 for f in range(0, 9)]
        demands = demands[:48]
        wins = P.alloc_search(demands, w.workers, w.slo_us, w.comm_us)
        idxs = [r.index if r.status == binding.LOKI_FOUND else (7 * m) % P.num_candidates() for m, r in enumerate(wins)]
        batch = P.route_table_batch(idxs, demands)
        for idx, d, got in zip(idxs, demands, batch):
            host = P.route_table(idx, d)
            assert bytes(got) == bytes(host), (w.name, idx, d)
            ro = O.route_table(idx, d)
            for i in range(w.pipeline.n_tasks):
                assert (got.demand[i], got.unserved[i]) == (ro.demand[i], ro.unserved[i])
                for k in range(w.pipeline.n_variants[i]):
                    assert (got.routed[i][k], got.leftover[i][k]) == (ro.routed[i][k], ro.leftover[i][k])
                    for k2 in range(oracle.MAX_VARIANTS):
                        assert bits(got.prob[i][k][k2]) == bits(ro.prob[i][k][k2])


def test_plan_trace_follows_the_two_step_resource_manager():
    """EWMA demand estimate, one allocation per estimate, and the phase (hardware scaling while the most
    accurate variants suffice, then accuracy scaling, then overload): Section 4 and Section 4.2, and the
    shape of the paper's Figure 1 walk-through on a rising demand ramp."""
    from fractions import Fraction
    w = wl.config(1)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    rng = random.Random(4)
    ramp = [int(3_000 * t + rng.randint(0, 2_000)) for t in range(120)]
    alpha = 300_000
    steps = P.plan_trace(ramp, alpha, w.workers, w.slo_us)
    top = O.search(0, w.workers, w.slo_us).accuracy          # zero demand: the most accurate variants
    est = None
    phases = []
    for t, (d, s) in enumerate(zip(ramp, steps)):
        est = d if t == 0 else (Fraction(alpha * d + (10**6 - alpha) * est, 10**6)).__floor__()
        assert s.estimate_mqps == est
        check(s.plan, O.search(est, w.workers, w.slo_us), f"trace step {t}")
        want = binding.LOKI_PHASE_OVERLOAD if s.plan.status != binding.LOKI_FOUND else (
            binding.LOKI_PHASE_HARDWARE if s.plan.accuracy == top else binding.LOKI_PHASE_ACCURACY)
        assert s.phase == want
        phases.append(s.phase)
    # estimates of a rising ramp rise, so the phases come in order and all three occur
    assert phases == sorted(phases) and set(phases) == {0, 1, 2}
    hw = [s for s in steps if s.phase == binding.LOKI_PHASE_HARDWARE]
    assert all(a.plan.workers_used <= b.plan.workers_used for a, b in zip(hw, hw[1:]))   # servers added first
    assert hw[-1].plan.workers_used <= w.workers
    acc = [s.plan.accuracy for s in steps if s.phase != binding.LOKI_PHASE_OVERLOAD]
    assert all(a >= b for a, b in zip(acc, acc[1:]))                                      # then accuracy is traded
    # a constant trace is its own estimate
    flat = P.plan_trace([77_777] * 5, 1, w.workers, w.slo_us)
    assert [s.estimate_mqps for s in flat] == [77_777] * 5


def test_per_variant_factors_on_benchmark_profiles():
    """Config 1 in full and a 2^26-plan slice of config 2, with r(i,k) growing with accuracy."""
    for cfg, span in ((1, None), (2, 1 << 26)):
        w = wl.config(cfg)
        p = w.pipeline
        p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]   # 0.75 .. 1.5
        P, O = binding.Problem(p), oracle.Problem(p)
        n = P.num_candidates()
        d = w.demand_mqps[0] // 2
        spans = [(0, n)] if span is None else [(0, span), (n // 2 - 12345, n // 2 - 12345 + span)]
        for lo, hi in spans:
            for flags in (0, TIE):
                res = P.alloc_search([d], w.workers, w.slo_us, flags=flags, begin=lo, end=hi)[0]
                ref = O.search(d, w.workers, w.slo_us, tie_index_only=bool(flags & TIE), begin=lo, end=hi)
                check(res, ref, f"cfg{cfg} vf [{lo},{hi}) flags={flags}")


def test_hardware_scaling_step_through_the_same_search():
    """Step 1 of Section 4 (eq. (8)-(11)): only the most accurate variant of every task may be hosted
    (replica limit 0 for the others, eq. (10)) and the winner is the plan with the fewest servers.  On
    config 4's profiles, for demands from 0 to 160 QPS: the masked search against the checker, and
    against the full search, which must return the same accuracy and server count wherever Step 1 has
    a solution."""
    import copy
    w = wl.config(4)
    p = w.pipeline
    masked = copy.deepcopy(p)
    v = 0
    for i in range(p.n_tasks):
        top = max(p.acc_ppm[v:v + p.n_variants[i]])
        for k in range(p.n_variants[i]):
            if p.acc_ppm[v + k] != top:
                masked.max_replicas[v + k] = 0
        v += p.n_variants[i]
    P1, O1, P2 = binding.Problem(masked), oracle.Problem(masked), binding.Problem(p)
    assert P1.num_candidates() == 16 ** 3                        # one variant, 0..3 replicas, 4 batch sizes
    demands = list(range(0, 160_000, 2_500))
    step1 = P1.alloc_search(demands, w.workers, w.slo_us)
    full = P2.alloc_search(demands, w.workers, w.slo_us)
    solved = 0
    for d, s1, f in zip(demands, step1, full):
        check(s1, O1.search(d, w.workers, w.slo_us), f"step 1 at {d}")
        if s1.status == binding.LOKI_FOUND:
            solved += 1
            assert f.status == binding.LOKI_FOUND and bits(f.accuracy) == bits(s1.accuracy), d
            assert f.workers_used == s1.workers_used, d
        elif f.status == binding.LOKI_FOUND:
            assert f.accuracy < step1[0].accuracy, d             # Step 2: accuracy is given up
    assert 10 < solved < len(step1) and step1[0].status == binding.LOKI_FOUND
    assert any(f.status == binding.LOKI_FOUND and s.status != binding.LOKI_FOUND for s, f in zip(step1, full))


def test_per_variant_factors_class_by_class_on_a_detector_with_two_classifiers():
    """Config 4's tree (0 -> 1, 0 -> 2) with factors rising with accuracy: the other tasks' demand depends
    on the first task's choice only through the requests it creates, and the library runs the tabulated
    kernels once per distinct amount.  Against the kernel that scores whole plans per lane at every demand
    point, against the checker on two of them (2^30 plans each), and on split ranges."""
    w = wl.config(4)
    p = w.pipeline
    p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]   # 0.75 .. 1.5
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    p_choices = 4 ** 4 * 4      # choices of the first task

    def usable(O, c0, d):       # the first task's choice c0 hosts something and serves all of demand d
        r = O.route_table(c0, d)
        return r.unserved[0] == 0 and any(r.capacity[0][k] > 0 for k in range(4))

    demands = sorted(w.demand_mqps)[::40] + [0, 30_000]
    for flags in (0, TIE):
        by_class = P.alloc_search(demands, w.workers, w.slo_us, flags=flags)
        per_lane = P.alloc_search(demands, w.workers, w.slo_us, flags=flags | LANE)
        for d, a, b in zip(demands, by_class, per_lane):
            assert a.as_tuple()[0] == b.as_tuple()[0] and bits(a.accuracy) == bits(b.accuracy) and \
                a.as_tuple()[2:] == b.as_tuple()[2:], (d, flags, a.as_tuple(), b.as_tuple())
    assert sum(r.status == binding.LOKI_FOUND for r in by_class) >= 3
    # the kernels of the last call (per lane) scored every plan; class by class, plans whose first-task
    # choice cannot serve the demand never reach them
    assert P.last_search_plans_scored() == n * len(demands)
    P.alloc_search(demands, w.workers, w.slo_us)
    served = sum(sum(1 for c0 in range(p_choices) if usable(O, c0, d)) for d in demands)
    assert P.last_search_plans_scored() == served * (n // p_choices) < n * len(demands)
    for d in (demands[1], 30_000):
        check(P.alloc_search([d], w.workers, w.slo_us)[0], O.search(d, w.workers, w.slo_us), f"demand {d}")
    cut = n // 3 + 777
    d = demands[1]
    lo = P.alloc_search([d], w.workers, w.slo_us, begin=0, end=cut)[0]
    hi = P.alloc_search([d], w.workers, w.slo_us, begin=cut, end=n)[0]
    whole = P.alloc_search([d], w.workers, w.slo_us)[0]
    assert lo.n_feasible + hi.n_feasible == whole.n_feasible
    best = min((r for r in (lo, hi) if r.status == binding.LOKI_FOUND),
               key=lambda r: (-r.accuracy, r.workers_used, r.index))
    assert (best.index, bits(best.accuracy), best.workers_used) == (whole.index, bits(whole.accuracy), whole.workers_used)


def test_per_variant_factors_with_more_classes_than_one_call_takes():
    """65,535 demand points on a small detector-and-classifier pipeline with factors: the (demand point,
    class) pairs exceed what the descriptor arrays hold, so the library takes the demand points in groups;
    12,000 points fit one group.  Both against the checker on samples."""
    p = SimpleNamespace(n_tasks=2, parent=[-1, 0], fanout_q4=[4, 6], n_variants=[2, 2], n_batches=[2, 1],
                        batch_size=[1, 4, 2], max_replicas=[2, 2, 3, 3], acc_ppm=[700000, 900000, 650000, 880000],
                        latency_us=[3000, 9000, 5000, 14000, 4000, 7000],
                        thr_mqps=[333333, 444444, 200000, 285714, 500000, 285714],
                        variant_factor_q4=[3, 6, 4, 4])
    P, O = binding.Problem(p), oracle.Problem(p)
    rng = random.Random(17)

    def classes(d):   # distinct amounts of requests the first task's usable choices create (18 choices)
        amounts = set()
        for c0 in range(18):
            r = O.route_table(c0, d)
            if r.unserved[0] == 0 and any(r.capacity[0][k] > 0 for k in range(2)):
                amounts.add(sum(r.routed[0][k] * p.variant_factor_q4[k] for k in range(2)))
        return len(amounts)

    sample = [rng.randint(0, 1_500_000) for _ in range(500)]
    per_point = sum(classes(d) for d in sample) / len(sample)
    assert per_point * 65_535 > 80_000 and per_point * 12_000 < 50_000, per_point
    for n_points in (65_535, 12_000):
        demands = [rng.randint(0, 1_500_000) for _ in range(n_points)]
        out = P.alloc_search(demands, 9, 60_000)
        assert P.last_search_plans_scored() < P.num_candidates() * n_points     # class by class, not per lane
        for j in list(range(0, n_points, 997)) + [n_points - 1]:
            check(out[j], O.search(demands[j], 9, 60_000), f"{n_points} points, point {j}")


def _star_with_factors(n_tasks, seed, variants=2, replicas=2, batches=(1, 4)):
    rng = wl.SplitMix64(seed)
    p = wl.make_pipeline([-1] + [0] * (n_tasks - 1), variants, replicas, batches, rng)
    # factors that grow with accuracy (Section 4.2), 0.75 .. 2.25
    p.variant_factor_q4 = [3 + (a - 600000) // 60000 for a in p.acc_ppm]
    return p


@pytest.mark.parametrize("n_tasks,seed", [(4, 5), (5, 9), (3, 2)])
def test_per_variant_factors_on_stars_with_three_and_more_leaves(n_tasks, seed):
    """A detector feeding 2, 3 and 4 classifiers: with classes the tiles hold task 1's choices and the
    first task's choices of the class become part of the work item, with the tasks after task 1.  Odd path
    counts divide the objective, 18 choices per task leave most lanes' slots empty.  Against the checker's
    brute force and the kernel that scores whole plans per lane, at demands from idle to overload, with
    worker budgets and latency limits that bind."""
    p = _star_with_factors(n_tasks, seed)
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    assert n == 18 ** n_tasks
    demands = [0, 20_000, 90_000, 250_000, 600_000, 2_000_000]
    found = 0
    for workers, slo in ((4 * n_tasks, 400_000), (n_tasks + 2, 400_000), (4 * n_tasks, 60_000)):
        for flags in (0, TIE):
            by_class = P.alloc_search(demands, workers, slo, flags=flags)
            per_lane = P.alloc_search(demands, workers, slo, flags=flags | LANE)
            for d, a, b in zip(demands, by_class, per_lane):
                assert a.as_tuple()[0] == b.as_tuple()[0] and bits(a.accuracy) == bits(b.accuracy) and \
                    a.as_tuple()[2:] == b.as_tuple()[2:], (d, workers, slo, flags, a.as_tuple(), b.as_tuple())
            if n <= 18 ** 4:
                for d, a in zip(demands[:4], by_class[:4]):
                    check(a, O.search(d, workers, slo, tie_index_only=bool(flags & TIE)), f"demand {d} workers {workers}")
            found += sum(r.status == binding.LOKI_FOUND for r in by_class)
    assert found >= 8


def test_per_variant_factors_on_a_star_with_a_batch_size_per_variant():
    """The class-by-class search with the other index layout (a batch size per hosted variant)."""
    p = _star_with_factors(3, 21, variants=2, replicas=2, batches=(1, 4))
    p.per_variant_batch = True
    P, O = binding.Problem(p), oracle.Problem(p)
    assert P.num_candidates() == 25 ** 3
    demands = [0, 40_000, 150_000, 500_000]
    for workers, slo in ((12, 400_000), (5, 400_000), (12, 50_000)):
        by_class = P.alloc_search(demands, workers, slo)
        per_lane = P.alloc_search(demands, workers, slo, flags=LANE)
        for d, a, b in zip(demands, by_class, per_lane):
            assert a.as_tuple()[0] == b.as_tuple()[0] and bits(a.accuracy) == bits(b.accuracy) and \
                a.as_tuple()[2:] == b.as_tuple()[2:], (d, workers, slo, a.as_tuple(), b.as_tuple())
            check(a, O.search(d, workers, slo), f"demand {d} workers {workers} slo {slo}")


def test_per_variant_factors_on_a_star_whose_second_task_cannot_be_ordered_into_runs():
    """Task 1 has 66 replica counts x 64 profiled latencies, more buckets than the ordering kernel sorts,
    so its choices cannot fill the tiles: the class-by-class search keeps the first task's choices there."""
    rng = random.Random(5)
    k1, nb1 = 8, 8
    p = SimpleNamespace(
        n_tasks=3, parent=[-1, 0, 0], fanout_q4=[4, 6, 3], n_variants=[2, k1, 2], n_batches=[1, nb1, 1],
        batch_size=[2] + [1 << b for b in range(nb1)] + [4],
        max_replicas=[2, 2] + [63, 1, 1, 0, 0, 0, 0, 0] + [3, 3],
        acc_ppm=[700000, 900000] + [600000 + 40000 * k for k in range(k1)] + [650000, 880000],
        latency_us=[4000, 9000] + [1000 + 37 * (k * nb1 + b) for k in range(k1) for b in range(nb1)] + [5000, 8000],
        thr_mqps=[300000, 200000] + [20000 + 5000 * b + 1000 * k for k in range(k1) for b in range(nb1)] + [400000, 250000],
        variant_factor_q4=[3, 6] + [4] * k1 + [4, 4])
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    assert n == 9 * (64 * 2 * 2 * nb1) * 16
    demands = [0, 60_000, 200_000, 450_000]
    hit = 0
    for workers, slo in ((70, 200_000), (9, 200_000), (70, 24_000)):
        by_class = P.alloc_search(demands, workers, slo)
        per_lane = P.alloc_search(demands, workers, slo, flags=LANE)
        for d, a, b in zip(demands, by_class, per_lane):
            assert a.as_tuple()[0] == b.as_tuple()[0] and bits(a.accuracy) == bits(b.accuracy) and \
                a.as_tuple()[2:] == b.as_tuple()[2:], (d, workers, slo, a.as_tuple(), b.as_tuple())
        check(by_class[1], O.search(demands[1], workers, slo), f"workers {workers} slo {slo}")
        hit += sum(r.status == binding.LOKI_FOUND for r in by_class)
    assert hit >= 4


@pytest.mark.parametrize("parent,seed", [([-1, 0, 1, 0], 3), ([-1, 0, 0, 1], 4), ([-1, 0, 1, 1], 6),
                                         ([-1, 0, 1, 0, 3], 8), ([-1, 0, 1, 0, 0], 11)])
def test_per_variant_factors_on_deeper_trees_class_by_class(parent, seed):
    """Trees with several tasks that have children (config 5's shape among them): a point of the launch
    fixes one amount of created requests per such task, the first leaf's choices fill the tiles, the
    lists of the other tasks' choices make up the work items.  Against the kernel that scores whole
    plans per lane and, on the four-task trees, the checker's brute force."""
    rng = wl.SplitMix64(seed)
    p = wl.make_pipeline(parent, 2, 2, (1, 4), rng)
    p.variant_factor_q4 = [3 + (a - 600000) // 60000 for a in p.acc_ppm]
    P, O = binding.Problem(p), oracle.Problem(p)
    n_tasks = len(parent)
    n = P.num_candidates()
    assert n == 18 ** n_tasks
    demands = [0, 20_000, 90_000, 250_000, 600_000]
    found = 0
    for workers, slo in ((4 * n_tasks, 600_000), (n_tasks + 2, 600_000), (4 * n_tasks, 90_000)):
        for flags in (0, TIE):
            by_class = P.alloc_search(demands, workers, slo, flags=flags)
            scored = P.last_search_plans_scored()
            per_lane = P.alloc_search(demands, workers, slo, flags=flags | LANE)
            assert scored < n * len(demands) == P.last_search_plans_scored()
            for d, a, b in zip(demands, by_class, per_lane):
                assert a.as_tuple()[0] == b.as_tuple()[0] and bits(a.accuracy) == bits(b.accuracy) and \
                    a.as_tuple()[2:] == b.as_tuple()[2:], (d, workers, slo, flags, a.as_tuple(), b.as_tuple())
            if n_tasks == 4:
                for d, a in zip(demands[:4], by_class[:4]):
                    check(a, O.search(d, workers, slo, tie_index_only=bool(flags & TIE)), f"demand {d} workers {workers}")
            found += sum(r.status == binding.LOKI_FOUND for r in by_class)
    assert found >= 6
    # ragged index ranges run class by class as well (every tile entry then carries its own interval of the
    # last task's choices): against the checker on the same ranges
    cuts = [0, n // 5 + 3, n // 2 + 77, n - n // 7, n]
    for d in demands[1:4]:
        parts = []
        for a, b in zip(cuts, cuts[1:]):
            res = P.alloc_search([d], 4 * n_tasks, 600_000, begin=a, end=b)[0]
            assert P.last_search_plans_scored() < n       # (an upper estimate of what the kernels scored)
            if n_tasks == 4:
                check(res, O.search(d, 4 * n_tasks, 600_000, begin=a, end=b), f"demand {d} range {a}..{b}")
            parts.append(res)
        whole = P.alloc_search([d], 4 * n_tasks, 600_000)[0]
        assert sum(r.n_feasible for r in parts) == whole.n_feasible
        hits = [r for r in parts if r.status == binding.LOKI_FOUND]
        if hits:
            best = min(hits, key=lambda r: (-r.accuracy, r.workers_used, r.index))
            assert (best.index, bits(best.accuracy), best.workers_used) == \
                (whole.index, bits(whole.accuracy), whole.workers_used)


@pytest.mark.parametrize("full_task", [2, 3])
def test_per_variant_factors_on_config_5s_tree_with_full_size_tiles(full_task):
    """Config 5's profiles and tree (0 -> 1 -> 2, 0 -> 3) with factors, one variant masked out in three of
    the four tasks (256 choices each) and all 1,024 choices in the first leaf (two tiles of 512 entries) or
    in the last task (8 register slots per lane): 2^34 plans per demand point, class by class against the
    kernel that scores whole plans per lane, the winners also through the checker."""
    import copy
    w = wl.config(5)
    p = copy.deepcopy(w.pipeline)
    p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]
    for i in range(4):
        if i != full_task:
            p.max_replicas[4 * i + 1] = 0
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    assert n == 1 << 34
    demands = [100_000, 300_000, 700_000]
    by_class = P.alloc_search(demands, w.workers, w.slo_us)
    assert P.last_search_plans_scored() < n * len(demands)
    per_lane = P.alloc_search(demands, w.workers, w.slo_us, flags=LANE)
    for d, a, b in zip(demands, by_class, per_lane):
        assert a.as_tuple()[0] == b.as_tuple()[0] and bits(a.accuracy) == bits(b.accuracy) and \
            a.as_tuple()[2:] == b.as_tuple()[2:], (d, a.as_tuple(), b.as_tuple())
        if a.status == binding.LOKI_FOUND:
            e = O.eval(a.index, d, w.workers, w.slo_us)
            assert e.infeasible == 0 and bits(e.accuracy) == bits(a.accuracy) and e.workers == a.workers_used
    assert sum(r.status == binding.LOKI_FOUND and r.n_feasible > 1000 for r in by_class) >= 2


@pytest.mark.parametrize("cfg", [4, 5])
def test_unit_factors_class_by_class_reproduce_the_stored_full_size_results(cfg):
    """r(i,k) = 1.00 for every variant is the model with one factor per edge (eq. (1)), but the library
    cannot know that and searches class by class: every task with children then has one class (all of its
    usable choices), and the search with swapped roles must return, on the benchmark's full sizes, the
    stored results of the checker for the plain model bit for bit (2^40 plans on config 5)."""
    import copy
    doc, w = golden(cfg)
    p = copy.deepcopy(w.pipeline)
    p.variant_factor_q4 = [4] * len(p.acc_ppm)
    P = binding.Problem(p)
    points = list(range(0, len(w.demand_mqps), 37))
    demands = [w.demand_mqps[m] for m in points]
    out = P.alloc_search(demands, w.workers, w.slo_us, w.comm_us)
    assert P.last_search_plans_scored() <= doc["n_candidates"] * len(points)
    for m, res in zip(points, out):
        check(res, doc["results"][m], f"cfg{cfg} point {m} with unit factors")


@pytest.mark.parametrize("n_tasks,seed", [(3, 31), (4, 32), (3, 34)])
def test_per_variant_factors_on_chains_class_by_class(n_tasks, seed):
    """A chain has one leaf, the last task, so nothing spare to fill the tiles with: the choices of the
    last task's parent that belong to the point do, and its accuracy and latency enter the last task's
    path per entry.  Against the kernel that scores whole plans per lane and the checker's brute force."""
    rng = wl.SplitMix64(seed)
    p = wl.make_pipeline([-1] + list(range(n_tasks - 1)), 2, 2, (1, 4), rng)
    p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    # (four tasks deep the fixed-point range leaves room for some tens of queries per second only)
    demands = [0, 10_000, 40_000, 120_000, 400_000] if n_tasks == 3 else [0, 2_000, 8_000, 20_000, 30_000]
    found = 0
    for workers, slo in ((4 * n_tasks, 900_000), (n_tasks + 2, 900_000), (4 * n_tasks, 120_000)):
        for flags in (0, TIE):
            by_class = P.alloc_search(demands, workers, slo, flags=flags)
            assert P.last_search_plans_scored() < n * len(demands)
            per_lane = P.alloc_search(demands, workers, slo, flags=flags | LANE)
            for d, a, b in zip(demands, by_class, per_lane):
                assert a.as_tuple()[0] == b.as_tuple()[0] and bits(a.accuracy) == bits(b.accuracy) and \
                    a.as_tuple()[2:] == b.as_tuple()[2:], (d, workers, slo, flags, a.as_tuple(), b.as_tuple())
            if n_tasks <= 4:
                for d, a in zip(demands[:4], by_class[:4]):
                    check(a, O.search(d, workers, slo, tie_index_only=bool(flags & TIE)), f"demand {d} workers {workers}")
            found += sum(r.status == binding.LOKI_FOUND for r in by_class)
    assert found >= 6


def test_per_variant_factors_on_config_2s_chain_at_full_size():
    """Config 2 (a chain of three tasks, 2^30 plans) with factors: class by class against per lane, and
    with unit factors against the stored results of the checker for the plain model."""
    import copy
    doc, w = golden(2)
    p = copy.deepcopy(w.pipeline)
    p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]
    P = binding.Problem(p)
    demands = [50_000, 150_000, 400_000]
    by_class = P.alloc_search(demands, w.workers, w.slo_us)
    assert P.last_search_plans_scored() < P.num_candidates() * len(demands)
    per_lane = P.alloc_search(demands, w.workers, w.slo_us, flags=LANE)
    for d, a, b in zip(demands, by_class, per_lane):
        assert a.as_tuple()[0] == b.as_tuple()[0] and bits(a.accuracy) == bits(b.accuracy) and \
            a.as_tuple()[2:] == b.as_tuple()[2:], (d, a.as_tuple(), b.as_tuple())
    assert sum(r.status == binding.LOKI_FOUND for r in by_class) >= 2
    p.variant_factor_q4 = [4] * len(p.acc_ppm)
    out = binding.Problem(p).alloc_search(w.demand_mqps, w.workers, w.slo_us, w.comm_us)
    check(out[0], doc["results"][0], "cfg2 with unit factors")


def test_plan_trace_with_per_variant_factors():
    """The demand-trace planner with per-variant factors: its batched search runs class by class; every
    step against the checker, on a two-task pipeline and on a detector with two classifiers."""
    for parent, seed in (([-1, 0], 41), ([-1, 0, 0], 42)):
        rng = wl.SplitMix64(seed)
        p = wl.make_pipeline(parent, 2, 2, (1, 4), rng)
        p.variant_factor_q4 = [3 + (a - 600000) // 60000 for a in p.acc_ppm]
        P, O = binding.Problem(p), oracle.Problem(p)
        ramp = [9_000 * t for t in range(40)]
        steps = P.plan_trace(ramp, 400_000, 3 * len(parent), 500_000)
        found = 0
        for t, s in enumerate(steps):
            check(s.plan, O.search(s.estimate_mqps, 3 * len(parent), 500_000), f"{parent} step {t}")
            found += s.plan.status == binding.LOKI_FOUND
        assert 5 <= found < len(steps)


def test_model_variants_at_full_size_against_stored_checker_results():
    """Per-variant factors on config 2's chain and config 4's tree, profiled path accuracies on both,
    both together on both: 2^30 plans per demand point, the library's default search (class by class;
    on the chain tabulated feasibility with the walk for feasible plans, on the tree the objective leaf
    by leaf) against results of the checker's plain per-index search stored by
    tests/golden/make_golden.py --variants."""
    path = os.path.join(HERE, "golden", "variants.json")
    with open(path) as f:
        doc = json.load(f)
    for name, case in doc["cases"].items():
        w = wl.config(case["config"])
        p = w.pipeline
        if case["what"] in ("variant_factors", "both"):
            p.variant_factor_q4 = [3 + (a - 600000) // 90000 for a in p.acc_ppm]
        if case["what"] in ("path_tables", "both"):
            p.path_acc_ppm = wl.draw_path_tables(p, wl.SplitMix64(w.seed + 1))
        assert case["workload_digest"] == w.digest(), "stored results are for different inputs"
        P = binding.Problem(p)
        assert P.num_candidates() == case["n_candidates"]
        demands = [r["demand_mqps"] for r in case["results"]]
        out = P.alloc_search(demands, case["workers"], case["slo_us"], case["comm_us"])
        for res, ref in zip(out, case["results"]):
            check(res, ref, f"{name} demand {ref['demand_mqps']}")
        assert any(r["found"] and r["n_feasible"] > 1000 for r in case["results"]), name


def test_per_variant_factors_sweep_on_a_deeper_tree_in_groups():
    """Config 5's shape (0 -> 1 -> 2, 0 -> 3) with 3 variants per task and 4,000 demand points: two tasks have
    children, so a demand point has hundreds of (class, class) points and the call is taken in several
    groups of demand points.  Sampled demand points against the checker's brute force (65,536 plans each)."""
    rng = wl.SplitMix64(77)
    p = wl.make_pipeline([-1, 0, 1, 0], 3, 1, (1, 4), rng)
    p.variant_factor_q4 = [3 + (a - 600000) // 60000 for a in p.acc_ppm]
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    assert n == 16 ** 4
    r = random.Random(5)
    demands = [r.randint(0, 400_000) for _ in range(4000)]
    out = P.alloc_search(demands, 10, 700_000)
    scored = P.last_search_plans_scored()
    assert scored < n * len(demands)
    found = 0
    for j in list(range(0, len(demands), 131)) + [len(demands) - 1]:
        check(out[j], O.search(demands[j], 10, 700_000), f"point {j} demand {demands[j]}")
        found += out[j].status == binding.LOKI_FOUND
    assert found >= 5
