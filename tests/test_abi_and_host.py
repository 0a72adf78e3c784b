"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol,
and its host-side logic (validation, decode, routing table) agrees with the CPU
checker.  No kernels are launched."""
import os
import re
from types import SimpleNamespace

import pytest

import oracle
from paper_2407_03583_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "loki_alloc.h")).read()
    declared = set(re.findall(r"\b(loki_[a-z_]+)\s*\(", header))
    declared -= {"loki_problem"}  # type name
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(binding.EXPORTS)
    # the instruction-rate probe is a library of its own with a header of its own
    probe = set(re.findall(r"\b(loki_[a-z_]+)\s*\(", open(os.path.join(ROOT, "include", "loki_probe.h")).read()))
    assert probe == set(binding.PROBE_EXPORTS) and not probe & declared
    for name in probe:
        assert hasattr(binding.probe_lib(), name) and not hasattr(L, name), name


def test_num_candidates_and_decode_match_the_checker():
    for cfg in (1, 2, 3, 4, 5):
        w = wl.config(cfg)
        P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
        n = P.num_candidates()
        assert n == O.num_candidates() == w.pipeline.num_candidates()
        batches = w.pipeline.batch_size
        for idx in (0, 1, n - 1, n // 2, n // 3 + 7, 12345 % n):
            x, b = P.decode(idx)
            xo, beta = O.decode(idx)
            assert x == xo
            off = 0
            for i in range(w.pipeline.n_tasks):
                assert b[i] == batches[off + beta[i]]
                off += w.pipeline.n_batches[i]
        with pytest.raises(binding.LokiError) as e:
            P.decode(n)
        assert e.value.code == binding.LOKI_E_RANGE
        assert P.workspace_bytes(len(w.demand_mqps)) > 0


def test_validation_rejects_bad_inputs():
    good = dict(n_tasks=2, parent=[-1, 0], fanout_q4=[4, 8], n_variants=[1, 1], n_batches=[1, 1], batch_size=[1, 1],
                max_replicas=[2, 2], acc_ppm=[900000, 800000], latency_us=[5000, 6000], thr_mqps=[200000, 150000])
    binding.Problem(SimpleNamespace(**good))
    cases = [
        (dict(parent=[0, 0]), binding.LOKI_E_INVALID_GRAPH),
        (dict(parent=[-1, 1]), binding.LOKI_E_INVALID_GRAPH),
        (dict(parent=[-1, -1]), binding.LOKI_E_INVALID_GRAPH),
        (dict(n_tasks=9, parent=[-1] + list(range(8))), binding.LOKI_E_RANGE),
        (dict(fanout_q4=[4, 0]), binding.LOKI_E_RANGE),
        (dict(n_variants=[0, 1]), binding.LOKI_E_RANGE),
        (dict(n_batches=[1, 9]), binding.LOKI_E_RANGE),
        (dict(max_replicas=[2, 256]), binding.LOKI_E_RANGE),
        (dict(acc_ppm=[900000, 1000001]), binding.LOKI_E_RANGE),
        (dict(latency_us=[0, 6000]), binding.LOKI_E_RANGE),
        (dict(thr_mqps=[-1, 150000]), binding.LOKI_E_RANGE),
        (dict(variant_factor_q4=[4, 0]), binding.LOKI_E_RANGE),
        (dict(variant_factor_q4=[65, 4]), binding.LOKI_E_RANGE),
        (dict(path_acc_ppm=[1000001]), binding.LOKI_E_RANGE),
        (dict(path_acc_ppm=[-1]), binding.LOKI_E_RANGE),
        (dict(n_batches=[2, 1], batch_size=[2, 2, 1], latency_us=[5000, 5000, 6000],
              thr_mqps=[200000, 200000, 150000]), binding.LOKI_E_RANGE),
    ]
    for change, code in cases:
        bad = dict(good)
        bad.update(change)
        with pytest.raises(binding.LokiError) as e:
            binding.Problem(SimpleNamespace(**bad))
        assert e.value.code == code, change
    binding.Problem(SimpleNamespace(**dict(good, path_acc_ppm=[123456])))
    # more profiled path accuracies than the library takes: a chain of 6 tasks with 8 variants each
    deep = dict(n_tasks=6, parent=[-1, 0, 1, 2, 3, 4], fanout_q4=[4] * 6, n_variants=[8] * 6, n_batches=[1] * 6,
                batch_size=[1] * 6, max_replicas=[1] * 48, acc_ppm=[500000] * 48, latency_us=[1000] * 48,
                thr_mqps=[1000] * 48, path_acc_ppm=[0] * 8)   # the count is checked before the table is read
    with pytest.raises(binding.LokiError) as e:
        binding.Problem(SimpleNamespace(**deep))
    assert e.value.code == binding.LOKI_E_RANGE
    # too many choices in one task: 8 variants with 255 replicas
    big = dict(n_tasks=1, parent=[-1], fanout_q4=[4], n_variants=[8], n_batches=[1], batch_size=[1],
               max_replicas=[255] * 8, acc_ppm=[1] * 8, latency_us=[1] * 8, thr_mqps=[1] * 8)
    with pytest.raises(binding.LokiError):
        binding.Problem(SimpleNamespace(**big))


@pytest.mark.parametrize("seed", range(30))
def test_route_table_matches_the_checker(seed):
    w = wl.random_small(700 + seed, max_tasks=4, max_candidates=5000, variant_factors=seed % 2 == 1,
                        per_variant_batch=seed % 3 == 2)
    P, O = binding.Problem(w.pipeline), oracle.Problem(w.pipeline)
    n = P.num_candidates()
    d = w.demand_mqps[0]
    for idx in {0, n - 1, n // 2, (seed * 7919) % n}:
        r, ro = P.route_table(idx, d), O.route_table(idx, d)
        x, batch = P.decode(idx)
        v = 0
        for i in range(w.pipeline.n_tasks):
            assert (r.demand[i], r.scale[i], r.unserved[i]) == (ro.demand[i], ro.scale[i], ro.unserved[i])
            for k in range(w.pipeline.n_variants[i]):
                assert r.replicas[i][k] == x[v + k]
                want_batch = batch[v + k] if w.pipeline.per_variant_batch else (batch[i] if x[v + k] > 0 else 0)
                assert r.batch[i][k] == want_batch
                assert (r.capacity[i][k], r.routed[i][k], r.leftover[i][k], r.budget_us[i][k]) == \
                    (ro.capacity[i][k], ro.routed[i][k], ro.leftover[i][k], ro.budget_us[i][k])
                for k2 in range(oracle.MAX_VARIANTS):
                    assert r.prob[i][k][k2] == ro.prob[i][k][k2]
            v += w.pipeline.n_variants[i]
    with pytest.raises(binding.LokiError):
        P.route_table(n, d)
    with pytest.raises(binding.LokiError):
        P.route_table(0, -1)


def test_workload_generator_is_stable():
    """Digest of every benchmark configuration's arrays (guards against drift of the generator)."""
    import json
    path = os.path.join(ROOT, "tests", "golden", "workload_digests.json")
    want = json.load(open(path))
    for cfg in (1, 2, 3, 4, 5):
        assert wl.config(cfg).digest() == want[str(cfg)], cfg


def test_decode_with_per_variant_batch_sizes():
    for seed in range(10):
        w = wl.random_small(900 + seed, max_variants=2, max_replicas=2, max_candidates=5000, per_variant_batch=True)
        p = w.pipeline
        P, O = binding.Problem(p), oracle.Problem(p)
        n = P.num_candidates()
        assert n == O.num_candidates() == p.num_candidates()
        for idx in {0, n - 1, n // 2, (seed * 104729) % n}:
            x, batch = P.decode(idx)
            xo, beta = O.decode(idx)
            assert x == xo
            v = b = 0
            for i in range(p.n_tasks):
                for k in range(p.n_variants[i]):
                    assert batch[v + k] == (p.batch_size[b + beta[v + k]] if x[v + k] > 0 else 0)
                v += p.n_variants[i]
                b += p.n_batches[i]


def test_bench_refuses_more_than_one_gpu_and_counts_operations():
    """bench.py: more than one GPU is refused with a message (one GPU per run); the operation counts
    behind `roofline.achieved` are the documented ones."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""
    sys.path.insert(0, root)
    import bench
    p5 = wl.config(5).pipeline
    assert bench.algorithmic_lane_ops(4, 2, False, p5) == 3          # multiply, add, max/compare
    assert bench.algorithmic_lane_ops(3, 1, False, wl.config(2).pipeline) == 2
    assert bench.algorithmic_lane_ops(1, 1, False, p5) == 1
    assert bench.algorithmic_lane_ops(4, 2, True, p5) == (8 * 4 + 12) + 3 * (8 * 4 + 32) / 64.0
    assert abs(bench.VALU_PEAK_TLANEOPS - 39.3216) < 1e-9
    # the HBM traffic figure is reported only for the sources it was measured with
    t = bench.measured_traffic("cfg5_tree4_k4", "tabulated")
    assert t is None or t == (2175 + 7216) * 1024
    assert bench.measured_traffic("cfg1_chain2_k3", "tabulated") is None


def test_workspace_covers_the_searches_a_handle_may_run():
    """The size a caller must provide grows with what the handle's searches keep on the device: with
    per-variant factors the descriptors of up to 65,535 (demand point, classes) points and a batch of per-point
    task tables; with profiled path accuracies the table itself, and on trees with two or more leaves the same
    descriptors and batch.  Chains, stars and deeper trees alike."""
    import copy
    for cfg in (2, 4, 5):
        w = wl.config(cfg)
        plain = binding.Problem(w.pipeline).workspace_bytes(4)
        p = copy.deepcopy(w.pipeline)
        p.variant_factor_q4 = [4] * len(p.acc_ppm)
        with_factors = binding.Problem(p).workspace_bytes(4)
        assert with_factors > plain + 65_535 * 8 * (8 + 8 + 4), (cfg, plain, with_factors)
        assert with_factors < (1 << 30)
        q = copy.deepcopy(w.pipeline)
        q.path_acc_ppm = wl.draw_path_tables(q, wl.SplitMix64(1))
        with_tables = binding.Problem(q).workspace_bytes(4)
        if cfg == 2:   # a chain: the plan space is walked as without tables
            assert plain < with_tables <= plain + 8 * len(q.path_acc_ppm) + 256
        else:          # two leaves: searched point by point like per-variant factors (one point per demand point)
            assert with_factors <= with_tables <= with_factors + 8 * len(q.path_acc_ppm) + 256
    # that route is taken with at most 64 variant combinations above every leaf: a path of five tasks with two
    # variants each has 16 above its leaf, with three variants 81
    for k, by_leaf in ((2, True), (3, False)):
        t = wl.make_pipeline([-1, 0, 1, 2, 3, 0], k, 1, (2,), wl.SplitMix64(3))
        plain = binding.Problem(t).workspace_bytes(4)
        t.path_acc_ppm = wl.draw_path_tables(t, wl.SplitMix64(4))
        with_tables = binding.Problem(t).workspace_bytes(4)
        assert (with_tables > plain + 65_535 * 8 * (8 + 8 + 4)) == by_leaf, (k, plain, with_tables)


def test_static_scratch_search_refuses_oversize_before_touching_the_gpu():
    """The limits of the entry point that allocates nothing are checked on the host, ahead of any HIP call."""
    import ctypes as C
    w = wl.config(3)
    P = binding.Problem(w.pipeline)
    n = P.num_candidates()
    for m in (64, 65):
        out = (binding.Result * m)()
        rc = binding.lib().loki_alloc_search_static(P._h, (C.c_int64 * m)(*([w.demand_mqps[0]] * m)), m, w.workers,
                                                    w.slo_us, 0, 0, 0, n, None, out)
        assert rc == binding.LOKI_E_STATIC_LIMIT
    assert b"static" in binding.lib().loki_strerror(binding.LOKI_E_STATIC_LIMIT)
    header = open(os.path.join(ROOT, "include", "loki_alloc.h")).read()
    assert f"#define LOKI_STATIC_SCRATCH_BYTES ({binding.LOKI_STATIC_SCRATCH_BYTES >> 20}u << 20)" in header
    assert f"#define LOKI_STATIC_MAX_DEMAND_POINTS {binding.LOKI_STATIC_MAX_DEMAND_POINTS}" in header
