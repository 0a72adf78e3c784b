"""The kernel that scores whole plans per lane fills the variants (eq. (2), Algorithm 1's fill rule) in 32-bit
arithmetic where the host has shown that every capacity and demand of the call fits, else in 64-bit: both against
the CPU checker, bit for bit, on problems that force each."""
import copy
import struct

import pytest

import oracle
from paper_2407_03583_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

TIE = binding.LOKI_TIE_INDEX_ONLY
LANE = binding.LOKI_SEARCH_PER_LANE


def bits(x):
    return struct.unpack("<Q", struct.pack("<d", x))[0]


def agree(res, ref):
    got, want = res.as_tuple(), ref.as_tuple()
    return got[0] == want[0] and bits(got[1]) == bits(want[1]) and got[2:] == want[2:]


def searches_agree(w, p, demands, want_bits):
    P, O = binding.Problem(p), oracle.Problem(p)
    found = 0
    for flags in (LANE, LANE | TIE):
        out = P.alloc_search(demands, w.workers, w.slo_us, w.comm_us, flags=flags)
        assert P.last_search_fill_bits() == want_bits
        for d, res in zip(demands, out):
            ref = O.search(d, w.workers, w.slo_us, w.comm_us, tie_index_only=bool(flags & TIE))
            assert agree(res, ref), (d, flags, res.as_tuple(), ref.as_tuple())
            found += ref.found
    n = P.num_candidates()
    a, b = n // 3, n - n // 5
    res = P.alloc_search(demands[:1], w.workers, w.slo_us, w.comm_us, flags=LANE, begin=a, end=b)[0]
    assert agree(res, O.search(demands[0], w.workers, w.slo_us, w.comm_us, begin=a, end=b))
    return found


@pytest.mark.parametrize("variant_factors", [False, True])
@pytest.mark.parametrize("per_variant_batch", [False, True])
def test_both_widths_on_small_random_problems(variant_factors, per_variant_batch):
    found32 = found64 = 0
    for seed in range(24):
        w = wl.random_small(seed, max_candidates=6000, variant_factors=variant_factors, per_variant_batch=per_variant_batch)
        found32 += searches_agree(w, w.pipeline, w.demand_mqps[:2], 32)
        # one variant with a throughput of 2^33 milli-QPS per replica: its capacity is beyond 32 bits, and a plan
        # that hosts it serves any demand with it
        p = copy.deepcopy(w.pipeline)
        nb = p.n_batches[0]
        k = max(range(p.n_variants[0]), key=lambda v: (p.max_replicas[v] > 0, (v + seed) % p.n_variants[0]))
        for b in range(nb):
            p.thr_mqps[k * nb + b] = 1 << 33
        if p.max_replicas[k] > 0:   # (a first task whose variants may not be hosted at all cannot be made wide)
            found64 += searches_agree(w, p, w.demand_mqps[:2], 64)
    assert found32 >= 4 and found64 >= 4, (found32, found64)


def test_a_demand_beyond_32_bits():
    """1.2e6 and 1.5e6 QPS at the root of a two-task chain: 6e9 and 7.5e9 at the second task in its own units
    (quarters of a milli-QPS, fan-out 1.25), beyond 32 bits, so the demand alone rules the 32-bit fill out;
    replicas of 2^29 .. 2^33 milli-QPS serve it."""
    p = wl.Pipeline(n_tasks=2, parent=[-1, 0], fanout_q4=[4, 5], n_variants=[3, 2], n_batches=[1, 2], batch_size=[1, 1, 4],
                    max_replicas=[3, 2, 3, 3, 2], acc_ppm=[910_000, 780_000, 850_000, 930_000, 700_000],
                    latency_us=[9000, 4000, 6000, 8000, 12000, 3000, 5000],
                    thr_mqps=[1 << 29, 1 << 30, 3 << 28, 1 << 29, 3 << 29, 1 << 30, 1 << 31])
    w = wl.Workload(name="wide", seed=0, pipeline=p, demand_mqps=[1_200_000_000, 1_500_000_000], workers=9, slo_us=60_000,
                    comm_us=1000)
    assert searches_agree(w, p, w.demand_mqps, 64) >= 2


def test_config_2_takes_the_32_bit_fill():
    w = wl.config(2)
    P = binding.Problem(w.pipeline)
    n = P.num_candidates()
    res = P.alloc_search(w.demand_mqps, w.workers, w.slo_us, w.comm_us, flags=LANE)
    assert P.last_search_fill_bits() == 32
    ref = P.alloc_search(w.demand_mqps, w.workers, w.slo_us, w.comm_us)
    assert [r.as_tuple() for r in res] == [r.as_tuple() for r in ref] and n == 1 << 30


@pytest.mark.parametrize("wide", [False, True])
def test_stepping_through_the_choices_of_a_last_task_with_eight_variants(wide):
    """The per-lane search decodes the last task's choice once per strip of 64 and steps from there.  Here the
    last task has eight variants with replica limits 255, 0, 1, 0, 2, 1, 0, 1 (radices 256 and 1 among them, a
    carry out of the low four variants into the high four every 512 choices) and two batch sizes on top:
    12,288 choices, 147,456 plans with the first task's 12; whole space and ranges that start and end inside
    strips, both fill widths, against the CPU checker."""
    limits = [255, 0, 1, 0, 2, 1, 0, 1]
    acc = [600_000, 990_000, 950_000, 640_000, 900_000, 700_000, 980_000, 850_000]
    lat, thr = [], []
    for k in range(8):
        lat += [3000 + 900 * k, 5000 + 1100 * k]
        thr += [(40 + 7 * k) * 1000, (70 + 9 * k) * 1000]
    if wide:
        thr[8] = thr[9] = 1 << 33   # variant 4: one replica serves anything, and its capacity is beyond 32 bits
    p = wl.Pipeline(n_tasks=2, parent=[-1, 0], fanout_q4=[4, 6], n_variants=[2, 8], n_batches=[2, 2],
                    batch_size=[1, 4, 1, 8], max_replicas=[2, 1] + limits, acc_ppm=[900_000, 800_000] + acc,
                    latency_us=[4000, 7000, 3000, 5000] + lat, thr_mqps=[2_000_000, 3_500_000, 2_500_000, 4_000_000] + thr)
    P, O = binding.Problem(p), oracle.Problem(p)
    n = P.num_candidates()
    assert n == 12 * 12288
    found = 0
    for demand, W, slo in ((900_000, 40, 60_000), (2_400_000, 90, 45_000), (5_000_000, 200, 80_000), (0, 5, 30_000),
                           (12_000_000, 262, 100_000)):
        for flags in (LANE, LANE | TIE):
            res = P.alloc_search([demand], W, slo, 500, flags=flags)[0]
            assert P.last_search_fill_bits() == (64 if wide else 32)
            ref = O.search(demand, W, slo, 500, tie_index_only=bool(flags & TIE))
            assert agree(res, ref), (demand, W, flags, res.as_tuple(), ref.as_tuple())
            found += ref.found
        for a, b in ((12 * 500 + 7, 12 * 1100 + 3), (12 * 4090, 12 * 4103 + 5), (n - 12 * 70, n), (12 * 6143 + 11, 12 * 6145)):
            res = P.alloc_search([demand], W, slo, 500, flags=LANE, begin=a, end=b)[0]
            ref = O.search(demand, W, slo, 500, begin=a, end=b)
            assert agree(res, ref), (demand, W, a, b, res.as_tuple(), ref.as_tuple())
    assert found >= 6, found
