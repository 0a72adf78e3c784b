"""The search that allocates nothing (loki_alloc_search_static) against loki_alloc_search, through the C-ABI."""
import struct

import pytest

from paper_2407_03583_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

TIE, LANE = binding.LOKI_TIE_INDEX_ONLY, binding.LOKI_SEARCH_PER_LANE


def same(a, b):
    ta, tb = a.as_tuple(), b.as_tuple()
    return ta[0] == tb[0] and struct.pack("<d", ta[1]) == struct.pack("<d", tb[1]) and ta[2:] == tb[2:]


def test_static_scratch_search_equals_the_workspace_search_on_two_calls_in_a_row():
    """Config 2 (2^30 plans, three demand points), then the smaller config 1 in the same scratch array:
    what the first call left behind must not show in the second."""
    big, small = wl.config(2), wl.config(1)
    P2, P1 = binding.Problem(big.pipeline), binding.Problem(small.pipeline)
    d2 = [big.demand_mqps[0], big.demand_mqps[0] // 2, 0]
    want2 = P2.alloc_search(d2, big.workers, big.slo_us, big.comm_us)
    got2 = P2.alloc_search_static(d2, big.workers, big.slo_us, big.comm_us)
    assert all(same(g, w) for g, w in zip(got2, want2)), ([g.as_tuple() for g in got2], [w.as_tuple() for w in want2])
    assert any(w.status == binding.LOKI_FOUND for w in want2)
    for flags in (0, TIE, LANE):
        want1 = P1.alloc_search(small.demand_mqps, small.workers, small.slo_us, small.comm_us, flags=flags)
        got1 = P1.alloc_search_static(small.demand_mqps, small.workers, small.slo_us, small.comm_us, flags=flags)
        assert all(same(g, w) for g, w in zip(got1, want1)), (flags, got1[0].as_tuple(), want1[0].as_tuple())
    # an index range, and the first problem again after the small one
    n = P1.num_candidates()
    want = P1.alloc_search(small.demand_mqps, small.workers, small.slo_us, begin=n // 3, end=n // 2 + 7)
    got = P1.alloc_search_static(small.demand_mqps, small.workers, small.slo_us, begin=n // 3, end=n // 2 + 7)
    assert same(got[0], want[0])
    again = P2.alloc_search_static(d2, big.workers, big.slo_us, big.comm_us)
    assert all(same(g, w) for g, w in zip(again, want2))


def test_static_scratch_search_rejects_what_does_not_fit():
    """Config 3's 31,250 choices per demand point: 64 points need 33 MB of tables, 65 points exceed the limit on
    points; both are refused before anything is launched, and a search that fits still works afterwards."""
    w = wl.config(3)
    P = binding.Problem(w.pipeline)
    for m in (64, 65):
        with pytest.raises(binding.LokiError) as err:
            P.alloc_search_static(list(w.demand_mqps[:1]) * m, w.workers, w.slo_us)
        assert err.value.code == binding.LOKI_E_STATIC_LIMIT
    d = list(w.demand_mqps[:2])
    assert all(same(g, r) for g, r in zip(P.alloc_search_static(d, w.workers, w.slo_us),
                                          P.alloc_search(d, w.workers, w.slo_us)))
