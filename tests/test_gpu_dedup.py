"""GPU parity of mole_dedup_ids: distinct ids, inverse map and count are bit-exact against the oracle
(which is pinned to numpy.unique); the grouping plan is checked for validity (any token order inside a
group is correct, so only what is unique is compared)."""
import numpy as np
import pytest

import oracle
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl

pytestmark = pytest.mark.gpu

PLAN_HEADER, PLAN_GROUP = 16, 8


def run_dedup(ids, V):
    import torch
    T = len(ids)
    ids_d = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).cuda()
    uniq = torch.full((max(T, 1),), -5, dtype=torch.int32, device="cuda")
    inv = torch.full((max(T, 1),), -5, dtype=torch.int32, device="cuda")
    nu = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.zeros((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, T, V, uniq, inv, nu, err, plan)
    torch.cuda.synchronize()
    U = int(nu.item())
    return uniq.cpu().numpy()[:U], inv.cpu().numpy()[:T], U, int(err.item()), plan.cpu().numpy()


def check_plan(plan, ids, V, uniq, U):
    T = len(ids)
    cap = 2 * T + 2
    n_items = plan[0]
    assert plan[1] == U and plan[2] == T and plan[3] == PLAN_GROUP and plan[4] == V
    o_uniq, o_order = PLAN_HEADER, PLAN_HEADER + T
    o_u, o_b, o_c = o_order + T, o_order + T + cap, o_order + T + 2 * cap
    np.testing.assert_array_equal(plan[o_uniq:o_uniq + U], uniq)
    order = plan[o_order:o_order + T]
    np.testing.assert_array_equal(np.sort(order), np.arange(T))               # a permutation of the tokens
    item_u, item_b, item_c = plan[o_u:o_u + n_items], plan[o_b:o_b + n_items], plan[o_c:o_c + n_items]
    assert (item_c >= 1).all() and (item_c <= PLAN_GROUP).all()
    assert item_c.sum() == T
    seen = np.zeros(T, bool)
    for u, b, c in zip(item_u, item_b, item_c):
        toks = order[b:b + c]
        assert not seen[toks].any()
        seen[toks] = True
        if u < U:
            assert (ids[toks] == uniq[u]).all()                               # a group reads one row block
        else:
            assert u == U and ((ids[toks] < 0) | (ids[toks] >= V)).all()      # the out-of-range bucket
    assert seen.all()
    in_range = ((ids >= 0) & (ids < V))
    counts = np.bincount(ids[in_range], minlength=1)
    want_items = sum((c + PLAN_GROUP - 1) // PLAN_GROUP for c in counts if c) + ((~in_range).sum() + 7) // 8
    assert n_items == want_items


@pytest.mark.parametrize("T,V,dist", [(1, 50304, "zipf"), (32, 50304, "zipf"), (64, 50304, "zipf"),
                                      (256, 50304, "zipf"), (16384, 50304, "zipf"), (16384, 50304, "uniform"),
                                      (256, 1024, "uniform"), (1000, 7, "uniform"), (5000, 524288, "uniform"),
                                      (40000, 50304, "zipf")])
def test_dedup_matches_oracle(T, V, dist):
    ids = wl.make_ids(T, V, seed=3 * T + V, dist=dist)
    uniq, inv, U, err, plan = run_dedup(ids, V)
    r_uniq, r_inv, r_U, r_err = oracle.dedup(ids, V)
    assert U == r_U and err == r_err == 0
    np.testing.assert_array_equal(uniq, r_uniq)
    np.testing.assert_array_equal(inv, r_inv)
    check_plan(plan, ids, V, uniq, U)


def test_dedup_edge_cases():
    uniq, inv, U, err, plan = run_dedup(np.zeros((0,), np.int32), 100)
    assert U == 0 and err == 0 and plan[0] == 0
    ids = np.full((100,), 42, np.int32)
    uniq, inv, U, err, plan = run_dedup(ids, 100)
    assert U == 1 and list(uniq) == [42] and (inv == 0).all() and plan[0] == 13
    check_plan(plan, ids, 100, uniq, U)
    ids = np.array([5, 99, 100, -1, 5, 2 ** 31 - 1, 0], np.int32)
    uniq, inv, U, err, plan = run_dedup(ids, 100)
    r_uniq, r_inv, r_U, r_err = oracle.dedup(ids, 100)
    assert err == 1 == r_err and U == r_U
    np.testing.assert_array_equal(uniq, r_uniq)
    np.testing.assert_array_equal(inv, r_inv)
    check_plan(plan, ids, 100, uniq, U)


def test_expected_distinct_counts_of_the_workloads():
    """The Zipf(1.1) batches have the reuse the benchmark configurations rely on."""
    for name, lo, hi in [("decode410m", 120, 180), ("prefill410m", 3700, 4600), ("prefill410m_uniform", 13500, 14500)]:
        w = wl.CONFIGS[name]
        ids = wl.token_ids(w)
        _, _, U, _, _ = run_dedup(ids, w.V)
        assert lo < U < hi, (name, U)
