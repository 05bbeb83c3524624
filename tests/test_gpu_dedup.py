"""GPU parity of mole_dedup_ids: distinct ids, inverse map and count are bit-exact against the oracle
(which is pinned to numpy.unique); the visiting plan is checked for validity (any order of tokens with
equal ids is correct, so only what is unique is compared)."""
import numpy as np
import pytest

import oracle
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl

pytestmark = pytest.mark.gpu

PLAN_HEADER, PLAN_SINGLE = 16, 0x80000000


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
    """The plan lists every token once, in id order (out-of-range ids last); the order of tokens with
    equal ids is free.  Bit 31 marks tokens whose id occurs once."""
    T = len(ids)
    assert plan[0] == U and plan[2] == T and plan[4] == V
    o_uniq, o_order, o_start = PLAN_HEADER, PLAN_HEADER + T, PLAN_HEADER + 2 * T
    np.testing.assert_array_equal(plan[o_uniq:o_uniq + U], uniq)
    raw = plan[o_order:o_order + T].astype(np.int64) & 0xFFFFFFFF
    order, single = (raw & 0x7FFFFFFF).astype(np.int64), (raw & PLAN_SINGLE) != 0
    np.testing.assert_array_equal(np.sort(order), np.arange(T))               # a permutation of the tokens
    in_range = (ids >= 0) & (ids < V)
    key = np.where(in_range, ids.astype(np.int64), np.int64(V))               # out-of-range ids sort last
    assert (np.diff(key[order]) >= 0).all()                                   # id order
    counts = np.bincount(ids[in_range], minlength=V)
    want_single = in_range[order] & (counts[np.where(in_range, ids, 0)][order] == 1)
    np.testing.assert_array_equal(single, want_single)
    start = plan[o_start:o_start + U + 2]
    np.testing.assert_array_equal(start[:U], np.concatenate([[0], np.cumsum(counts[uniq])])[:U])
    assert start[U] == in_range.sum() and start[U + 1] == T


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


@pytest.mark.parametrize("T,V,dist", [(256, 50304, "zipf"), (16384, 50304, "zipf"), (17000, 50304, "uniform"),
                                      (20000, 50304, "zipf")])
def test_generic_kernel(tuning, T, V, dist):
    """The kernel for batches beyond 16 tokens per thread (or V too large for the LDS staging area),
    forced on sizes the register-resident one would take, with and without its LDS staging."""
    tuning("MOLE_DEDUP_GENERIC", "1")
    ids = wl.make_ids(T, V, seed=T + 1, dist=dist)
    ids[T // 2] = V + 1
    uniq, inv, U, err, plan = run_dedup(ids, V)
    r_uniq, r_inv, r_U, r_err = oracle.dedup(ids, V)
    assert U == r_U and err == r_err == 1
    np.testing.assert_array_equal(uniq, r_uniq)
    np.testing.assert_array_equal(inv, r_inv)
    check_plan(plan, ids, V, uniq, U)


@pytest.mark.parametrize("T,V,dist", [(4097, 50304, "zipf"), (8192, 50304, "uniform"), (16384, 50304, "zipf"),
                                      (16384, 7, "uniform"), (9000, 200, "zipf"), (12000, 524288, "uniform")])
@pytest.mark.parametrize("split", [True, False])
def test_large_batches_one_and_eight_workgroups(tuning, T, V, dist, split):
    """Batches of more than 4096 tokens take the kernel that spreads the id ranges over eight workgroups;
    the one-workgroup kernel stays reachable.  Out-of-range ids (the last bucket of the last workgroup), ids at
    both ends of the range, V smaller than the number of workgroups' words."""
    if not split:
        tuning("MOLE_DEDUP_GENERIC", "2")
    ids = wl.make_ids(T, V, seed=7 * T + V, dist=dist)
    ids[[1, T // 2, T - 1]] = [V + 3, -1, V]
    ids[[0, 2]] = [0, V - 1]
    uniq, inv, U, err, plan = run_dedup(ids, V)
    r_uniq, r_inv, r_U, r_err = oracle.dedup(ids, V)
    assert U == r_U and err == r_err == 1
    np.testing.assert_array_equal(uniq, r_uniq)
    np.testing.assert_array_equal(inv, r_inv)
    check_plan(plan, ids, V, uniq, U)


@pytest.mark.parametrize("seed", range(16))
def test_seeded_random_batches(tuning, seed):
    """T, V, the id distribution, the share of out-of-range ids and the kernel drawn at random."""
    rng = np.random.default_rng(4000 + seed)
    T = int(rng.choice([1, 2, 63, 64, 65, 1023, 1024, 1025, 4097, 9000, 16384, 16385, 30000]))
    V = int(rng.choice([1, 2, 31, 32, 33, 1000, 50304, 200000]))
    which = int(rng.integers(4))
    if which < 2:
        tuning("MOLE_DEDUP_GENERIC", str(which + 1))        # 1: the generic kernel, 2: one workgroup only
    ids = wl.make_ids(T, V, seed=seed, dist=str(rng.choice(["zipf", "uniform"])))
    bad = rng.random(T) < float(rng.choice([0.0, 0.01, 0.5]))
    ids = np.where(bad, rng.choice(np.array([-1, V, V + 7, 2 ** 31 - 1], np.int64), T), ids).astype(np.int32)
    uniq, inv, U, err, plan = run_dedup(ids, V)
    r_uniq, r_inv, r_U, r_err = oracle.dedup(ids, V)
    assert U == r_U and err == r_err
    np.testing.assert_array_equal(uniq, r_uniq)
    np.testing.assert_array_equal(inv, r_inv)
    check_plan(plan, ids, V, uniq, U)


def test_dedup_edge_cases():
    uniq, inv, U, err, plan = run_dedup(np.zeros((0,), np.int32), 100)
    assert U == 0 and err == 0 and plan[0] == 0 and plan[5] == 0x4D4F4C45
    ids = np.full((100,), 42, np.int32)
    uniq, inv, U, err, plan = run_dedup(ids, 100)
    assert U == 1 and list(uniq) == [42] and (inv == 0).all()
    check_plan(plan, ids, 100, uniq, U)
    ids = np.array([5, 99, 100, -1, 5, 2 ** 31 - 1, 0], np.int32)
    uniq, inv, U, err, plan = run_dedup(ids, 100)
    r_uniq, r_inv, r_U, r_err = oracle.dedup(ids, 100)
    assert err == 1 == r_err and U == r_U
    np.testing.assert_array_equal(uniq, r_uniq)
    np.testing.assert_array_equal(inv, r_inv)
    check_plan(plan, ids, 100, uniq, U)


@pytest.mark.parametrize("case", ["all equal", "out of range", "two hot ids", "all distinct", "edges of V"])
def test_degenerate_large_batches(case):
    """One id for everybody, ids outside the table throughout, two ids sharing the batch, all distinct
    (descending), first / last ids of V and of a bitmap word."""
    T, V = 6000, 50304
    rng = np.random.default_rng(5)
    if case == "all equal":
        ids = np.full((T,), 777, np.int32)
    elif case == "out of range":
        ids = rng.integers(0, V, T).astype(np.int32)
        ids[::7] = V + 3
        ids[5::64] = -9
    elif case == "two hot ids":
        ids = np.where(rng.random(T) < 0.5, 31, 32).astype(np.int32)
    elif case == "all distinct":
        ids = np.arange(T, dtype=np.int32)[::-1].copy()
    else:
        ids = rng.choice(np.array([0, 1, 31, 32, V - 33, V - 32, V - 1], np.int32), T)
    uniq, inv, U, err, plan = run_dedup(ids, V)
    r_uniq, r_inv, r_U, r_err = oracle.dedup(ids, V)
    assert U == r_U and err == r_err
    np.testing.assert_array_equal(uniq, r_uniq)
    np.testing.assert_array_equal(inv, r_inv)
    check_plan(plan, ids, V, uniq, U)


def test_expected_distinct_counts_of_the_workloads():
    """The Zipf(1.1) batches have the reuse the benchmark configurations rely on."""
    for name, lo, hi in [("decode410m", 120, 180), ("prefill410m", 3700, 4600), ("prefill410m_uniform", 13500, 14500)]:
        w = wl.CONFIGS[name]
        ids = wl.token_ids(w)
        _, _, U, _, _ = run_dedup(ids, w.V)
        assert lo < U < hi, (name, U)
