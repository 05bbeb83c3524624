"""GPU parity of mole_lookup_forward / mole_lookup_forward_layers against the fp64 oracle.
Everything goes through the C ABI (via the ctypes binding).  Inputs are seeded and synthetic."""
import numpy as np
import pytest

import oracle
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl
from helpers import DT, assert_close, gathered_rows, to_dev, to_host

pytestmark = pytest.mark.gpu


def torch_mod():
    import torch
    return torch


def run_forward(w, table, ids, li, shared=True, residual=False, slot=None, rows=None, dedup=False,
                want_dbg=True, table_dev=None, runs=False):
    """One call of mole_lookup_forward on numpy inputs; returns numpy outputs."""
    torch = torch_mod()
    dev = "cuda"
    T = len(ids)
    tab_d = table_dev if table_dev is not None else to_dev(table, w.dtype)
    n_rows = rows if rows is not None else tab_d.shape[0]
    ids_d = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).to(dev)
    slot_d = None if slot is None else torch.from_numpy(np.ascontiguousarray(slot, dtype=np.int32)).to(dev)
    h_d, wr_d = to_dev(li["h"], w.dtype), to_dev(li["W_r"], w.dtype)
    sh_d = to_dev(li["shared"], w.dtype) if shared else None
    rs_d = to_dev(li["residual"], w.dtype) if residual else None
    out_d = torch.full((max(T, 1), w.d), float("nan"), dtype=h_d.dtype, device=dev)
    gates_d = torch.full((max(T, 1), w.N), -1.0, dtype=torch.float32, device=dev) if want_dbg else None
    rows_d = torch.full((max(T, 1),), -7, dtype=torch.int64, device=dev) if want_dbg else None
    err_d = torch.zeros((1,), dtype=torch.int32, device=dev)
    flags, plan = 0, None
    if dedup:
        plan = torch.empty((mb.mole_dedup_workspace(T, w.V) // 4,), dtype=torch.int32, device=dev)
        uq = torch.empty((max(T, 1),), dtype=torch.int32, device=dev)
        iv = torch.empty((max(T, 1),), dtype=torch.int32, device=dev)
        nu = torch.zeros((1,), dtype=torch.int32, device=dev)
        mb.mole_dedup_ids(ids_d, T, w.V, uq, iv, nu, err_d, plan)
        flags = mb.MOLE_FLAG_DEDUP | (mb.MOLE_FLAG_RUNS if runs else 0)
    mb.mole_lookup_forward(tab_d, ids_d, slot_d, h_d, wr_d, sh_d, rs_d, out_d, gates_d, rows_d, err_d,
                           T, n_rows, w.d, w.N, DT[w.dtype], flags, plan)
    torch.cuda.synchronize()
    res = dict(out=to_host(out_d, w.dtype)[:T], err=int(err_d.item()))
    if want_dbg:
        res["gates"] = gates_d.cpu().numpy()[:T]
        res["rows"] = rows_d.cpu().numpy()[:T]
    return res


def check_against_oracle(w, table, ids, li, shared=True, residual=False, dedup=False, runs=False):
    ref_out, ref_g, ref_rows, ref_err = oracle.lookup_forward(
        table, ids, li["h"], li["W_r"], li["shared"] if shared else None, li["residual"] if residual else None)
    got = run_forward(w, table, ids, li, shared=shared, residual=residual, dedup=dedup, runs=runs)
    np.testing.assert_array_equal(got["rows"], ref_rows)                     # gathered row indices: bit-exact
    assert got["err"] == ref_err
    assert_close(got["gates"].astype(np.float64), ref_g, wl.F32 if w.dtype == wl.F32 else wl.BF16, "gates")
    assert_close(wl.storage_to_f64(got["out"], w.dtype), ref_out, w.dtype, f"out ({w.name})")
    # the kernels that write no debug outputs are variants of their own (same arithmetic): the same bits
    plain = run_forward(w, table, ids, li, shared=shared, residual=residual, dedup=dedup, runs=runs, want_dbg=False)
    np.testing.assert_array_equal(plain["out"], got["out"])
    assert plain["err"] == got["err"]
    return got


# ---- config 1: the tiny fp32 layer, table built by the (pinned) oracle ------------------------------
def test_tiny_fp32_layer():
    w = wl.CONFIGS["tiny"]
    ew = wl.expert_weights(w)
    table = oracle.build_lut(ew["E"], ew["W1"], ew["W2"]).astype(np.float32)
    li, ids = wl.layer_inputs(w), wl.token_ids(w)
    got = check_against_oracle(w, table, ids, li)
    assert np.abs(got["gates"].sum(axis=1) - 1.0).max() < 1e-6                 # gates sum to one


# ---- bf16 shapes: several tiles, ragged tails, every specialised N, generic N, d not a multiple of 512 ----
@pytest.mark.parametrize("d,N,T,V", [
    (1024, 16, 333, 4096),     # 410M-shaped rows, T not a multiple of the workgroup's tokens
    (768, 16, 64, 4096),       # 160M-shaped: d = 1.5 chunks of 512 columns
    (1024, 32, 203, 2048),     # prefill-shaped N
    (2048, 4, 77, 1024),       # 1B-shaped
    (256, 8, 130, 512),
    (128, 64, 50, 300),
    (1024, 64, 75, 300),       # N = 64: the experts of a chunk pass through the row registers in two halves
    (520, 64, 9, 64),
    (520, 16, 9, 64),          # d = 512 + 8: a chunk with a single active lane
    (1024, 2, 70, 512),        # two experts: the router is padded to four, the extra gates must be exactly 0
    (520, 2, 9, 64),
    (64, 1, 40, 100),          # generic path
    (1024, 5, 33, 256),        # generic path, N not a power of two
    (512, 12, 31, 256),
    (4096, 16, 20, 64),        # router weight of 131 KB: one workgroup per CU
    (8192, 16, 10, 32),        # router weight too large for LDS: generic path
    (4096, 32, 12, 32),        # the same at N = 32
])
@pytest.mark.parametrize("residual", [False, True])
def test_bf16_shapes(d, N, T, V, residual):
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"bf16 d{d} N{N} T{T}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    li["W_r"] = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)    # gates well away from 1/N
    check_against_oracle(w, table, ids, li, residual=residual)


@pytest.mark.parametrize("split", ["1", "2"])
@pytest.mark.parametrize("wpb", ["4", "8"])
@pytest.mark.parametrize("d,N,T,V", [(1024, 16, 333, 4096), (768, 16, 64, 4096), (1544, 8, 50, 300), (1024, 32, 203, 2048),
                                     (1024, 64, 41, 100)])
def test_launch_variants(tuning, split, wpb, d, N, T, V):
    """Both item granularities (whole token / one 512-column chunk) and both workgroup widths."""
    tuning("MOLE_FWD_SPLIT", split)
    tuning("MOLE_FWD_WPB", wpb)
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"split{split} wpb{wpb} d{d} N{N}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    ids = ids.copy()
    ids[T // 2] = V + 5                                    # an out-of-range id in the middle of the stream
    for dedup in (False, True):
        ref_out, ref_g, ref_rows, ref_err = oracle.lookup_forward(table, ids, li["h"], li["W_r"], li["shared"], li["residual"])
        got = run_forward(w, table, ids, li, residual=True, dedup=dedup)
        assert got["err"] == 1 == ref_err
        np.testing.assert_array_equal(got["rows"], ref_rows)
        assert_close(got["gates"].astype(np.float64), ref_g, wl.BF16, "gates")
        assert_close(wl.storage_to_f64(got["out"], w.dtype), ref_out, w.dtype, f"out ({w.name})")


@pytest.mark.parametrize("d,N,T", [(64, 4, 256), (128, 16, 100), (32, 3, 17)])
def test_fp32_shapes(d, N, T):
    w = wl.scaled(wl.CONFIGS["tiny"], V=777, d=d, N=N, T=T, name=f"fp32 d{d} N{N}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    li["W_r"] = (li["W_r"] * np.float32(5.0)).astype(np.float32)
    check_against_oracle(w, table, ids, li, residual=True)


def test_routed_term_alone():
    """Without the O(1) shared term the routed term (~0.02) carries the whole comparison."""
    w = wl.scaled(wl.CONFIGS["decode410m"], V=2048, T=100, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    got = check_against_oracle(w, table, ids, li, shared=False)
    assert np.abs(wl.storage_to_f64(got["out"], w.dtype)).mean() > 1e-3


@pytest.mark.parametrize("seed", range(24))
def test_seeded_random_shapes(tuning, seed):
    """Shapes drawn from the documented ranges (d a multiple of 8 up to 2304, any N up to 64, small T and V),
    with a random choice of residual, plan, out-of-range ids and of the launch switches: every dispatch
    path (streaming, chunk items, run kernel, generic) against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.integers(1, 289)) * 8
    N = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 24, 32, 33, 48, 64]))
    T = int(rng.integers(1, 90))
    V = int(rng.integers(max(2, T // 8), 400))
    dedup, residual = bool(rng.integers(2)), bool(rng.integers(2))
    for var in ("MOLE_FWD_SPLIT", "MOLE_FWD_NTA", "MOLE_FWD_RUN"):
        tuning(var, str(int(rng.integers(1, 3))))
    tuning("MOLE_FWD_WPB", str(int(rng.choice([4, 8]))))
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, ids=str(rng.choice(["zipf", "uniform"])),
                  name=f"random seed {seed}: d{d} N{N} T{T} V{V} dedup{int(dedup)} res{int(residual)}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    li["W_r"] = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)
    ids = ids.copy()
    if rng.integers(2) and T > 2:
        ids[int(rng.integers(T))] = V + int(rng.integers(1, 5))
    check_against_oracle(w, table, ids, li, residual=residual, dedup=dedup)


@pytest.mark.parametrize("d,N,T,V,dedup,runs,residual", [
    (1032, 32, 16384, 900, False, False, True),   # N = 32: rows in two parts of 16, doubled grid, ragged third chunk
    (520, 32, 20000, 2500, False, False, False),
    (1024, 64, 9001, 400, False, False, True),    # N = 64: four parts
    (1544, 32, 16384, 1200, True, False, False),  # with a plan: the streaming kernel in id order
    (1544, 32, 16384, 1200, True, True, False),   # MOLE_FLAG_RUNS: the run kernel
    (1024, 16, 9001, 300, True, True, True),
    (768, 16, 20000, 700, False, False, True),
])
def test_large_batches_with_many_experts(d, N, T, V, dedup, runs, residual):
    """Whole outputs of large single-layer batches against the oracle (the full-size tests sample theirs)."""
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"large d{d} N{N} T{T}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    li["W_r"] = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)
    check_against_oracle(w, table, ids, li, residual=residual, dedup=dedup, runs=runs)


def test_plan_does_not_change_a_bit_and_the_run_hint_stays_in_tolerance():
    """MOLE_FLAG_DEDUP alone: the same bits as the plain call.  MOLE_FLAG_RUNS: another summation order."""
    w = wl.scaled(wl.CONFIGS["decode410m"], V=500, d=1024, N=32, T=9000, L=1, name="flags N32")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    plain = run_forward(w, table, ids, li, residual=True)
    planned = run_forward(w, table, ids, li, residual=True, dedup=True)
    hinted = run_forward(w, table, ids, li, residual=True, dedup=True, runs=True)
    np.testing.assert_array_equal(plain["out"], planned["out"])
    np.testing.assert_array_equal(plain["gates"], planned["gates"])
    assert_close(wl.storage_to_f64(hinted["out"], w.dtype), wl.storage_to_f64(plain["out"], w.dtype), w.dtype,
                 "run hint against the plain call")
    assert not np.array_equal(hinted["out"], plain["out"])      # it did take the other kernel


@pytest.mark.parametrize("cfg,d,N", [("decode410m", 512, 64), ("tiny", 64, 4), ("decode410m", 256, 5)])
def test_run_hint_is_ignored_where_it_does_not_apply(cfg, d, N):
    """MOLE_FLAG_RUNS is defined for bf16 and N <= 32 (powers of two): elsewhere the call is the planned one."""
    w = wl.scaled(wl.CONFIGS[cfg], V=300, d=d, N=N, T=500, L=1, name=f"hint ignored {cfg} N{N}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    planned = run_forward(w, table, ids, li, dedup=True)
    hinted = run_forward(w, table, ids, li, dedup=True, runs=True)
    np.testing.assert_array_equal(planned["out"], hinted["out"])
    check_against_oracle(w, table, ids, li, dedup=True, runs=True)


# ---- special cases with exact answers ----------------------------------------------------------------
@pytest.mark.parametrize("N", [16, 5])
def test_saturated_router_returns_the_row_exactly(N):
    w = wl.scaled(wl.CONFIGS["decode410m"], V=512, d=256, N=N, T=64, L=1)
    table, ids = wl.random_table(w), wl.token_ids(w)
    h = np.zeros((w.T, w.d), np.float32)
    star, kk = np.arange(w.T) % N, np.arange(w.T)
    h[np.arange(w.T), kk] = 1.0
    Wr = np.zeros((w.d, N), np.float32)
    Wr[kk, star] = 1.0e4
    li = dict(h=wl.to_storage(h, w.dtype), W_r=wl.to_storage(Wr, w.dtype), shared=None, residual=None)
    got = run_forward(w, table, ids, li, shared=False)
    np.testing.assert_array_equal(wl.storage_to_f64(got["out"], w.dtype),
                                  wl.storage_to_f64(table, w.dtype)[ids, star, :])
    onehot = np.zeros((w.T, N), np.float32)
    onehot[np.arange(w.T), star] = 1.0
    np.testing.assert_array_equal(got["gates"], onehot)


def test_zero_router_gives_mean_of_rows():
    w = wl.scaled(wl.CONFIGS["decode410m"], V=512, d=512, N=16, T=40, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    li["W_r"] = np.zeros_like(li["W_r"])
    got = run_forward(w, table, ids, li, shared=False)
    np.testing.assert_array_equal(got["gates"], np.full((w.T, w.N), 1.0 / 16, np.float32))
    ref = wl.storage_to_f64(table, w.dtype)[ids].mean(axis=1)
    assert_close(wl.storage_to_f64(got["out"], w.dtype), ref, w.dtype, "mean of rows")


# ---- edge cases --------------------------------------------------------------------------------------
def test_single_token_and_no_tokens():
    w = wl.scaled(wl.CONFIGS["decode410m"], V=1024, T=1, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    check_against_oracle(w, table, ids, li)
    got = run_forward(w, table, ids[:0], {k: v[:0] if k != "W_r" else v for k, v in li.items()})
    assert got["out"].shape[0] == 0 and got["err"] == 0


@pytest.mark.parametrize("N", [16, 5])
@pytest.mark.parametrize("dedup", [False, True])
def test_out_of_range_ids(N, dedup):
    w = wl.scaled(wl.CONFIGS["decode410m"], V=300, d=256, N=N, T=40, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    ids = ids.copy()
    ids[[3, 17, 39]] = [300, -1, 2 ** 31 - 1]
    ref_out, _, ref_rows, ref_err = oracle.lookup_forward(table, ids, li["h"], li["W_r"], li["shared"])
    got = run_forward(w, table, ids, li, dedup=dedup)
    assert got["err"] == 1 == ref_err
    np.testing.assert_array_equal(got["rows"], ref_rows)
    assert_close(wl.storage_to_f64(got["out"], w.dtype), ref_out, w.dtype, "out with bad ids")
    np.testing.assert_array_equal(got["out"][[3, 17, 39]], li["shared"][[3, 17, 39]])     # routed term = 0


def test_slot_indirection_reads_the_staging_rows():
    """row(t) = slot[t]: a compacted table of the distinct ids gives the same output bit for bit."""
    w = wl.scaled(wl.CONFIGS["decode410m"], V=2048, d=512, T=128, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    uniq, inv = np.unique(ids, return_inverse=True)
    a = run_forward(w, table, ids, li)
    b = run_forward(w, np.ascontiguousarray(table[uniq]), ids, li, slot=inv.astype(np.int32))
    np.testing.assert_array_equal(a["out"], b["out"])
    np.testing.assert_array_equal(b["rows"], inv)


# ---- dedup flag, layer-batched launch, determinism ---------------------------------------------------
@pytest.mark.parametrize("d,N,T,V,dist", [(1024, 16, 256, 4096, "zipf"), (1024, 32, 2000, 512, "zipf"),
                                           (768, 16, 64, 50304, "zipf"), (256, 5, 300, 40, "uniform"),
                                           (64, 4, 256, 1024, "uniform")])
def test_dedup_flag_does_not_change_the_output(d, N, T, V, dist):
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, ids=dist)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    a = check_against_oracle(w, table, ids, li, dedup=False)
    b = check_against_oracle(w, table, ids, li, dedup=True)
    np.testing.assert_array_equal(a["out"], b["out"])
    np.testing.assert_array_equal(a["gates"], b["gates"])


def test_heavy_repeats_with_plan():
    w = wl.scaled(wl.CONFIGS["decode410m"], V=64, d=256, N=16, T=500, L=1)
    table, li = wl.random_table(w), wl.layer_inputs(w)
    ids = np.full((w.T,), 7, np.int32)
    ids[::50] = 9
    check_against_oracle(w, table, ids, li, dedup=True)


# ---- the run kernel (MOLE_FLAG_RUNS; forced here through the environment on small shapes) ---------------
@pytest.mark.parametrize("d,N,T,V,dist", [
    (1024, 32, 203, 64, "zipf"),       # long runs of equal ids, two chunks
    (1024, 16, 333, 4096, "zipf"),     # mostly distinct ids
    (768, 16, 64, 40, "uniform"),      # d = 1.5 chunks
    (520, 8, 37, 16, "uniform"),       # a chunk with a single active lane
    (1544, 8, 50, 300, "zipf"),        # four chunks
    (1024, 2, 70, 32, "uniform"),      # two experts padded to one group of four
    (2048, 4, 77, 50, "zipf"),
    (256, 8, 130, 7, "uniform"),       # one chunk, runs longer than a span
    (1024, 16, 1, 100, "zipf"),
    (512, 32, 3, 100, "zipf"),
    (2048, 32, 40, 10, "uniform"),     # N = 32 with a router weight of 132 KB: one workgroup per CU
    (4096, 32, 12, 8, "uniform"),      # too large for the run kernel's LDS: falls back to the generic path
])
def test_run_kernel_shapes(tuning, d, N, T, V, dist):
    tuning("MOLE_FWD_RUN", "1")
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, ids=dist, name=f"run d{d} N{N} T{T} V{V}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    li["W_r"] = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)
    ids = ids.copy()
    if T > 8:
        ids[[2, T // 2]] = [V + 5, -3]                     # out-of-range ids: sorted last by the plan
    for residual in (False, True):
        check_against_oracle(w, table, ids, li, residual=residual, dedup=True)


@pytest.mark.parametrize("d,T,V,dist", [
    (1024, 1, 8, "uniform"),           # one token: 31 empty columns in the tile
    (1024, 31, 40, "zipf"),            # a ragged single tile
    (1024, 33, 10, "zipf"),            # one full tile and one token
    (1024, 1000, 300, "zipf"),         # many tiles, ragged tail
    (520, 70, 20, "uniform"),          # d / 8 odd: the last router step has one 16-byte piece; ragged chunk
    (2048, 130, 64, "zipf"),           # four chunks per token
    (72, 40, 12, "uniform"),           # fewer router steps than waves
    (1024, 600, 5000, "uniform"),      # mostly distinct ids
])
def test_tile_kernel_shapes(tuning, d, T, V, dist):
    """The tile kernel (N = 32, large batches), forced on small shapes, against the oracle: plain and planned
    order, with and without a residual, out-of-range ids."""
    tuning("MOLE_FWD_TILE", "1")
    w = wl.scaled(wl.CONFIGS["prefill410m"], V=V, d=d, N=32, T=T, L=1, ids=dist, name=f"tile d{d} T{T} V{V}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    li["W_r"] = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)
    ids = ids.copy()
    if T > 8:
        ids[[2, T // 2]] = [V + 5, -3]
    for residual in (False, True):
        for dedup in (False, True):
            check_against_oracle(w, table, ids, li, residual=residual, dedup=dedup)


def test_tile_kernel_with_slot_indirection(tuning):
    """Rows through the slot indirection (offloaded mode), gates and row indices reported."""
    tuning("MOLE_FWD_TILE", "1")
    w = wl.scaled(wl.CONFIGS["prefill410m"], V=300, d=1024, N=32, T=200, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    uniq, inv = np.unique(ids, return_inverse=True)
    ref_out, ref_g, _, _ = oracle.lookup_forward(table, ids, li["h"], li["W_r"], li["shared"])
    for dedup in (False, True):
        got = run_forward(w, np.ascontiguousarray(table[uniq]), ids, li, slot=inv.astype(np.int32), dedup=dedup)
        np.testing.assert_array_equal(got["rows"], inv)
        assert_close(wl.storage_to_f64(got["out"], w.dtype), ref_out, w.dtype, "tile kernel, staged rows")
        np.testing.assert_allclose(got["gates"], ref_g, rtol=2e-5, atol=1e-7)


def test_run_kernel_saturated_router_returns_the_row_exactly(tuning):
    """A gate of exactly 1 splits into hi = 1, lo = 0, and 0 into 0 + 0: the row comes back bit for bit."""
    tuning("MOLE_FWD_RUN", "1")
    N = 16
    w = wl.scaled(wl.CONFIGS["decode410m"], V=24, d=1024, N=N, T=96, L=1, ids="uniform")
    table, ids = wl.random_table(w), wl.token_ids(w)
    h = np.zeros((w.T, w.d), np.float32)
    star, kk = np.arange(w.T) % N, np.arange(w.T)
    h[np.arange(w.T), kk] = 1.0
    Wr = np.zeros((w.d, N), np.float32)
    Wr[kk, star] = 1.0e4
    li = dict(h=wl.to_storage(h, w.dtype), W_r=wl.to_storage(Wr, w.dtype), shared=None, residual=None)
    got = run_forward(w, table, ids, li, shared=False, dedup=True)
    np.testing.assert_array_equal(wl.storage_to_f64(got["out"], w.dtype),
                                  wl.storage_to_f64(table, w.dtype)[ids, star, :])


def test_run_kernel_with_slot_indirection(tuning):
    """Offloaded mode: the plan orders tokens by id, the rows come from the compacted staging table."""
    tuning("MOLE_FWD_RUN", "1")
    w = wl.scaled(wl.CONFIGS["decode410m"], V=300, d=1024, N=16, T=200, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    uniq, inv = np.unique(ids, return_inverse=True)
    ref_out, ref_g, _, _ = oracle.lookup_forward(table, ids, li["h"], li["W_r"], li["shared"])
    got = run_forward(w, np.ascontiguousarray(table[uniq]), ids, li, slot=inv.astype(np.int32), dedup=True)
    np.testing.assert_array_equal(got["rows"], inv)
    assert_close(wl.storage_to_f64(got["out"], w.dtype), ref_out, w.dtype, "run kernel, staged rows")


@pytest.mark.parametrize("dedup", [False, True])
@pytest.mark.parametrize("N,tile", [(16, False), (32, False), (32, True)])
def test_layer_batched_launch_equals_per_layer_calls(tuning, dedup, N, tile):
    """tile: the tile kernel forced for the batched launch and for the per-layer calls alike."""
    torch = torch_mod()
    if tile:
        tuning("MOLE_FWD_TILE", "1")
    w = wl.scaled(wl.CONFIGS["decode410m"], V=1024, d=512, N=N, T=70, L=3)
    ids = wl.token_ids(w)
    tabs = [wl.random_table(w, l) for l in range(w.L)]
    lis = [wl.layer_inputs(w, l) for l in range(w.L)]
    per_layer = [run_forward(w, tabs[l], ids, lis[l], residual=True, dedup=dedup) for l in range(w.L)]

    stack = lambda key: to_dev(np.stack([li[key] for li in lis]), w.dtype)
    tab_d = to_dev(np.stack(tabs), w.dtype)
    ids_d = torch.from_numpy(ids).cuda()
    h_d, wr_d, sh_d, rs_d = stack("h"), stack("W_r"), stack("shared"), stack("residual")
    out_d = torch.zeros_like(h_d)
    gates_d = torch.zeros((w.L, w.T, w.N), dtype=torch.float32, device="cuda")
    rows_d = torch.zeros((w.T,), dtype=torch.int64, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    flags, plan = 0, None
    if dedup:
        plan = torch.empty((mb.mole_dedup_workspace(w.T, w.V) // 4,), dtype=torch.int32, device="cuda")
        uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
        mb.mole_dedup_ids(ids_d, w.T, w.V, uq, iv, torch.zeros_like(err_d), err_d, plan)
        flags = mb.MOLE_FLAG_DEDUP
    mb.mole_lookup_forward_layers(tab_d, w.V * w.N * w.d, ids_d, None, h_d, wr_d, sh_d, rs_d, out_d, w.T * w.d,
                                  gates_d, rows_d, err_d, w.L, w.T, w.V, w.d, w.N, DT[w.dtype], flags, plan)
    torch.cuda.synchronize()
    out = to_host(out_d, w.dtype)
    for l in range(w.L):
        np.testing.assert_array_equal(out[l], per_layer[l]["out"])
        np.testing.assert_array_equal(gates_d[l].cpu().numpy(), per_layer[l]["gates"])
    np.testing.assert_array_equal(rows_d.cpu().numpy(), ids)
    assert int(err_d.item()) == 0


def test_two_runs_are_bit_identical():
    w = wl.scaled(wl.CONFIGS["decode410m"], V=4096, T=256, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    for dedup in (False, True):
        a = run_forward(w, table, ids, li, dedup=dedup)
        b = run_forward(w, table, ids, li, dedup=dedup)
        np.testing.assert_array_equal(a["out"], b["out"])


# ---- full benchmark sizes, in the launch configuration the benchmark times: WHOLE outputs ---------------
# The tables exist only on the device (up to 39.6 GB); the rows a batch looks up are copied back by plain
# indexing and the oracle runs on all tokens of all layers.
def _plan_for(torch, ids_d, T, V, err_d):
    plan = torch.empty((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
    uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
    mb.mole_dedup_ids(ids_d, T, V, uq, iv, torch.zeros_like(err_d), err_d, plan)
    return plan


def _whole_output_check(w, tabs_d, ids, lis, out, what):
    """out [L, T, d] storage array against the oracle, every layer, every token."""
    for l in range(w.L):
        rows, inv = gathered_rows(tabs_d[l], ids)
        ref, _, _, err = oracle.lookup_forward(rows, inv, lis[l]["h"], lis[l]["W_r"], lis[l]["shared"])
        assert err == 0
        assert_close(wl.storage_to_f64(out[l], w.dtype), ref, w.dtype, f"{what} layer {l}")


@pytest.mark.parametrize("name,mode", [
    ("prefill410m", "plain"), ("prefill410m", "plan"), ("prefill410m", "plan+runs"),
    ("prefill410m", "plain, streaming kernel"), ("prefill410m", "plan, streaming kernel"),
    ("prefill410m_uniform", "plain"), ("prefill410m_uniform", "plan"),
    ("decode1b_4e", "plain"), ("decode1b_4e", "plan"), ("decode410m_n2", "plain"), ("decode410m_n4", "plan"),
    ("decode410m_n8", "plain")])
def test_full_size_single_layer(tuning, name, mode):
    """One layer of the benchmark shapes through the single-layer entry point: all T tokens (16384 for the
    prefills, whose 3.3 GB table puts row offsets beyond 32 bits) against the oracle.  The prefills take the
    tile kernel by default; the streaming kernel is forced for two more cases."""
    torch = torch_mod()
    if "streaming" in mode:
        tuning("MOLE_FWD_TILE", "2")
    w = wl.scaled(wl.CONFIGS[name], L=1)
    tab_d = wl.device_table(w, 0, "cuda")
    if name.startswith("prefill"):
        assert tab_d.numel() * 2 > 2 ** 31                           # byte offsets beyond 32 bits
    ids, li = wl.token_ids(w), wl.layer_inputs(w)
    got = run_forward(w, None, ids, li, dedup=mode.startswith("plan"), runs=mode == "plan+runs", table_dev=tab_d, want_dbg=True)
    np.testing.assert_array_equal(got["rows"], ids)
    assert got["err"] == 0
    _whole_output_check(w, tab_d[None], ids, [li], got["out"][None], f"{name} ({mode})")
    ref_g = oracle.gates(li["h"], li["W_r"])
    assert_close(got["gates"].astype(np.float64), ref_g, wl.BF16, f"{name} gates")


@pytest.fixture(scope="module")
def tables_410m():
    """The 24 tables of the 410M decode configuration (39.6 GB), generated once for the tests below."""
    torch = torch_mod()
    w = wl.CONFIGS["decode410m"]
    tabs = torch.empty((w.L, w.V, w.N, w.d), dtype=torch.bfloat16, device="cuda")
    for l in range(w.L):
        wl.device_table(w, l, "cuda", out=tabs[l])
    yield tabs
    del tabs
    torch.cuda.empty_cache()


def _layers_step(w, tabs, ids, lis, plan_mode):
    """One launch of the layer-batched entry point as bench.py issues it; returns out [L, T, d] on the host."""
    torch = torch_mod()
    lis_d = {k: to_dev(np.stack([li[k] for li in lis]), w.dtype) for k in ("h", "W_r", "shared")}
    ids_d = torch.from_numpy(ids).cuda()
    out_d = torch.full_like(lis_d["h"], float("nan"))
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    flags, plan = 0, None
    if plan_mode:
        plan = _plan_for(torch, ids_d, w.T, w.V, err_d)
        flags = mb.MOLE_FLAG_DEDUP
    mb.mole_lookup_forward_layers(tabs, w.V * w.N * w.d, ids_d, None, lis_d["h"], lis_d["W_r"], lis_d["shared"],
                                  None, out_d, w.T * w.d, None, None, err_d, w.L, w.T, w.V, w.d, w.N,
                                  DT[w.dtype], flags, plan)
    torch.cuda.synchronize()
    assert int(err_d.item()) == 0
    return to_host(out_d, w.dtype)


@pytest.mark.parametrize("T", [1, 32, 256])
@pytest.mark.parametrize("plan_mode", [False, True])
def test_full_size_decode410m_all_layers(tables_410m, T, plan_mode):
    """24 layers x T tokens in one launch over the 39.6 GB table set, for the three batch sizes of the decode
    configuration (each takes another dispatch: chunk items in wide workgroups at T = 1 and 32, whole tokens
    at 256): every output element of every layer against the oracle."""
    w = wl.scaled(wl.CONFIGS["decode410m"], T=T, name=f"decode410m T={T}")
    ids = wl.token_ids(w)
    lis = [wl.layer_inputs(w, l) for l in range(w.L)]
    out = _layers_step(w, tables_410m, ids, lis, plan_mode)
    _whole_output_check(w, tables_410m, ids, lis, out, f"{w.name} plan={plan_mode}")


@pytest.mark.parametrize("plan_mode", [False, True])
def test_full_size_decode160m_all_layers(plan_mode):
    """The 160M decode step as bench.py launches it: 12 layers x 64 tokens, d = 768 (1.5 chunks), one launch."""
    torch = torch_mod()
    w = wl.CONFIGS["decode160m"]
    tabs = torch.empty((w.L, w.V, w.N, w.d), dtype=torch.bfloat16, device="cuda")
    for l in range(w.L):
        wl.device_table(w, l, "cuda", out=tabs[l])
    ids = wl.token_ids(w)
    lis = [wl.layer_inputs(w, l) for l in range(w.L)]
    out = _layers_step(w, tabs, ids, lis, plan_mode)
    _whole_output_check(w, tabs, ids, lis, out, f"decode160m plan={plan_mode}")


@pytest.mark.parametrize("N,L,T", [(16, 8, 3000), (16, 24, 512), (16, 24, 200), (8, 8, 3333), (16, 1, 1300), (16, 4, 300)])
@pytest.mark.parametrize("plan_mode", [False, True])
def test_oversubscribed_grids(N, L, T, plan_mode):
    """Launch shapes at 8 and 16 experts whose grid is not the all-resident one (at most four tokens per wave, a
    finer grid where resident places would stay empty, whole tokens instead of chunks from 1024 tokens on) and, with
    the plan, the all-resident grid on the same shapes: every output element of every layer against the oracle."""
    torch = torch_mod()
    w = wl.scaled(wl.CONFIGS["decode410m"], V=1500, N=N, L=L, T=T, seed=300 + T, name=f"grid N{N} L{L} T{T}")
    tabs = torch.stack([to_dev(wl.random_table(w, l), w.dtype) for l in range(w.L)])
    ids = wl.token_ids(w)
    lis = [wl.layer_inputs(w, l) for l in range(w.L)]
    out = _layers_step(w, tabs, ids, lis, plan_mode)
    _whole_output_check(w, tabs, ids, lis, out, f"{w.name} plan={plan_mode}")
