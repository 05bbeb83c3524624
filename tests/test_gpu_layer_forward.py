"""GPU parity of mole_layer_forward (post-attention RMSNorm and residual inside the lookup kernel) against the
fp64 oracle of the inference listing, at the plain tolerance.  Through the C ABI; seeded synthetic inputs."""
import numpy as np
import pytest

import oracle
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl
from helpers import DT, assert_close, gathered_rows, to_dev, to_host

pytestmark = pytest.mark.gpu
EPS = 1e-5


def inputs(w, layer=0, router_scale=5.0):
    li, ni = wl.layer_inputs(w, layer), wl.norm_inputs(w, layer)
    W_r = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * router_scale, w.dtype)   # gates away from 1/N
    return dict(x=ni["x"], ln_w=ni["ln_w"], W_r=W_r, shared=li["shared"])


def run(w, table, ids, inp, shared=True, dedup=False, eps=EPS, want_dbg=True):
    import torch
    T = len(ids)
    tab_d = to_dev(table, w.dtype)
    ids_d = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).cuda()
    x_d, lw_d, wr_d = (to_dev(inp[k], w.dtype) for k in ("x", "ln_w", "W_r"))
    sh_d = to_dev(inp["shared"], w.dtype) if shared else None
    out_d = torch.full((T, w.d), float("nan"), dtype=x_d.dtype, device="cuda")
    gates_d = torch.full((T, w.N), -1.0, dtype=torch.float32, device="cuda") if want_dbg else None
    rows_d = torch.full((T,), -7, dtype=torch.int64, device="cuda") if want_dbg else None
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    flags, plan = 0, None
    if dedup:
        plan = torch.empty((mb.mole_dedup_workspace(T, w.V) // 4,), dtype=torch.int32, device="cuda")
        uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
        nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
        mb.mole_dedup_ids(ids_d, T, w.V, uq, iv, nu, err_d, plan)
        flags = mb.MOLE_FLAG_DEDUP
    mb.mole_layer_forward(tab_d, 0, ids_d, None, x_d, lw_d, eps, wr_d, sh_d, out_d, 0, gates_d, rows_d, err_d,
                          1, T, w.V, w.d, w.N, DT[w.dtype], flags, plan)
    torch.cuda.synchronize()
    if not want_dbg:
        return dict(out=to_host(out_d, w.dtype), err=int(err_d.item()))
    return dict(out=to_host(out_d, w.dtype), gates=gates_d.cpu().numpy(), rows=rows_d.cpu().numpy(),
                err=int(err_d.item()))


def check(w, table, ids, inp, shared=True, dedup=False, eps=EPS):
    """Output, gates, rows and error flag against the layer as the listing has it: the oracle applies the
    norm weight to the state in fp64 and feeds router and adds from there."""
    sh = inp["shared"] if shared else None
    ref_out, ref_g, _, ref_rows, ref_err = oracle.layer_forward(table, ids, inp["x"], inp["ln_w"], eps, inp["W_r"], sh)
    got = run(w, table, ids, inp, shared=shared, dedup=dedup, eps=eps)
    np.testing.assert_array_equal(got["rows"], ref_rows)
    assert got["err"] == ref_err
    assert_close(got["gates"].astype(np.float64), ref_g, w.dtype, f"gates ({w.name})")
    assert_close(wl.storage_to_f64(got["out"], w.dtype), ref_out, w.dtype, f"out ({w.name})")
    # the kernels that write no debug outputs are variants of their own (same arithmetic): the same bits
    plain = run(w, table, ids, inp, shared=shared, dedup=dedup, eps=eps, want_dbg=False)
    np.testing.assert_array_equal(plain["out"], got["out"])


@pytest.mark.parametrize("d,N,T,V", [
    (1024, 16, 333, 4096),     # 410M-shaped rows
    (768, 16, 64, 4096),       # 160M-shaped: 1.5 chunks
    (1024, 32, 203, 2048),     # prefill-shaped N
    (2048, 4, 77, 1024),       # 1B-shaped: four chunks, the residual of chunks 2 and 3 is read again
    (1544, 8, 50, 300),        # ragged third chunk
    (256, 8, 130, 512),
    (128, 64, 50, 300),
    (1024, 64, 40, 100),       # N = 64: two halves of experts per chunk
    (520, 16, 9, 64),          # a chunk with a single active lane
    (64, 1, 40, 100),          # generic kernel
    (1024, 5, 33, 256),        # generic kernel, N not a power of two
    (1024, 2, 45, 256),        # the smallest expert count of the ablation (router padded to four)
])
@pytest.mark.parametrize("dedup", [False, True])
def test_bf16_shapes(d, N, T, V, dedup):
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"norm bf16 d{d} N{N} T{T}")
    check(w, wl.random_table(w), wl.token_ids(w), inputs(w), dedup=dedup)


@pytest.mark.parametrize("split", ["1", "2"])
@pytest.mark.parametrize("wpb", ["4", "8"])
@pytest.mark.parametrize("nta", ["1", "2"])
@pytest.mark.parametrize("d,N,T,V", [(1024, 16, 333, 4096), (1544, 8, 50, 300), (1024, 32, 203, 2048)])
def test_launch_variants(tuning, split, wpb, nta, d, N, T, V):
    """Item granularity, workgroup width and load kind all change which registers hold the residual."""
    tuning("MOLE_FWD_SPLIT", split)
    tuning("MOLE_FWD_WPB", wpb)
    tuning("MOLE_FWD_NTA", nta)
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"norm split{split} wpb{wpb} nta{nta}")
    ids = wl.token_ids(w).copy()
    ids[T // 3] = -2                                       # an id outside the table: x + shared only, flagged
    inp = inputs(w)
    check(w, wl.random_table(w), ids, inp, dedup=False)
    check(w, wl.random_table(w), ids, inp, dedup=True, shared=False)


@pytest.mark.parametrize("d,N,T,V", [(1024, 32, 203, 64), (1024, 16, 333, 4096), (1544, 8, 50, 30), (520, 4, 37, 16),
                                     (1024, 2, 45, 20)])
def test_run_kernel(tuning, d, N, T, V):
    """The kernel that large planned batches take, forced on small shapes: the residual is the state
    itself, re-read per chunk."""
    tuning("MOLE_FWD_RUN", "1")
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"norm run d{d} N{N} T{T}")
    ids = wl.token_ids(w).copy()
    ids[T // 3] = -2
    inp = inputs(w)
    check(w, wl.random_table(w), ids, inp, dedup=True)
    check(w, wl.random_table(w), ids, inp, dedup=True, shared=False)


@pytest.mark.parametrize("d,T,V", [(1024, 203, 64), (1024, 1, 4), (520, 37, 16), (2048, 70, 500), (72, 33, 9)])
def test_tile_kernel(tuning, d, T, V):
    """The tile kernel with the norm inside (state times norm weight as a bf16 hi + lo pair on the matrix pipe,
    1 / rms on the logits), forced on small shapes."""
    tuning("MOLE_FWD_TILE", "1")
    w = wl.scaled(wl.CONFIGS["prefill410m"], V=V, d=d, N=32, T=T, L=1, name=f"norm tile d{d} T{T}")
    ids = wl.token_ids(w).copy()
    if T > 2:
        ids[T // 3] = -2
    inp = inputs(w)
    for dedup in (False, True):
        check(w, wl.random_table(w), ids, inp, dedup=dedup)
        check(w, wl.random_table(w), ids, inp, dedup=dedup, shared=False)


@pytest.mark.parametrize("seed", range(12))
def test_seeded_random_shapes(tuning, seed):
    """Shapes and launch switches drawn from the documented ranges: every dispatch path of the fused-norm
    call against the oracle."""
    rng = np.random.default_rng(2000 + seed)
    d = int(rng.integers(1, 289)) * 8
    N = int(rng.choice([1, 2, 3, 4, 8, 12, 16, 32, 40, 64]))
    T = int(rng.integers(1, 90))
    V = int(rng.integers(max(2, T // 8), 400))
    for var in ("MOLE_FWD_SPLIT", "MOLE_FWD_NTA", "MOLE_FWD_RUN", "MOLE_FWD_TILE"):
        tuning(var, str(int(rng.integers(1, 3))))
    tuning("MOLE_FWD_WPB", str(int(rng.choice([4, 8]))))
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, ids=str(rng.choice(["zipf", "uniform"])),
                  name=f"norm random seed {seed}: d{d} N{N} T{T} V{V}")
    ids = wl.token_ids(w).copy()
    if rng.integers(2) and T > 2:
        ids[int(rng.integers(T))] = -1
    check(w, wl.random_table(w), ids, inputs(w), shared=bool(rng.integers(2)), dedup=bool(rng.integers(2)))


@pytest.mark.parametrize("d,N,T", [(64, 4, 256), (128, 16, 100), (32, 3, 17)])
def test_fp32_shapes(d, N, T):
    w = wl.scaled(wl.CONFIGS["tiny"], V=777, d=d, N=N, T=T, name=f"norm fp32 d{d} N{N}")
    check(w, wl.random_table(w), wl.token_ids(w), inputs(w))
    check(w, wl.random_table(w), wl.token_ids(w), inputs(w), eps=0.0, dedup=True)


def test_layers_in_one_launch_match_single_layer_calls():
    import torch
    L, V, d, N, T = 3, 900, 1024, 16, 70
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=L, name="norm layers")
    tabs = np.stack([wl.random_table(w, l) for l in range(L)])
    inps = [inputs(w, l) for l in range(L)]
    ids = wl.token_ids(w)
    stack = lambda k: to_dev(np.stack([i[k] for i in inps]), w.dtype)
    x_d, lw_d, wr_d, sh_d = stack("x"), stack("ln_w"), stack("W_r"), stack("shared")
    tab_d = to_dev(tabs, w.dtype)
    ids_d = torch.from_numpy(ids).cuda()
    out_d = torch.zeros_like(x_d)
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    mb.mole_layer_forward(tab_d, V * N * d, ids_d, None, x_d, lw_d, EPS, wr_d, sh_d, out_d, T * d, None, None, err_d,
                          L, T, V, d, N, DT[w.dtype])
    torch.cuda.synchronize()
    out = to_host(out_d, w.dtype)
    for l in range(L):
        ref, *_ = oracle.layer_forward(tabs[l], ids, inps[l]["x"], inps[l]["ln_w"], EPS, inps[l]["W_r"],
                                       inps[l]["shared"])
        assert_close(wl.storage_to_f64(out[l], w.dtype), ref, w.dtype, f"layer {l}")
        single = run(w, tabs[l], ids, inps[l])
        np.testing.assert_array_equal(single["out"], out[l])


def test_equals_unfused_path_fed_with_a_rounded_norm():
    """Cross-check inside the library: the fused call against mole_lookup_forward given the normed state
    (computed here in fp64 and rounded to bf16) and the residual.  They differ by bf16 roundings only."""
    import torch
    w = wl.scaled(wl.CONFIGS["decode410m"], V=2000, T=128, L=1, name="norm vs unfused")
    table, ids, inp = wl.random_table(w), wl.token_ids(w), inputs(w)
    fused = run(w, table, ids, inp)
    x = wl.storage_to_f64(inp["x"], w.dtype)
    hn = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + EPS) * wl.storage_to_f64(inp["ln_w"], w.dtype)
    out_d = torch.zeros((w.T, w.d), dtype=torch.bfloat16, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    mb.mole_lookup_forward(to_dev(table, w.dtype), torch.from_numpy(ids).cuda(), None,
                           to_dev(wl.to_storage(hn, w.dtype), w.dtype), to_dev(inp["W_r"], w.dtype),
                           to_dev(inp["shared"], w.dtype), to_dev(inp["x"], w.dtype), out_d, None, None, err_d,
                           w.T, w.V, w.d, w.N, DT[w.dtype])
    torch.cuda.synchronize()
    assert_close(wl.storage_to_f64(fused["out"], w.dtype), wl.storage_to_f64(to_host(out_d, w.dtype), w.dtype),
                 w.dtype, "fused vs unfused")


@pytest.mark.parametrize("name,dedup", [("prefill410m_uniform", False), ("prefill410m", True), ("decode1b_4e", False),
                                        ("decode410m", False)])
def test_full_size_single_layer(name, dedup):
    """Benchmark sizes in the benchmark's launch configuration: the whole output (all T tokens) and the
    gates against the oracle; the rows the batch looks up are copied back with plain indexing."""
    import torch
    w = wl.scaled(wl.CONFIGS[name], L=1)
    tab_d = wl.device_table(w, 0, "cuda")
    ids, inp = wl.token_ids(w), inputs(w)
    ids_d = torch.from_numpy(ids).cuda()
    x_d, lw_d, wr_d, sh_d = (to_dev(inp[k], w.dtype) for k in ("x", "ln_w", "W_r", "shared"))
    out_d = torch.full_like(x_d, float("nan"))
    gates_d = torch.zeros((w.T, w.N), dtype=torch.float32, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    flags, plan = 0, None
    if dedup:
        plan = torch.empty((mb.mole_dedup_workspace(w.T, w.V) // 4,), dtype=torch.int32, device="cuda")
        uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
        mb.mole_dedup_ids(ids_d, w.T, w.V, uq, iv, torch.zeros_like(err_d), err_d, plan)
        flags = mb.MOLE_FLAG_DEDUP
    mb.mole_layer_forward(tab_d, 0, ids_d, None, x_d, lw_d, EPS, wr_d, sh_d, out_d, 0, gates_d, None, err_d, 1, w.T,
                          w.V, w.d, w.N, DT[w.dtype], flags, plan)
    torch.cuda.synchronize()
    assert int(err_d.item()) == 0
    rows, inv = gathered_rows(tab_d, ids)
    ref, ref_g, *_ = oracle.layer_forward(rows, inv, inp["x"], inp["ln_w"], EPS, inp["W_r"], inp["shared"])
    assert_close(gates_d.cpu().numpy().astype(np.float64), ref_g, w.dtype, f"{name} fused-norm gates")
    assert_close(wl.storage_to_f64(to_host(out_d, w.dtype), w.dtype), ref, w.dtype, f"{name} fused-norm output")
