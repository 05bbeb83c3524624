"""GPU parity of mole_dedup_forward (dedup and forward as one call; for large batches at N = 32 the dedup runs
beside the router inside one launch and a gather kernel follows) through the C ABI: distinct ids, inverse map
and count bit-exact against the oracle's dedup, the plan left in the workspace checked for validity, the output
against the fp64 oracle at the forward's tolerance and, bit for bit, against the two separate calls."""
import numpy as np
import pytest

import oracle
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl
from helpers import DT, assert_close, to_dev, to_host
from test_gpu_dedup import check_plan

pytestmark = pytest.mark.gpu
EPS = 1e-5


def run_fused(w, table, ids, li, ni, norm, residual, shared=True):
    import torch
    T = len(ids)
    tab_d = to_dev(table, w.dtype)
    ids_d = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).cuda()
    h_d = to_dev(ni["x"] if norm else li["h"], w.dtype)
    lw_d = to_dev(ni["ln_w"], w.dtype) if norm else None
    wr_d = to_dev(li["W_r"], w.dtype)
    sh_d = to_dev(li["shared"], w.dtype) if shared else None
    rs_d = to_dev(li["residual"], w.dtype) if residual else None
    out_d = torch.full((T, w.d), float("nan"), dtype=h_d.dtype, device="cuda")
    uq = torch.full((T,), -5, dtype=torch.int32, device="cuda")
    iv = torch.full((T,), -5, dtype=torch.int32, device="cuda")
    nu = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    ws = torch.zeros((mb.mole_dedup_forward_workspace(T, w.V, w.N, 1) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_forward(tab_d, 0, ids_d, h_d, lw_d, EPS, wr_d, sh_d, rs_d, out_d, 0, uq, iv, nu, err_d, 1, T, w.V, w.d,
                          w.N, DT[w.dtype], ws)
    torch.cuda.synchronize()
    U = int(nu.item())
    # the plan in the front of the workspace serves a further planned call on the same ids
    out2_d = torch.full_like(out_d, float("nan"))
    err2_d = torch.zeros_like(err_d)
    nplan = mb.mole_dedup_workspace(T, w.V) // 4
    if norm:
        mb.mole_layer_forward(tab_d, 0, ids_d, None, h_d, lw_d, EPS, wr_d, sh_d, out2_d, 0, None, None, err2_d, 1, T, w.V,
                              w.d, w.N, DT[w.dtype], mb.MOLE_FLAG_DEDUP, ws[:nplan])
    else:
        mb.mole_lookup_forward(tab_d, ids_d, None, h_d, wr_d, sh_d, rs_d, out2_d, None, None, err2_d, T, w.V, w.d, w.N,
                               DT[w.dtype], mb.MOLE_FLAG_DEDUP, ws[:nplan])
    torch.cuda.synchronize()
    assert int(err2_d.item()) & 2 == 0                      # the plan was accepted
    return dict(out=to_host(out_d, w.dtype), out_again=to_host(out2_d, w.dtype), uniq=uq.cpu().numpy()[:U],
                inv=iv.cpu().numpy(), U=U, err=int(err_d.item()), plan=ws.cpu().numpy()[:nplan])


def check(w, table, ids, norm, residual, tuning, shared=True):
    li, ni = wl.layer_inputs(w), wl.norm_inputs(w)
    li["W_r"] = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)      # gates away from 1 / N
    got = run_fused(w, table, ids, li, ni, norm, residual, shared)
    r_uniq, r_inv, r_U, r_err = oracle.dedup(ids, w.V)
    assert got["U"] == r_U and got["err"] == r_err
    np.testing.assert_array_equal(got["uniq"], r_uniq)
    np.testing.assert_array_equal(got["inv"], r_inv)
    check_plan(got["plan"], ids, w.V, got["uniq"], got["U"])
    sh = li["shared"] if shared else None
    if norm:
        ref = oracle.layer_forward(table, ids, ni["x"], ni["ln_w"], EPS, li["W_r"], sh)[0]
    else:
        ref = oracle.lookup_forward(table, ids, li["h"], li["W_r"], sh, li["residual"] if residual else None)[0]
    assert_close(wl.storage_to_f64(got["out"], w.dtype), ref, w.dtype, f"{w.name} against the oracle")
    np.testing.assert_array_equal(got["out_again"], got["out"])       # a planned call on the plan it left behind
    # the two calls one after the other (the fused launch switched off): the same bits
    tuning("MOLE_FWD_TILE", 2)
    two = run_fused(w, table, ids, li, ni, norm, residual, shared)
    tuning("MOLE_FWD_TILE", 0)
    np.testing.assert_array_equal(two["uniq"], got["uniq"])
    np.testing.assert_array_equal(two["inv"], got["inv"])
    if w.N == 32 and len(ids) * 1 >= 4096:
        # with the tile kernel as the two-call path the gates, and so the outputs, are the same bit for bit
        two_tile = run_fused_two_calls(w, table, ids, li, ni, norm, residual, shared)
        np.testing.assert_array_equal(two_tile, got["out"])
    assert_close(wl.storage_to_f64(two["out"], w.dtype), ref, w.dtype, f"{w.name}, two calls, against the oracle")


def run_fused_two_calls(w, table, ids, li, ni, norm, residual, shared):
    """mole_dedup_ids, then the planned forward (the library's own choice of kernel): the output."""
    import torch
    T = len(ids)
    tab_d = to_dev(table, w.dtype)
    ids_d = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).cuda()
    h_d = to_dev(ni["x"] if norm else li["h"], w.dtype)
    lw_d = to_dev(ni["ln_w"], w.dtype) if norm else None
    wr_d = to_dev(li["W_r"], w.dtype)
    sh_d = to_dev(li["shared"], w.dtype) if shared else None
    rs_d = to_dev(li["residual"], w.dtype) if residual else None
    out_d = torch.full((T, w.d), float("nan"), dtype=h_d.dtype, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(T, w.V) // 4,), dtype=torch.int32, device="cuda")
    uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
    mb.mole_dedup_ids(ids_d, T, w.V, uq, iv, torch.zeros_like(err_d), err_d, plan)
    if norm:
        mb.mole_layer_forward(tab_d, 0, ids_d, None, h_d, lw_d, EPS, wr_d, sh_d, out_d, 0, None, None, err_d, 1, T, w.V,
                              w.d, w.N, DT[w.dtype], mb.MOLE_FLAG_DEDUP, plan)
    else:
        mb.mole_lookup_forward(tab_d, ids_d, None, h_d, wr_d, sh_d, rs_d, out_d, None, None, err_d, T, w.V, w.d, w.N,
                               DT[w.dtype], mb.MOLE_FLAG_DEDUP, plan)
    torch.cuda.synchronize()
    return to_host(out_d, w.dtype)


@pytest.mark.parametrize("d,N,V,T,dist,norm,residual,bad", [
    (1024, 32, 3000, 16384, "zipf", False, False, True),      # the fused launch, 16 tokens per dedup thread
    (1024, 32, 50304, 8192, "uniform", False, True, False),   # 8 per thread, few repeats, a residual
    (1024, 32, 2000, 5000, "zipf", True, False, True),        # ragged last tile, the norm inside
    (520, 32, 700, 4100, "zipf", False, False, False),        # ragged second chunk, just above the threshold
    (1536, 32, 800, 4500, "zipf", False, False, False),       # router weight too large for its transposed LDS copy
    (1024, 32, 3000, 4096, "zipf", False, False, False),      # at the threshold: the two calls
    (1024, 16, 4096, 6000, "zipf", False, True, True),        # N = 16: the two calls
    (768, 16, 2000, 333, "zipf", True, False, False),         # small batch, norm
    (64, 4, 1024, 256, "uniform", False, False, True),        # fp32
])
def test_dedup_forward_matches_oracle_and_the_two_calls(tuning, d, N, V, T, dist, norm, residual, bad):
    cfg = "tiny" if d == 64 else "decode410m"
    w = wl.scaled(wl.CONFIGS[cfg], V=V, d=d, N=N, T=T, L=1, ids=dist, seed=77 + T, name=f"dedup_forward d{d} N{N} T{T}")
    table, ids = wl.random_table(w), wl.token_ids(w).copy()
    if bad:
        ids[T // 3] = V + 5                                  # an id outside the table: flagged, routed term 0
        ids[T - 1] = -2
    check(w, table, ids, norm, residual, tuning)


def test_without_shared_output_and_every_id_equal(tuning):
    """No shared term (the routed term alone must meet the tolerance), and a batch with one distinct id."""
    w = wl.scaled(wl.CONFIGS["decode410m"], V=512, d=1024, N=32, T=4500, L=1, seed=5, name="dedup_forward one id")
    table = wl.random_table(w)
    check(w, table, np.full((w.T,), 77, dtype=np.int32), False, False, tuning, shared=False)


def test_full_size_prefill(tuning):
    """The prefill configuration as bench.py launches it (16384 tokens, N = 32, 3.3 GB table on the device): whole
    output against the oracle on the rows copied back by plain indexing."""
    import torch
    from helpers import gathered_rows
    w = wl.CONFIGS["prefill410m"]
    tab_d = torch.empty((w.V, w.N, w.d), dtype=torch.bfloat16, device="cuda")
    wl.device_table(w, 0, "cuda", out=tab_d)
    ids = wl.token_ids(w)
    li = wl.layer_inputs(w)
    T = w.T
    ids_d = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).cuda()
    h_d, wr_d, sh_d = (to_dev(li[k], w.dtype) for k in ("h", "W_r", "shared"))
    out_d = torch.full((T, w.d), float("nan"), dtype=h_d.dtype, device="cuda")
    uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    ws = torch.empty((mb.mole_dedup_forward_workspace(T, w.V, w.N, 1) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_forward(tab_d, 0, ids_d, h_d, None, 0.0, wr_d, sh_d, None, out_d, 0, uq, iv, nu, err_d, 1, T, w.V, w.d,
                          w.N, DT[w.dtype], ws)
    torch.cuda.synchronize()
    r_uniq, r_inv, r_U, r_err = oracle.dedup(ids, w.V)
    assert int(nu.item()) == r_U and int(err_d.item()) == 0
    np.testing.assert_array_equal(uq.cpu().numpy()[:r_U], r_uniq)
    np.testing.assert_array_equal(iv.cpu().numpy(), r_inv)
    rows, inv = gathered_rows(tab_d, ids)
    ref = oracle.lookup_forward(rows, inv, li["h"], li["W_r"], li["shared"], None)[0]
    assert_close(wl.storage_to_f64(to_host(out_d, w.dtype), w.dtype), ref, w.dtype, "prefill410m, dedup + forward")


def test_host_errors():
    import torch
    a = torch.zeros((4096,), dtype=torch.int32, device="cuda")
    need = mb.mole_dedup_forward_workspace(100, 1000, 32, 1)
    assert need == (mb.mole_dedup_workspace(100, 1000) + 15) // 16 * 16 + 100 * 32 * 4
    with pytest.raises(mb.MoleError) as e:
        mb.mole_dedup_forward(a, 0, a, a, None, 0.0, a, None, None, a, 0, a, a, a, None, 1, 100, 1000, 64, 32, mb.MOLE_BF16,
                              a, workspace_bytes=need - 4)
    assert e.value.status == mb.MOLE_EWORKSPACE
    with pytest.raises(mb.MoleError) as e:
        mb.mole_dedup_forward(a, 0, a, a, a, 1e-5, a, None, a, a, 0, a, a, a, None, 1, 100, 1000, 64, 32, mb.MOLE_BF16, a)
    assert e.value.status == mb.MOLE_EINVAL and "residual" in e.value.message


def test_hip_graph_replay_of_a_two_layer_step():
    """A model's use of the call, captured in a HIP graph: layer 0 through mole_dedup_forward (the fused launches),
    layer 1 through the planned forward on the plan that call left in its workspace.  Every replay, with new ids and
    eager work in between, must give the bits of the eager two-call path."""
    import torch
    w = wl.scaled(wl.CONFIGS["decode410m"], V=2000, d=1024, N=32, T=5000, L=2, seed=9)
    tabs = [to_dev(wl.random_table(w, l), w.dtype) for l in range(w.L)]
    lis = [wl.layer_inputs(w, l) for l in range(w.L)]
    hs, wrs, shs = ([to_dev(li[k], w.dtype) for li in lis] for k in ("h", "W_r", "shared"))
    ids_d = torch.from_numpy(wl.token_ids(w)).cuda()
    uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    ws = torch.empty((mb.mole_dedup_forward_workspace(w.T, w.V, w.N, 1) // 4,), dtype=torch.int32, device="cuda")
    nplan = mb.mole_dedup_workspace(w.T, w.V) // 4
    outs = [torch.zeros_like(h) for h in hs]
    s = torch.cuda.Stream()

    def step(dst):
        mb.mole_dedup_forward(tabs[0], 0, ids_d, hs[0], None, 0.0, wrs[0], shs[0], None, dst[0], 0, uq, iv, nu, err, 1,
                              w.T, w.V, w.d, w.N, DT[w.dtype], ws, stream=s)
        mb.mole_lookup_forward(tabs[1], ids_d, None, hs[1], wrs[1], shs[1], None, dst[1], None, None, err, w.T, w.V, w.d,
                               w.N, DT[w.dtype], mb.MOLE_FLAG_DEDUP, ws[:nplan], stream=s)

    with torch.cuda.stream(s):
        step(outs)
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            step(outs)
    plan2 = torch.empty((nplan,), dtype=torch.int32, device="cuda")
    for rep in range(4):
        for o in outs:
            o.zero_()
        ids_d.copy_(torch.from_numpy(wl.token_ids(w, batch=rep)).cuda())
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        U = int(nu.item())
        r_uniq, r_inv, r_U, _ = oracle.dedup(ids_d.cpu().numpy(), w.V)
        assert U == r_U
        np.testing.assert_array_equal(uq.cpu().numpy()[:U], r_uniq)
        np.testing.assert_array_equal(iv.cpu().numpy(), r_inv)
        refs = [torch.zeros_like(o) for o in outs]
        with torch.cuda.stream(s):
            mb.mole_dedup_ids(ids_d, w.T, w.V, torch.empty_like(uq), torch.empty_like(iv), torch.zeros_like(nu), err,
                              plan2, stream=s)
            for l in range(w.L):
                mb.mole_lookup_forward(tabs[l], ids_d, None, hs[l], wrs[l], shs[l], None, refs[l], None, None, err, w.T,
                                       w.V, w.d, w.N, DT[w.dtype], mb.MOLE_FLAG_DEDUP, plan2, stream=s)
        s.synchronize()
        for l in range(w.L):
            assert torch.equal(outs[l].view(torch.int16), refs[l].view(torch.int16)), f"replay {rep}, layer {l}"
    assert int(err.item()) == 0
