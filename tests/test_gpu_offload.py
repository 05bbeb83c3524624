"""GPU parity of the offloaded-LUT mode: rows fetched from pinned host memory are byte-identical to the
host rows, and the staged forward equals the resident forward bit for bit (and the oracle within
tolerance)."""
import numpy as np
import pytest

import oracle
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl
from helpers import DT, assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("L,V,d,N,T,dtype", [(3, 3000, 1024, 16, 32, wl.BF16), (1, 500, 768, 16, 64, wl.BF16),
                                             (2, 400, 64, 4, 50, wl.F32), (2, 300, 520, 5, 9, wl.BF16)])
def test_fetch_then_forward(L, V, d, N, T, dtype):
    import torch
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, N=N, T=T, L=L, dtype=dtype)
    tabs = np.stack([wl.random_table(w, l) for l in range(L)])                     # [L,V,N,d] storage
    host_t = to_dev(tabs, dtype, device="cpu").pin_memory()
    ids = wl.token_ids(w)
    lis = [wl.layer_inputs(w, l) for l in range(L)]
    ids_d = torch.from_numpy(ids).cuda()
    uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, T, V, uniq_d, inv_d, nu_d, err_d, plan)
    U_cap = T
    staging = torch.zeros((L, U_cap, N, d), dtype=host_t.dtype, device="cuda")
    mb.mole_offload_fetch(host_t, V * N * d, uniq_d, nu_d, staging, U_cap * N * d, err_d, L, U_cap, V, d, N, DT[dtype])
    torch.cuda.synchronize()
    U = int(nu_d.item())
    r_uniq, r_inv, r_U, _ = oracle.dedup(ids, V)
    assert U == r_U
    st = to_host(staging, dtype)
    np.testing.assert_array_equal(st[:, :U], tabs[:, r_uniq])                      # byte-identical rows
    assert (st[:, U:] == 0).all()                                                  # nothing else touched

    stack = lambda key: to_dev(np.stack([li[key] for li in lis]), dtype)
    h_d, wr_d, sh_d = stack("h"), stack("W_r"), stack("shared")
    out_staged, out_res = torch.zeros_like(h_d), torch.zeros_like(h_d)
    tab_d = to_dev(tabs, dtype)
    for flags, pl in ((0, None), (mb.MOLE_FLAG_DEDUP, plan)):
        mb.mole_lookup_forward_layers(staging, U_cap * N * d, ids_d, inv_d, h_d, wr_d, sh_d, None, out_staged,
                                      T * d, None, None, err_d, L, T, U_cap, d, N, DT[dtype], flags, pl)
        mb.mole_lookup_forward_layers(tab_d, V * N * d, ids_d, None, h_d, wr_d, sh_d, None, out_res, T * d,
                                      None, None, err_d, L, T, V, d, N, DT[dtype], flags, pl)
        torch.cuda.synchronize()
        assert int(err_d.item()) == 0
        a, b = to_host(out_staged, dtype), to_host(out_res, dtype)
        np.testing.assert_array_equal(a, b)
        for l in range(L):
            ref, _, _, _ = oracle.lookup_forward(tabs[l], ids, lis[l]["h"], lis[l]["W_r"], lis[l]["shared"])
            assert_close(wl.storage_to_f64(a[l], dtype), ref, dtype, f"staged forward layer {l}")


@pytest.mark.parametrize("layout", ["layer-major", "id-major"])
def test_full_size_offload_step_sampled(layout):
    """The benchmark's offloaded step at its real size: 24 tables of 50304 x 16 x 1024 bf16 (39.6 GB) in
    pinned host memory, 32 Zipf tokens.  Fetched rows are compared byte for byte with the host table,
    the staged forward bit for bit with the forward on the device-resident tables, and sampled tokens
    of three layers with the oracle."""
    import gc
    import torch
    w = wl.CONFIGS["offload410m"]
    L, V, N, d, T = w.L, w.V, w.N, w.d, w.T
    tabs = torch.empty((L, V, N, d), dtype=torch.bfloat16, device="cuda")
    for l in range(L):
        wl.device_table(w, l, "cuda", out=tabs[l])
    if layout == "layer-major":
        host = torch.empty((L, V, N, d), dtype=torch.bfloat16, pin_memory=True)
        host.copy_(tabs)
    else:
        host = torch.empty((V, L, N, d), dtype=torch.bfloat16, pin_memory=True)
        for l in range(L):
            host[:, l].copy_(tabs[l])
    torch.cuda.synchronize()
    ids = wl.token_ids(w)
    lis = [wl.layer_inputs(w, l) for l in range(L)]
    lis_d = {k: to_dev(np.stack([li[k] for li in lis]), w.dtype) for k in ("h", "W_r", "shared")}
    ids_d = torch.from_numpy(ids).cuda()
    uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, T, V, uniq_d, inv_d, nu_d, err_d, plan)
    U_cap = T
    staging = torch.zeros((L, U_cap, N, d), dtype=torch.bfloat16, device="cuda")
    if layout == "layer-major":
        mb.mole_offload_fetch(host, V * N * d, uniq_d, nu_d, staging, U_cap * N * d, err_d, L, U_cap, V, d, N,
                              mb.MOLE_BF16)
    else:
        mb.mole_offload_fetch_idmajor(host, uniq_d, nu_d, staging, U_cap * N * d, err_d, L, U_cap, V, d, N,
                                      mb.MOLE_BF16)
    torch.cuda.synchronize()
    U = int(nu_d.item())
    r_uniq, r_inv, r_U, _ = oracle.dedup(ids, V)
    assert U == r_U and int(err_d.item()) == 0
    uq = torch.from_numpy(r_uniq.astype(np.int64))
    want = host[:, uq] if layout == "layer-major" else host[uq].transpose(0, 1)
    assert torch.equal(staging[:, :U].cpu().view(torch.int16), want.contiguous().view(torch.int16))
    assert not staging[:, U:].any()

    out_staged, out_res = torch.zeros_like(lis_d["h"]), torch.zeros_like(lis_d["h"])
    mb.mole_lookup_forward_layers(staging, U_cap * N * d, ids_d, inv_d, lis_d["h"], lis_d["W_r"], lis_d["shared"],
                                  None, out_staged, T * d, None, None, err_d, L, T, U_cap, d, N, mb.MOLE_BF16)
    mb.mole_lookup_forward_layers(tabs, V * N * d, ids_d, None, lis_d["h"], lis_d["W_r"], lis_d["shared"], None,
                                  out_res, T * d, None, None, err_d, L, T, V, d, N, mb.MOLE_BF16)
    torch.cuda.synchronize()
    assert int(err_d.item()) == 0
    a, b = to_host(out_staged, w.dtype), to_host(out_res, w.dtype)
    np.testing.assert_array_equal(a, b)
    sample = np.arange(T)
    for layer in (0, 11, 23):
        rows_host = to_host(tabs[layer][torch.from_numpy(ids[sample].astype(np.int64)).cuda()], w.dtype)
        ref, _, _, _ = oracle.lookup_forward(rows_host, np.arange(len(sample), dtype=np.int32), lis[layer]["h"][sample],
                                             lis[layer]["W_r"], lis[layer]["shared"][sample])
        assert_close(wl.storage_to_f64(a[layer][sample], w.dtype), ref, w.dtype, f"offloaded step, layer {layer}")
    del host, want
    gc.collect()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()         # pinned requests are rounded up to a power of two and cached


def test_forward_straight_from_pinned_host_table():
    """The table pointer may itself be pinned host memory: rows then cross the link inside the forward."""
    import torch
    w = wl.scaled(wl.CONFIGS["offload410m"], V=2000, T=32, L=1)
    tab = wl.random_table(w)
    host_t = to_dev(tab, w.dtype, device="cpu").pin_memory()
    li, ids = wl.layer_inputs(w), wl.token_ids(w)
    ids_d = torch.from_numpy(ids).cuda()
    h_d, wr_d, sh_d = (to_dev(li[k], w.dtype) for k in ("h", "W_r", "shared"))
    out_d = torch.zeros_like(h_d)
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    mb.mole_lookup_forward(host_t, ids_d, None, h_d, wr_d, sh_d, None, out_d, None, None, err_d, w.T, w.V, w.d, w.N,
                           DT[w.dtype])
    torch.cuda.synchronize()
    ref, _, _, _ = oracle.lookup_forward(tab, ids, li["h"], li["W_r"], li["shared"])
    assert_close(wl.storage_to_f64(to_host(out_d, w.dtype), w.dtype), ref, w.dtype, "host-table forward")


def test_fetch_reports_overflowing_staging():
    import torch
    w = wl.scaled(wl.CONFIGS["offload410m"], V=500, d=64, N=4, T=64, L=1, ids="uniform")
    tab = wl.random_table(w)
    host_t = to_dev(tab, w.dtype, device="cpu").pin_memory()
    ids = wl.token_ids(w)
    ids_d = torch.from_numpy(ids).cuda()
    uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(w.T, w.V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, w.T, w.V, uniq_d, inv_d, nu_d, err_d, plan)
    U_cap = 8
    staging = torch.zeros((U_cap + 4, w.N, w.d), dtype=host_t.dtype, device="cuda")
    mb.mole_offload_fetch(host_t, 0, uniq_d, nu_d, staging, 0, err_d, 1, U_cap, w.V, w.d, w.N, DT[w.dtype])
    torch.cuda.synchronize()
    assert int(nu_d.item()) > U_cap and int(err_d.item()) == 1
    st = to_host(staging, w.dtype)
    uniq = uniq_d.cpu().numpy()
    np.testing.assert_array_equal(st[:U_cap], tab[uniq[:U_cap]])
    assert (st[U_cap:] == 0).all()                                                 # no write past the capacity


@pytest.mark.parametrize("L,V,d,N,T,dtype", [(3, 3000, 1024, 16, 32, wl.BF16), (24, 300, 128, 4, 40, wl.BF16),
                                             (2, 400, 64, 4, 50, wl.F32), (5, 300, 520, 5, 9, wl.BF16)])
def test_fetch_from_id_major_host_table(L, V, d, N, T, dtype):
    """[V, L, N, d] host layout: the staging buffer must hold exactly what the layer-major fetch gives
    (rows are copied, so byte-identical to a numpy gather of the source tables)."""
    import torch
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, N=N, T=T, L=L, dtype=dtype)
    tabs = np.stack([wl.random_table(w, l) for l in range(L)])                     # [L,V,N,d]
    host_t = to_dev(np.ascontiguousarray(tabs.transpose(1, 0, 2, 3)), dtype, device="cpu").pin_memory()
    ids = wl.token_ids(w)
    ids_d = torch.from_numpy(ids).cuda()
    uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, T, V, uniq_d, inv_d, nu_d, err_d, plan)
    U_cap = T + 3
    staging = torch.zeros((L, U_cap, N, d), dtype=host_t.dtype, device="cuda")
    mb.mole_offload_fetch_idmajor(host_t, uniq_d, nu_d, staging, U_cap * N * d, err_d, L, U_cap, V, d, N, DT[dtype])
    torch.cuda.synchronize()
    r_uniq, r_inv, r_U, _ = oracle.dedup(ids, V)
    assert int(nu_d.item()) == r_U and int(err_d.item()) == 0
    st = to_host(staging, dtype)
    np.testing.assert_array_equal(st[:, :r_U], tabs[:, r_uniq])
    assert (st[:, r_U:] == 0).all()

    # staged forward against the oracle on one layer
    li = wl.layer_inputs(w, L - 1)
    h_d, wr_d, sh_d = (to_dev(li[k], dtype) for k in ("h", "W_r", "shared"))
    out_d = torch.zeros_like(h_d)
    mb.mole_lookup_forward(staging[L - 1], ids_d, inv_d, h_d, wr_d, sh_d, None, out_d, None, None, err_d, T, U_cap,
                           d, N, DT[dtype])
    torch.cuda.synchronize()
    ref, _, _, _ = oracle.lookup_forward(tabs[L - 1], ids, li["h"], li["W_r"], li["shared"])
    assert_close(wl.storage_to_f64(to_host(out_d, dtype), dtype), ref, dtype, "forward from id-major fetch")


def test_id_major_fetch_reports_overflowing_staging():
    import torch
    w = wl.scaled(wl.CONFIGS["offload410m"], V=500, d=64, N=4, T=64, L=3, ids="uniform")
    tabs = np.stack([wl.random_table(w, l) for l in range(w.L)])
    host_t = to_dev(np.ascontiguousarray(tabs.transpose(1, 0, 2, 3)), w.dtype, device="cpu").pin_memory()
    ids_d = torch.from_numpy(wl.token_ids(w)).cuda()
    uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(w.T, w.V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, w.T, w.V, uniq_d, inv_d, nu_d, err_d, plan)
    U_cap = 8
    staging = torch.zeros((w.L, U_cap + 2, w.N, w.d), dtype=host_t.dtype, device="cuda")
    mb.mole_offload_fetch_idmajor(host_t, uniq_d, nu_d, staging, (U_cap + 2) * w.N * w.d, err_d, w.L, U_cap, w.V,
                                  w.d, w.N, DT[w.dtype])
    torch.cuda.synchronize()
    assert int(nu_d.item()) > U_cap and int(err_d.item()) == 1
    st = to_host(staging, w.dtype)
    uniq = uniq_d.cpu().numpy()
    np.testing.assert_array_equal(st[:, :U_cap], tabs[:, uniq[:U_cap]])
    assert (st[:, U_cap:] == 0).all()


@pytest.mark.parametrize("layout", [mb.MOLE_LAYOUT_LAYER_MAJOR, mb.MOLE_LAYOUT_ID_MAJOR])
def test_storage_tier_step(tmp_path, layout):
    """A whole step with the table in a file: dedup on the device, the distinct ids to the host, their rows
    read from the file into pinned memory, pulled to the device (identity ids), staged forward."""
    import torch
    L, V, d, N, T = 4, 2000, 256, 8, 48
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, N=N, T=T, L=L)
    dtype = w.dtype
    tabs = np.stack([wl.random_table(w, l) for l in range(L)])
    path = str(tmp_path / "lut.molelut")
    f = mb.mole_lut_file_create(path, DT[dtype], layout, L, V, N, d)
    for l in range(L):
        mb.mole_lut_file_write_layer(f, l, to_dev(tabs[l], dtype, device="cpu"), 4)
    mb.mole_lut_file_close(f)

    f, desc = mb.mole_lut_file_open(path)
    try:
        ids = wl.token_ids(w)
        ids_d = torch.from_numpy(ids).cuda()
        uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
        nu_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
        err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
        plan = torch.empty((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
        mb.mole_dedup_ids(ids_d, T, V, uniq_d, inv_d, nu_d, err_d, plan)
        U = int(nu_d.item())
        uniq_h = uniq_d[:U].cpu()
        U_cap = T
        pinned = torch.zeros((U_cap, L, N, d), dtype=torch.bfloat16).pin_memory()
        mb.mole_lut_file_read_rows(f, uniq_h, U, pinned, 4)
        staging = torch.zeros((L, U_cap, N, d), dtype=torch.bfloat16, device="cuda")
        mb.mole_offload_fetch_idmajor(pinned, None, nu_d, staging, U_cap * N * d, err_d, L, U_cap, U_cap, d, N,
                                      DT[dtype])
        lis = [wl.layer_inputs(w, l) for l in range(L)]
        stack = lambda key: to_dev(np.stack([li[key] for li in lis]), dtype)
        h_d, wr_d, sh_d = stack("h"), stack("W_r"), stack("shared")
        out_d = torch.zeros_like(h_d)
        mb.mole_lookup_forward_layers(staging, U_cap * N * d, ids_d, inv_d, h_d, wr_d, sh_d, None, out_d, T * d,
                                      None, None, err_d, L, T, U_cap, d, N, DT[dtype], mb.MOLE_FLAG_DEDUP, plan)
        torch.cuda.synchronize()
        assert int(err_d.item()) == 0
        r_uniq, _, r_U, _ = oracle.dedup(ids, V)
        assert U == r_U
        np.testing.assert_array_equal(to_host(staging, dtype)[:, :U], tabs[:, r_uniq])
        out = to_host(out_d, dtype)
        for l in range(L):
            ref, _, _, _ = oracle.lookup_forward(tabs[l], ids, lis[l]["h"], lis[l]["W_r"], lis[l]["shared"])
            assert_close(wl.storage_to_f64(out[l], dtype), ref, dtype, f"storage-tier forward layer {l}")
    finally:
        mb.mole_lut_file_close(f)
