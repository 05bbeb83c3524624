"""GPU parity of the NF4 / NF3 path: mole_quantize_lut is bit-exact against the codec oracle (codes,
packing and scales); mole_lookup_forward_nf matches the fp64 oracle forward run on the dequantised
table."""
import numpy as np
import pytest

import oracle
from oracle import nf_codec as nf
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl
from helpers import assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu


def gpu_quantize(table_bits, rows, N, d, bits, block, sb):
    import torch
    tab_d = to_dev(table_bits, wl.BF16)
    codes = torch.zeros((mb.mole_nf_codes_bytes(rows, N, d, bits),), dtype=torch.uint8, device="cuda")
    scales = torch.zeros((mb.mole_nf_scales_bytes(rows, N, d, block, sb),), dtype=torch.uint8, device="cuda")
    mb.mole_quantize_lut(tab_d, codes, scales, rows, N, d, bits, block, sb)
    torch.cuda.synchronize()
    return codes, scales


def scales_as_f32(scales_u8, sb):
    raw = scales_u8.cpu().numpy()
    return raw.view(np.float32) if sb == 4 else wl.bf16_bits_to_f32(raw.view(np.uint16))


@pytest.mark.parametrize("bits,block,sb,d,N,V", [
    (4, 768, 4, 768, 4, 300),       # the paper's NF4 setting on 160M rows: one block per row, spanning two chunks
    (3, 128, 2, 768, 4, 300),       # the paper's NF3 setting
    (4, 256, 2, 1024, 16, 128),     # 410M rows
    (3, 1024, 4, 1024, 16, 64),
    (4, 384, 4, 768, 2, 50),        # blocks that straddle the 512-column chunk boundary
    (3, 48, 2, 96, 3, 40),          # small ragged shapes
    (4, 8, 4, 2048, 4, 20),
])
def test_quantiser_is_bit_exact(bits, block, sb, d, N, V):
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, L=1, seed=bits * 7 + block)
    table = wl.random_table(w)                                       # bf16 bits [V,N,d]
    table[3, :, :] = 0                                               # all-zero blocks
    table[5, 0, : min(64, d)] = wl.f32_to_bf16_bits(np.full(min(64, d), 3.0, np.float32))   # many equal maxima
    codes_d, scales_d = gpu_quantize(table, V, N, d, bits, block, sb)
    ref_codes, ref_scales = nf.quantize(wl.bf16_bits_to_f32(table), bits, block)
    np.testing.assert_array_equal(scales_as_f32(scales_d, sb)[:ref_scales.size].reshape(ref_scales.shape), ref_scales)
    got = codes_d.cpu().numpy().reshape(V, N, d * bits // 8)
    np.testing.assert_array_equal(got, nf.pack(ref_codes, bits))                 # packed bytes, bit for bit
    np.testing.assert_array_equal(nf.unpack(got, bits, d), ref_codes)


def run_nf_forward(w, table, li, ids, bits, block, sb, L=1, dedup=False, residual=False):
    import torch
    tabs = table if L > 1 else [table]
    packs = [gpu_quantize(t, w.V, w.N, w.d, bits, block, sb) for t in tabs]
    codes_d = torch.stack([p[0] for p in packs])
    scales_d = torch.stack([p[1] for p in packs])
    lis = li if L > 1 else [li]
    stack = lambda k: to_dev(np.stack([x[k] for x in lis]), wl.BF16)
    h_d, wr_d, sh_d = stack("h"), stack("W_r"), stack("shared")
    rs_d = stack("residual") if residual else None
    ids_d = torch.from_numpy(ids).cuda()
    out_d = torch.full_like(h_d, float("nan"))
    T = len(ids)
    gates_d = torch.zeros((L, T, w.N), dtype=torch.float32, device="cuda")
    rows_d = torch.zeros((T,), dtype=torch.int64, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    flags, plan = 0, None
    if dedup:
        plan = torch.empty((mb.mole_dedup_workspace(T, w.V) // 4,), dtype=torch.int32, device="cuda")
        uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
        mb.mole_dedup_ids(ids_d, T, w.V, uq, iv, torch.zeros_like(err), err, plan)
        flags = mb.MOLE_FLAG_DEDUP
    mb.mole_lookup_forward_nf(codes_d, codes_d.shape[1], scales_d, scales_d.shape[1] // sb, ids_d, None, h_d, wr_d,
                              sh_d, rs_d, out_d, T * w.d, gates_d, rows_d, err, L, T, w.V, w.d, w.N, bits, block, sb,
                              flags, plan)
    # the kernel that writes no debug outputs is a variant of its own (same arithmetic): the same bits
    out2_d = torch.full_like(h_d, float("nan"))
    err2 = torch.zeros_like(err)
    mb.mole_lookup_forward_nf(codes_d, codes_d.shape[1], scales_d, scales_d.shape[1] // sb, ids_d, None, h_d, wr_d,
                              sh_d, rs_d, out2_d, T * w.d, None, None, err2, L, T, w.V, w.d, w.N, bits, block, sb,
                              flags, plan)
    torch.cuda.synchronize()
    assert torch.equal(out_d.view(torch.int16), out2_d.view(torch.int16)) and int(err.item()) == int(err2.item())
    return to_host(out_d, wl.BF16), gates_d.cpu().numpy(), rows_d.cpu().numpy(), int(err.item())


def oracle_nf_forward(table, li, ids, bits, block, residual=False):
    codes, scales = nf.quantize(wl.bf16_bits_to_f32(table), bits, block)
    deq = nf.dequantize(codes, scales, bits, block)                    # fp32 values the GPU sees after dequant
    return oracle.lookup_forward(deq, ids, wl.storage_to_f64(li["h"], wl.BF16), wl.storage_to_f64(li["W_r"], wl.BF16),
                                 wl.storage_to_f64(li["shared"], wl.BF16),
                                 wl.storage_to_f64(li["residual"], wl.BF16) if residual else None)


@pytest.mark.parametrize("bits,block,sb,d,N,T,V", [
    (4, 768, 4, 768, 4, 100, 500),
    (3, 128, 2, 768, 4, 100, 500),
    (4, 256, 4, 1024, 16, 333, 1000),
    (3, 128, 2, 1024, 16, 203, 1000),
    (4, 512, 2, 1024, 32, 77, 300),
    (3, 64, 4, 2048, 8, 40, 200),
    (4, 104, 4, 520, 16, 9, 64),         # ragged last chunk
    (3, 16, 2, 64, 64, 50, 100),
    (4, 1024, 4, 1024, 2, 90, 300),      # two experts: the router is padded to four
    (3, 128, 2, 768, 2, 61, 300),
])
@pytest.mark.parametrize("dedup", [False, True])
def test_forward_matches_oracle_on_dequantised_table(bits, block, sb, d, N, T, V, dedup):
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"nf{bits} d{d} N{N}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    li["W_r"] = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)
    out, gates, rows, err = run_nf_forward(w, table, li, ids, bits, block, sb, dedup=dedup, residual=True)
    ref, ref_g, ref_rows, ref_err = oracle_nf_forward(table, li, ids, bits, block, residual=True)
    assert err == 0 == ref_err
    np.testing.assert_array_equal(rows, ref_rows)
    assert_close(gates[0].astype(np.float64), ref_g, wl.BF16, "gates")
    assert_close(wl.storage_to_f64(out[0], wl.BF16), ref, wl.BF16, f"nf forward ({w.name})")


@pytest.mark.parametrize("seed", range(12))
def test_seeded_random_shapes(seed):
    """Bits, block, scale width, d, N and T drawn from what the quantised path documents."""
    rng = np.random.default_rng(3000 + seed)
    bits = int(rng.choice([3, 4]))
    block = int(rng.choice([8, 16, 64, 128])) * (2 if bits == 3 else 1)
    d = block * int(rng.integers(1, max(2, 1536 // block)))
    sb = int(rng.choice([2, 4]))
    N = int(rng.choice([2, 4, 8, 16, 32, 64]))
    while d * max(N, 4) * 2 > 150 * 1024:        # the router weight has to fit in LDS (else MOLE_EUNSUPPORTED)
        N //= 2
    T = int(rng.integers(1, 70))
    V = int(rng.integers(max(2, T // 8), 300))
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"nf random seed {seed}: nf{bits} "
                  f"block{block} sb{sb} d{d} N{N} T{T}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    li["W_r"] = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)
    residual, dedup = bool(rng.integers(2)), bool(rng.integers(2))
    out, gates, rows, err = run_nf_forward(w, table, li, ids, bits, block, sb, dedup=dedup, residual=residual)
    ref, ref_g, ref_rows, ref_err = oracle_nf_forward(table, li, ids, bits, block, residual=residual)
    assert err == 0 == ref_err
    np.testing.assert_array_equal(rows, ref_rows)
    assert_close(gates[0].astype(np.float64), ref_g, wl.BF16, "gates")
    assert_close(wl.storage_to_f64(out[0], wl.BF16), ref, wl.BF16, f"nf forward ({w.name})")


@pytest.mark.parametrize("bits,block,sb,d,N,T,V,dedup", [
    (4, 1024, 4, 1024, 32, 16384, 800, False),   # N = 32: two parts of 16 experts, eight waves, doubled grid
    (3, 128, 2, 1536, 32, 9001, 500, True),
    (4, 128, 2, 512, 64, 16384, 300, False),     # four parts
])
def test_large_batches_with_many_experts(bits, block, sb, d, N, T, V, dedup):
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"nf{bits} large d{d} N{N} T{T}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    out, gates, rows, err = run_nf_forward(w, table, li, ids, bits, block, sb, dedup=dedup, residual=True)
    ref, ref_g, ref_rows, ref_err = oracle_nf_forward(table, li, ids, bits, block, residual=True)
    assert err == 0 == ref_err
    np.testing.assert_array_equal(rows, ref_rows)
    assert_close(gates[0].astype(np.float64), ref_g, wl.BF16, "gates")
    assert_close(wl.storage_to_f64(out[0], wl.BF16), ref, wl.BF16, f"nf forward ({w.name})")


def test_layers_and_bad_ids():
    w = wl.scaled(wl.CONFIGS["decode410m"], V=400, d=1024, N=16, T=64, L=3)
    tabs = [wl.random_table(w, l) for l in range(w.L)]
    lis = [wl.layer_inputs(w, l) for l in range(w.L)]
    ids = wl.token_ids(w).copy()
    ids[[2, 60]] = [400, -3]
    out, gates, rows, err = run_nf_forward(w, tabs, lis, ids, 4, 256, 4, L=w.L)
    assert err == 1
    for l in range(w.L):
        ref, _, ref_rows, _ = oracle_nf_forward(tabs[l], lis[l], ids, 4, 256)
        assert_close(wl.storage_to_f64(out[l], wl.BF16), ref, wl.BF16, f"layer {l}")
        np.testing.assert_array_equal(out[l][[2, 60]], lis[l]["shared"][[2, 60]])
    np.testing.assert_array_equal(rows, ref_rows)


@pytest.mark.parametrize("bits,block,sb,d,N,T,V,L,pad", [
    (4, 1024, 4, 1024, 16, 32, 600, 3, 0),      # the benchmark's NF4 setting: 16-byte units
    (3, 128, 2, 1024, 16, 64, 600, 2, 0),       # NF3, bf16 scales
    (4, 16, 2, 16, 4, 40, 50, 2, 0),            # 8-byte scale rows: 4-byte units
    (4, 16, 2, 16, 4, 40, 50, 2, 1),            # scale layer stride of an odd number of bf16 values: 2-byte units
])
def test_offloaded_quantised_table(bits, block, sb, d, N, T, V, L, pad):
    """Codes and scales of all layers in pinned host memory: the rows of the distinct ids arrive byte for
    byte in the staging buffers, and the forward on them (slot = inverse map) equals the forward on the
    device-resident quantised tables bit for bit."""
    import torch
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, N=N, T=T, L=L, name=f"nf{bits} offload")
    tabs = [wl.random_table(w, l) for l in range(L)]
    lis = [wl.layer_inputs(w, l) for l in range(L)]
    ids = wl.token_ids(w)
    packs = [gpu_quantize(t, V, N, d, bits, block, sb) for t in tabs]
    code_row, scale_row = N * d * bits // 8, N * (d // block)                 # bytes / scale elements per id
    codes_d = torch.stack([p[0][:V * code_row] for p in packs])              # [L, V * code_row] bytes
    scales_d = torch.stack([p[1][:V * scale_row * sb] for p in packs])       # [L, V * scale_row * sb] bytes
    ls_scale = V * scale_row + pad                                            # host layer stride, scale elements
    host_codes = codes_d.cpu().pin_memory()
    host_scales = torch.zeros((L, ls_scale * sb), dtype=torch.uint8).pin_memory()
    host_scales[:, :V * scale_row * sb] = scales_d.cpu()

    ids_d = torch.from_numpy(ids).cuda()
    uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, T, V, uniq_d, inv_d, nu, err, plan)
    U_cap = T
    st_codes = torch.zeros((L, U_cap * code_row), dtype=torch.uint8, device="cuda")
    st_scales = torch.zeros((L, U_cap * scale_row * sb), dtype=torch.uint8, device="cuda")
    mb.mole_offload_fetch_nf(host_codes, V * code_row, host_scales, ls_scale, uniq_d, nu, st_codes, U_cap * code_row,
                             st_scales, U_cap * scale_row, err, L, U_cap, V, d, N, bits, block, sb)
    torch.cuda.synchronize()
    U = int(nu.item())
    uniq = np.unique(ids)
    assert U == len(uniq) and int(err.item()) == 0
    uq = torch.from_numpy(uniq.astype(np.int64))
    want_c = codes_d.cpu().view(L, V, code_row)[:, uq]
    want_s = scales_d.cpu().view(L, V, scale_row * sb)[:, uq]
    assert torch.equal(st_codes.cpu().view(L, U_cap, code_row)[:, :U], want_c)
    assert torch.equal(st_scales.cpu().view(L, U_cap, scale_row * sb)[:, :U], want_s)
    assert not st_codes.view(L, U_cap, code_row)[:, U:].any()

    stack = lambda k: to_dev(np.stack([x[k] for x in lis]), wl.BF16)
    h_d, wr_d, sh_d = stack("h"), stack("W_r"), stack("shared")
    out_staged, out_res = torch.zeros_like(h_d), torch.zeros_like(h_d)
    mb.mole_lookup_forward_nf(st_codes, U_cap * code_row, st_scales, U_cap * scale_row, ids_d, inv_d, h_d, wr_d, sh_d,
                              None, out_staged, T * d, None, None, err, L, T, U_cap, d, N, bits, block, sb)
    mb.mole_lookup_forward_nf(codes_d, V * code_row, scales_d, V * scale_row, ids_d, None, h_d, wr_d, sh_d, None,
                              out_res, T * d, None, None, err, L, T, V, d, N, bits, block, sb)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    a, b = to_host(out_staged, wl.BF16), to_host(out_res, wl.BF16)
    np.testing.assert_array_equal(a, b)
    ref, _, _, _ = oracle_nf_forward(tabs[L - 1], lis[L - 1], ids, bits, block)
    assert_close(wl.storage_to_f64(a[L - 1], wl.BF16), ref, wl.BF16, "staged quantised forward")


@pytest.mark.parametrize("bits,block,sb", [(4, 256, 4), (3, 128, 2)])
def test_storage_tier_step_with_quantised_tables(tmp_path, bits, block, sb):
    """The quantised table in two LUT files of raw bytes (codes, scales), id-major: the distinct ids' rows
    are read into pinned memory, pulled to the device and fed to the dequantising forward, which then
    equals the forward on the device-resident quantised tables bit for bit."""
    import torch
    L, V, d, N, T = 3, 800, 1024, 16, 48
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, N=N, T=T, L=L, name=f"nf{bits} files")
    tabs = [wl.random_table(w, l) for l in range(L)]
    lis = [wl.layer_inputs(w, l) for l in range(L)]
    ids = wl.token_ids(w)
    packs = [gpu_quantize(t, V, N, d, bits, block, sb) for t in tabs]
    cb, sbytes = d * bits // 8, (d // block) * sb                          # bytes per expert row
    codes_d = torch.stack([p[0][:V * N * cb] for p in packs])
    scales_d = torch.stack([p[1][:V * N * sbytes] for p in packs])
    paths = {}
    for name, src, width in (("codes", codes_d, cb), ("scales", scales_d, sbytes)):
        paths[name] = str(tmp_path / f"{name}.molelut")
        f = mb.mole_lut_file_create(paths[name], mb.MOLE_U8, mb.MOLE_LAYOUT_ID_MAJOR, L, V, N, width)
        for l in range(L):
            mb.mole_lut_file_write_layer(f, l, src[l].cpu(), 3)
        mb.mole_lut_file_close(f)

    ids_d = torch.from_numpy(ids).cuda()
    uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, T, V, uniq_d, inv_d, nu, err, plan)
    U = int(nu.item())
    uniq_h = uniq_d[:U].cpu()
    U_cap = T
    staged = {}
    for name, width in (("codes", cb), ("scales", sbytes)):
        f, desc = mb.mole_lut_file_open(paths[name])
        try:
            assert (desc.dtype, desc.L, desc.N, desc.d, desc.V) == (mb.MOLE_U8, L, N, width, V)
            pinned = torch.zeros((U_cap, L, N, width), dtype=torch.uint8).pin_memory()
            mb.mole_lut_file_read_rows(f, uniq_h, U, pinned, 3)
        finally:
            mb.mole_lut_file_close(f)
        staged[name] = torch.zeros((L, U_cap * N * width), dtype=torch.uint8, device="cuda")
        mb.mole_offload_fetch_idmajor(pinned, None, nu, staged[name], U_cap * N * width, err, L, U_cap, U_cap, width, N,
                                      mb.MOLE_U8)
    torch.cuda.synchronize()
    uq = torch.from_numpy(np.unique(ids).astype(np.int64))
    assert torch.equal(staged["codes"].cpu().view(L, U_cap, N * cb)[:, :U], codes_d.cpu().view(L, V, N * cb)[:, uq])
    assert torch.equal(staged["scales"].cpu().view(L, U_cap, N * sbytes)[:, :U],
                       scales_d.cpu().view(L, V, N * sbytes)[:, uq])

    stack = lambda k: to_dev(np.stack([x[k] for x in lis]), wl.BF16)
    h_d, wr_d, sh_d = stack("h"), stack("W_r"), stack("shared")
    out_staged, out_res = torch.zeros_like(h_d), torch.zeros_like(h_d)
    mb.mole_lookup_forward_nf(staged["codes"], U_cap * N * cb, staged["scales"], U_cap * N * (d // block), ids_d, inv_d,
                              h_d, wr_d, sh_d, None, out_staged, T * d, None, None, err, L, T, U_cap, d, N, bits, block,
                              sb)
    mb.mole_lookup_forward_nf(codes_d, V * N * cb, scales_d, V * N * (d // block), ids_d, None, h_d, wr_d, sh_d, None,
                              out_res, T * d, None, None, err, L, T, V, d, N, bits, block, sb)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    np.testing.assert_array_equal(to_host(out_staged, wl.BF16), to_host(out_res, wl.BF16))


def test_offloaded_quantised_table_reports_overflowing_staging():
    import torch
    V, N, d, T = 100, 4, 64, 50
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, N=N, T=T, L=1, ids="uniform")
    codes, scales = gpu_quantize(wl.random_table(w), V, N, d, 4, 64, 4)
    hc, hs = codes.cpu().pin_memory(), scales.cpu().pin_memory()
    ids_d = torch.from_numpy(wl.token_ids(w)).cuda()
    uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, T, V, uq, iv, nu, err, plan)
    U_cap = 5
    sc = torch.zeros((U_cap * N * d // 2 + 64,), dtype=torch.uint8, device="cuda")
    ss = torch.zeros((U_cap * N * 4 + 64,), dtype=torch.uint8, device="cuda")
    mb.mole_offload_fetch_nf(hc, 0, hs, 0, uq, nu, sc, 0, ss, 0, err, 1, U_cap, V, d, N, 4, 64, 4)
    torch.cuda.synchronize()
    assert int(nu.item()) > U_cap and int(err.item()) == 1
    assert not sc[U_cap * N * d // 2:].any() and not ss[U_cap * N * 4:].any()      # nothing past the capacity


@pytest.mark.parametrize("bits,block,sb,d,N,T,V", [
    (4, 1024, 4, 1024, 16, 203, 500),
    (3, 128, 2, 1024, 16, 64, 500),
    (4, 512, 2, 1024, 32, 77, 300),
    (4, 104, 4, 520, 8, 9, 64),          # ragged last chunk
    (3, 64, 4, 2048, 4, 40, 200),        # four chunks
])
@pytest.mark.parametrize("dedup", [False, True])
def test_layer_forward_on_quantised_table(bits, block, sb, d, N, T, V, dedup):
    """mole_layer_forward_nf (state after attention in, RMSNorm and residual inside the kernel) against the
    oracle of the inference listing run on the dequantised table."""
    import torch
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"nf{bits} layer d{d} N{N}")
    table, li, ni = wl.random_table(w), wl.layer_inputs(w), wl.norm_inputs(w, 0)
    W_r = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)
    ids = wl.token_ids(w).copy()
    if T > 8:
        ids[T // 3] = V + 2
    codes, scales = gpu_quantize(table, V, N, d, bits, block, sb)
    x_d, lw_d, wr_d, sh_d = (to_dev(a, wl.BF16) for a in (ni["x"], ni["ln_w"], W_r, li["shared"]))
    ids_d = torch.from_numpy(ids).cuda()
    out_d = torch.full_like(x_d, float("nan"))
    gates_d = torch.zeros((T, N), dtype=torch.float32, device="cuda")
    rows_d = torch.zeros((T,), dtype=torch.int64, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    flags, plan = 0, None
    if dedup:
        plan = torch.empty((mb.mole_dedup_workspace(T, V) // 4,), dtype=torch.int32, device="cuda")
        uq, iv = torch.empty_like(ids_d), torch.empty_like(ids_d)
        mb.mole_dedup_ids(ids_d, T, V, uq, iv, torch.zeros_like(err), torch.zeros_like(err), plan)
        flags = mb.MOLE_FLAG_DEDUP
    mb.mole_layer_forward_nf(codes, 0, scales, 0, ids_d, None, x_d, lw_d, 1e-5, wr_d, sh_d, out_d, 0, gates_d, rows_d, err,
                             1, T, V, d, N, bits, block, sb, flags, plan)
    torch.cuda.synchronize()
    q_codes, q_scales = nf.quantize(wl.bf16_bits_to_f32(table), bits, block)
    deq = nf.dequantize(q_codes, q_scales, bits, block)
    ref, ref_g, _, ref_rows, ref_err = oracle.layer_forward(deq, ids, ni["x"], ni["ln_w"], 1e-5, W_r, li["shared"])
    assert int(err.item()) == ref_err
    np.testing.assert_array_equal(rows_d.cpu().numpy(), ref_rows)
    assert_close(gates_d.cpu().numpy().astype(np.float64), ref_g, wl.BF16, "gates")
    assert_close(wl.storage_to_f64(to_host(out_d, wl.BF16), wl.BF16), ref, wl.BF16, f"layer forward nf ({w.name})")


def test_quantisation_error_is_what_the_levels_allow():
    """Against the unquantised table the routed term moves by at most the level gap times the scales."""
    w = wl.scaled(wl.CONFIGS["decode410m"], V=300, d=768, N=4, T=80, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    exact, g, _, _ = oracle.lookup_forward(table, ids, li["h"], li["W_r"], li["shared"])
    for bits, block, sb in ((4, 768, 4), (3, 128, 2)):
        out, _, _, _ = run_nf_forward(w, table, li, ids, bits, block, sb)
        _, scales = nf.quantize(wl.bf16_bits_to_f32(table), bits, block)
        gap = np.diff(nf.codebook(bits).astype(np.float64)).max() / 2
        bound = (g[:, :, None] * np.repeat(scales[ids].astype(np.float64), block, axis=-1)).sum(axis=1) * gap
        err = np.abs(wl.storage_to_f64(out[0], wl.BF16) - exact)
        assert (err <= bound + 1e-3 + 2e-2 * np.abs(exact)).all()
        assert err.mean() > 1e-4          # and it is not accidentally the unquantised table


@pytest.mark.parametrize("bits,block,sb,N", [(4, 256, 4, 16), (3, 128, 2, 8), (4, 1024, 2, 32)])
@pytest.mark.parametrize("k", [-60, 40])
def test_forward_is_invariant_under_power_of_two_table_scales(bits, block, sb, N, k):
    """The kernel carries gate x scale in fp16 relative to the largest of a chunk, so a table of very small
    or very large values must neither underflow nor overflow: scaling table and shared term by 2^k
    (exact in bf16; codes unchanged, scales times 2^k) scales the output by exactly 2^k."""
    w = wl.scaled(wl.CONFIGS["decode410m"], V=200, d=1024, N=N, T=70, L=1, seed=90 + bits)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    out0, _, _, err0 = run_nf_forward(w, table, li, ids, bits, block, sb)
    ref, _, _, _ = oracle_nf_forward(table, li, ids, bits, block)
    assert_close(wl.storage_to_f64(out0[0], wl.BF16), ref, wl.BF16, "unscaled")
    f = 2.0 ** k
    table_k = wl.to_storage(wl.storage_to_f64(table, wl.BF16) * f, wl.BF16)
    li_k = dict(li, shared=wl.to_storage(wl.storage_to_f64(li["shared"], wl.BF16) * f, wl.BF16))
    np.testing.assert_array_equal(wl.storage_to_f64(table_k, wl.BF16), wl.storage_to_f64(table, wl.BF16) * f)
    outk, _, _, errk = run_nf_forward(w, table_k, li_k, ids, bits, block, sb)
    assert err0 == errk == 0
    np.testing.assert_array_equal(wl.storage_to_f64(outk[0], wl.BF16), wl.storage_to_f64(out0[0], wl.BF16) * f)


@pytest.mark.parametrize("bits,block,sb", [(4, 1024, 4), (3, 128, 2)])
def test_full_size_layer_sampled(bits, block, sb):
    """One 410M layer at full size (V = 50304, N = 16, d = 1024, T = 256), the two formats the benchmark
    times: quantised on the device; the oracle runs on a sample of tokens, whose rows are copied back as
    bf16, quantised and dequantised by the codec oracle (the device quantiser is bit-exact, tested above)."""
    import torch
    w = wl.scaled(wl.CONFIGS["decode410m"], L=1)
    tab_d = wl.device_table(w, 0, "cuda")
    codes = torch.zeros((mb.mole_nf_codes_bytes(w.V, w.N, w.d, bits),), dtype=torch.uint8, device="cuda")
    scales = torch.zeros((mb.mole_nf_scales_bytes(w.V, w.N, w.d, block, sb),), dtype=torch.uint8, device="cuda")
    mb.mole_quantize_lut(tab_d, codes, scales, w.V, w.N, w.d, bits, block, sb)
    li, ids = wl.layer_inputs(w), wl.token_ids(w)
    h_d, wr_d, sh_d = (to_dev(li[k], wl.BF16) for k in ("h", "W_r", "shared"))
    ids_d = torch.from_numpy(ids).cuda()
    out_d = torch.full_like(h_d, float("nan"))
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    mb.mole_lookup_forward_nf(codes, 0, scales, 0, ids_d, None, h_d, wr_d, sh_d, None, out_d, 0, None, None, err, 1,
                              w.T, w.V, w.d, w.N, bits, block, sb, 0, None)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    out = to_host(out_d, wl.BF16)
    assert not np.isnan(wl.storage_to_f64(out, wl.BF16)).any()
    sample = np.unique(np.concatenate([np.random.default_rng(4).integers(0, w.T, 40), [0, w.T - 1]]))
    rows = to_host(tab_d[torch.from_numpy(ids[sample].astype(np.int64)).cuda()], wl.BF16)          # [S,N,d] bf16 bits
    c, sc = nf.quantize(wl.bf16_bits_to_f32(rows), bits, block)
    deq = nf.dequantize(c, sc, bits, block)
    f = lambda a: wl.storage_to_f64(a, wl.BF16)
    ref, *_ = oracle.lookup_forward(deq, np.arange(len(sample), dtype=np.int32), f(li["h"][sample]), f(li["W_r"]),
                                    f(li["shared"][sample]))
    assert_close(f(out[sample]), ref, wl.BF16, f"NF{bits} full-size sample")
