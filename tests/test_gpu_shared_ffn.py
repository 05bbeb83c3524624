"""GPU parity of mole_shared_ffn_forward (the layer with its shared expert inside: both products on the matrix
cores, gather and gate-weighted sum in the second product's epilogue) against the fp64 oracle, through the C
ABI.  Seeded synthetic inputs."""
import numpy as np
import pytest

import oracle
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl
from helpers import DT, assert_close, gathered_rows, to_dev, to_host

pytestmark = pytest.mark.gpu


def run(w, D_s, table, ids, li, fw, residual=True, slot=None, rows=None, act=mb.MOLE_GELU_ERF, table_dev=None):
    import torch
    T = len(ids)
    tab_d = table_dev if table_dev is not None else to_dev(table, w.dtype)
    n_rows = rows if rows is not None else tab_d.shape[0]
    ids_d = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).cuda()
    slot_d = None if slot is None else torch.from_numpy(np.ascontiguousarray(slot, dtype=np.int32)).cuda()
    h_d, wr_d = to_dev(li["h"], w.dtype), to_dev(li["W_r"], w.dtype)
    w1_d, w2_d, b1_d, b2_d = (to_dev(fw[k], w.dtype) for k in ("W1", "W2", "b1", "b2"))
    rs_d = to_dev(li["residual"], w.dtype) if residual else None
    out_d = torch.full((T, w.d), float("nan"), dtype=h_d.dtype, device="cuda")
    gates_d = torch.full((T, w.N), -1.0, dtype=torch.float32, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    ws = torch.empty((mb.mole_shared_ffn_workspace(T, w.d, D_s, w.N),), dtype=torch.uint8, device="cuda")
    mb.mole_shared_ffn_forward(tab_d, ids_d, slot_d, h_d, wr_d, w1_d, b1_d, w2_d, b2_d, rs_d, out_d, gates_d, err_d, T,
                               n_rows, w.d, D_s, w.N, DT[w.dtype], act, ws)
    torch.cuda.synchronize()
    return dict(out=to_host(out_d, w.dtype), gates=gates_d.cpu().numpy(), err=int(err_d.item()))


def check(w, D_s, table, ids, li, fw, residual=True, act=mb.MOLE_GELU_ERF):
    ref, ref_g, _, ref_err = oracle.layer_with_shared_ffn(
        table, ids, li["h"], li["W_r"], fw["W1"], fw["W2"], fw["b1"], fw["b2"], li["residual"] if residual else None,
        act=oracle.GELU_TANH if act == mb.MOLE_GELU_TANH else oracle.GELU_ERF)
    got = run(w, D_s, table, ids, li, fw, residual=residual, act=act)
    assert got["err"] == ref_err
    assert_close(got["gates"].astype(np.float64), ref_g, w.dtype, f"gates ({w.name})")
    assert_close(wl.storage_to_f64(got["out"], w.dtype), ref, w.dtype, f"out ({w.name})")
    return got


@pytest.mark.parametrize("d,D_s,N,T,V,bias,residual", [
    (256, 512, 16, 300, 500, True, True),       # 256-wide tiles (direct-to-LDS kernel), ragged last row tile
    (128, 384, 8, 77, 200, True, False),        # 128-wide tiles (register-staged kernel)
    (384, 256, 4, 513, 300, False, True),       # d not a multiple of 256: second product on the narrow kernel
    (1024, 512, 32, 260, 100, True, True),      # 410M-shaped rows, N = 32
    (256, 256, 2, 40, 50, False, False),        # two experts (router padded to four)
    (512, 1024, 64, 130, 64, True, True),       # N = 64
])
@pytest.mark.parametrize("hidden", [0, 1, 2])
def test_shapes(tuning, d, D_s, N, T, V, bias, residual, hidden):
    """hidden: the format the hidden activation is carried in -- chosen by the library (fp16 here: the values are
    small), forced to fp16, forced to the bf16 hi + lo pair."""
    tuning("MOLE_BUILD_HIDDEN", hidden)
    w = wl.scaled(wl.CONFIGS["decode410m"], V=V, d=d, N=N, T=T, L=1, name=f"shared ffn d{d} Ds{D_s} N{N} T{T}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w).copy()
    li["W_r"] = wl.to_storage(wl.storage_to_f64(li["W_r"], w.dtype) * 5.0, w.dtype)
    if T > 50:
        ids[T // 2] = V + 1                       # an id outside the table: shared + residual only, flagged
    check(w, D_s, table, ids, li, wl.shared_ffn_weights(w, D_s, bias=bias), residual=residual)


@pytest.mark.parametrize("gather_last", [0, 1])
def test_rows_gathered_before_or_behind_the_main_loop(tuning, gather_last):
    """Every other workgroup of the second product gathers its table rows BEFORE its main loop and starts the
    accumulators from them (the default), or all gather behind it (MOLE_FFN_GATHER_LAST = 1): both against the
    oracle, on a tile grid that holds both kinds (3 x 4 tiles, ragged last row tile, an id outside the table in a
    workgroup of each kind)."""
    tuning("MOLE_FFN_GATHER_LAST", gather_last)
    w = wl.scaled(wl.CONFIGS["decode410m"], V=300, d=1024, N=16, T=600, L=1, name=f"shared ffn gather_last={gather_last}")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w).copy()
    ids[10] = -1
    ids[300] = 300
    check(w, 512, table, ids, li, wl.shared_ffn_weights(w, 512, bias=True), residual=True)


def test_tanh_form_and_large_hidden_values():
    """GELU in its tanh form; then first-layer weights scaled so that pre-activations can leave the fp16 range (the
    bound is then violated and the library must take the hi + lo pair, which has no range limit)."""
    w = wl.scaled(wl.CONFIGS["decode410m"], V=300, d=256, N=16, T=150, L=1, name="shared ffn tanh")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    fw = wl.shared_ffn_weights(w, 512)
    check(w, 512, table, ids, li, fw, act=mb.MOLE_GELU_TANH)
    fw["W1"] = wl.to_storage(wl.storage_to_f64(fw["W1"], w.dtype) * 40000.0, w.dtype)
    fw["W2"] = wl.to_storage(wl.storage_to_f64(fw["W2"], w.dtype) / 40000.0, w.dtype)
    check(w, 512, table, ids, li, fw)


def test_equals_the_unfused_path_given_the_oracles_shared_term():
    """Cross-check inside the library: mole_lookup_forward fed with FFN_shared(h) from the oracle (rounded to
    bf16) and the residual; the two differ by that rounding only."""
    import torch
    w = wl.scaled(wl.CONFIGS["decode410m"], V=400, d=256, N=16, T=200, L=1, name="shared ffn vs unfused")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    fw = wl.shared_ffn_weights(w, 512)
    fused = run(w, 512, table, ids, li, fw)
    shared = wl.to_storage(oracle.shared_ffn(li["h"], fw["W1"], fw["W2"], fw["b1"], fw["b2"]), w.dtype)
    out_d = torch.zeros((w.T, w.d), dtype=torch.bfloat16, device="cuda")
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    mb.mole_lookup_forward(to_dev(table, w.dtype), torch.from_numpy(ids).cuda(), None, to_dev(li["h"], w.dtype),
                           to_dev(li["W_r"], w.dtype), to_dev(shared, w.dtype), to_dev(li["residual"], w.dtype), out_d,
                           None, None, err_d, w.T, w.V, w.d, w.N, DT[w.dtype])
    torch.cuda.synchronize()
    assert_close(wl.storage_to_f64(fused["out"], w.dtype), wl.storage_to_f64(to_host(out_d, w.dtype), w.dtype), w.dtype,
                 "fused against unfused")


def test_slot_indirection_and_zero_second_matrix():
    """Staged rows (slot = position among the distinct ids); with W2 = 0 the shared term is b2 exactly, so the call
    reduces to the plain lookup plus a constant row."""
    w = wl.scaled(wl.CONFIGS["decode410m"], V=300, d=256, N=8, T=120, L=1, name="shared ffn slot")
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    fw = wl.shared_ffn_weights(w, 256)
    fw["W2"] = np.zeros_like(fw["W2"])
    uniq, inv = np.unique(ids, return_inverse=True)
    got = run(w, 256, np.ascontiguousarray(table[uniq]), ids, li, fw, slot=inv.astype(np.int32), residual=False)
    b2 = np.tile(wl.storage_to_f64(fw["b2"], w.dtype), (w.T, 1))
    ref, _, _, _ = oracle.lookup_forward(table, ids, wl.storage_to_f64(li["h"], w.dtype), wl.storage_to_f64(li["W_r"], w.dtype), b2)
    assert_close(wl.storage_to_f64(got["out"], w.dtype), ref, w.dtype, "slot + zero second matrix")


def test_rejects_unsupported_shapes():
    import torch
    a = torch.zeros((256,), dtype=torch.int32, device="cuda")
    base = dict(table=a, ids=a, slot=None, h=a, W_r=a, W1=a, b1=None, W2=a, b2=None, residual=None, out=a, gates_dbg=None,
                err_flag=None, T=4, rows=10, d=128, D_s=128, N=4, dtype=mb.MOLE_BF16, act=mb.MOLE_GELU_ERF, workspace=a,
                workspace_bytes=1 << 20)
    for kw, status in ((dict(d=64), mb.MOLE_EUNSUPPORTED), (dict(D_s=200), mb.MOLE_EUNSUPPORTED),
                       (dict(N=5), mb.MOLE_EUNSUPPORTED), (dict(dtype=mb.MOLE_F32), mb.MOLE_EUNSUPPORTED),
                       (dict(W1=None), mb.MOLE_EINVAL), (dict(workspace_bytes=16), mb.MOLE_EWORKSPACE),
                       (dict(act=7), mb.MOLE_EINVAL)):
        args = dict(base)
        args.update(kw)
        with pytest.raises(mb.MoleError) as e:
            mb.mole_shared_ffn_forward(**args)
        assert e.value.status == status, kw
    args = dict(base)
    args.update(T=0)
    mb.mole_shared_ffn_forward(**args)


def test_full_size_prefill_layer():
    """The prefill shape at full size: 16384 tokens, N = 32, d = 1024, D_s = 4096 over the 3.3 GB table.  The
    gates of every token, and the output rows of every eighth token and of the last row tile, against the oracle
    (its fp64 shared expert takes two seconds per thousand tokens on the host cores)."""
    import torch
    w = wl.scaled(wl.CONFIGS["prefill410m"], L=1)
    tab_d = wl.device_table(w, 0, "cuda")
    ids, li = wl.token_ids(w), wl.layer_inputs(w)
    fw = wl.shared_ffn_weights(w, 4096)
    got = run(w, 4096, None, ids, li, fw, table_dev=tab_d)
    assert got["err"] == 0
    assert not np.isnan(wl.storage_to_f64(got["out"], w.dtype)).any()
    assert_close(got["gates"].astype(np.float64), oracle.gates(li["h"], li["W_r"]), w.dtype, "gates (prefill)")
    sample = np.unique(np.concatenate([np.arange(0, w.T, 8), np.arange(w.T - 256, w.T)]))
    rows, inv = gathered_rows(tab_d, ids[sample])
    ref, _, _, _ = oracle.layer_with_shared_ffn(rows, inv, li["h"][sample], li["W_r"], fw["W1"], fw["W2"], fw["b1"],
                                                fw["b2"], li["residual"][sample])
    assert_close(wl.storage_to_f64(got["out"][sample], w.dtype), ref, w.dtype, "out (prefill sample)")
