"""End-to-end on the GPU: the table built by mole_build_lut, looked up by mole_lookup_forward, must
reproduce the training-form layer (every expert FFN run on the token's embedding, Sec. 3.2) -- the
re-parameterization is exact.  Also the smaller shapes of the paper's model table, HIP-graph replay, and
misuse of the plan."""
import numpy as np
import pytest
import scipy.special

import oracle
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl
from helpers import DT, assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu


def training_form_layer(ew, li, ids, dtype):
    """sum_j softmax(h W_r)_j * FFN_j(E[id]) + shared, numpy fp64, one token at a time.  Each expert
    output is rounded to the table's storage type first: a bf16 table holds bf16(FFN_j(E[id])), and with
    shared ~ N(0,1) cancelling against the routed term that rounding (2^-9 of entries up to ~1) is
    visible at atol 1e-3 if it is left out of the reference."""
    f = lambda a: wl.storage_to_f64(a, dtype)
    E, W1, W2, Wr, h, sh = f(ew["E"]), f(ew["W1"]), f(ew["W2"]), f(li["W_r"]), f(li["h"]), f(li["shared"])
    out = np.zeros_like(h)
    for t in range(h.shape[0]):
        g = scipy.special.softmax(h[t] @ Wr)
        e = E[ids[t]]
        for j in range(W1.shape[0]):
            a = e @ W1[j]
            v = (0.5 * a * (1.0 + scipy.special.erf(a / np.sqrt(2.0)))) @ W2[j]
            out[t] += g[j] * wl.storage_to_f64(wl.to_storage(v, dtype), dtype)
        out[t] += sh[t]
    return out


@pytest.mark.parametrize("name,kw", [
    ("tiny", {}),                                                        # fp32, plain kernels
    ("decode410m", dict(V=600, d=256, D=512, N=16, T=100, L=1)),         # bf16: MFMA build + streaming forward
    ("decode410m", dict(V=300, d=2048, D=256, N=4, T=40, L=1)),          # 1B-4E row shape (d=2048, N=4)
    ("decode410m", dict(V=300, d=128, D=256, N=2, T=40, L=1)),           # N=2 (expert-count ablation)
    ("decode410m", dict(V=300, d=128, D=256, N=8, T=40, L=1)),
])
def test_built_table_reproduces_the_training_form_layer(name, kw):
    import torch
    w = wl.scaled(wl.CONFIGS[name], **kw)
    ew, li, ids = wl.expert_weights(w), wl.layer_inputs(w), wl.token_ids(w)
    dv = {k: to_dev(v, w.dtype) for k, v in ew.items()}
    lut = torch.empty((w.V, w.N, w.d), dtype=dv["E"].dtype, device="cuda")
    ws = torch.empty((mb.mole_build_lut_workspace(w.V, w.d, w.D, w.N, DT[w.dtype]),), dtype=torch.uint8, device="cuda")
    mb.mole_build_lut(dv["E"], dv["W1"], None, dv["W2"], None, None, 0.0, lut, w.V, w.d, w.D, w.N, DT[w.dtype],
                      mb.MOLE_GELU_ERF, ws)
    ids_d = torch.from_numpy(ids).cuda()
    h_d, wr_d, sh_d = (to_dev(li[k], w.dtype) for k in ("h", "W_r", "shared"))
    out_d = torch.empty_like(h_d)
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    mb.mole_lookup_forward(lut, ids_d, None, h_d, wr_d, sh_d, None, out_d, None, None, err_d, w.T, w.V, w.d, w.N,
                           DT[w.dtype])
    torch.cuda.synchronize()
    assert int(err_d.item()) == 0
    got = wl.storage_to_f64(to_host(out_d, w.dtype), w.dtype)
    ref = training_form_layer(ew, li, ids, w.dtype)
    tab = wl.to_storage(oracle.build_lut(ew["E"], ew["W1"], ew["W2"]), w.dtype)
    # one storage ulp of the largest looked-up entry on top of the forward tolerance: the device's entry
    # may be the neighbouring bf16 value of the reference's (fp32 against fp64 accumulation of the build)
    extra = 2.0 ** -8 * np.abs(wl.storage_to_f64(tab, w.dtype)[ids]).max() if w.dtype == wl.BF16 else 0.0
    assert_close(got, ref, w.dtype, f"end to end ({w.name} {kw})", extra_atol=extra)
    # the same through the oracle's two steps, with its table stored in the same type
    ref2, _, _, _ = oracle.lookup_forward(tab, ids, li["h"], li["W_r"], li["shared"])
    np.testing.assert_allclose(ref2, ref, rtol=1e-5 if w.dtype == wl.F32 else 1e-10, atol=1e-6 if w.dtype == wl.F32 else 1e-12)


def training_listing_layer(ew, x, ln_w, W_r, shared, ids, dtype, eps):
    """The MoLE part of the training listing from the post-attention state, numpy fp64, one token at a
    time: post-attention RMSNorm -> router softmax; RMSNorm of the embedding -> every expert FFN;
    residual + shared + gate-weighted sum.  One storage step is part of the reference because the
    output is a cancellation of terms of size ~10 and its rounding shows at atol 1e-3: expert outputs
    are rounded to the table's storage type (the table is a stored re-parameterization)."""
    f = lambda a: wl.storage_to_f64(a, dtype)
    E, W1, W2, nw = f(ew["E"]), f(ew["W1"]), f(ew["W2"]), f(ew["norm_w"])
    x, ln_w, W_r, shared = f(x), f(ln_w), f(W_r), f(shared)
    out = np.zeros_like(x)
    for t in range(x.shape[0]):
        g = scipy.special.softmax((x[t] / np.sqrt(np.mean(x[t] ** 2) + eps) * ln_w) @ W_r)
        e = E[ids[t]]
        e = e / np.sqrt(np.mean(e ** 2) + eps) * nw
        out[t] = x[t] + shared[t]
        for j in range(W1.shape[0]):
            a = e @ W1[j]
            v = (0.5 * a * (1.0 + scipy.special.erf(a / np.sqrt(2.0)))) @ W2[j]
            out[t] += g[j] * wl.storage_to_f64(wl.to_storage(v, dtype), dtype)
    return out


@pytest.mark.parametrize("name,kw", [
    ("tiny", {}),
    ("decode410m", dict(V=600, d=256, D=512, N=16, T=100, L=1)),
    ("decode1b_4e", dict(V=300, D=256, T=40, L=1)),                      # d = 2048, N = 4
    ("decode410m_n2", dict(V=300, d=128, D=256, T=40, L=1)),
])
def test_built_table_reproduces_the_training_listing_layer(name, kw):
    """Both norms of the listing in play: the embedding norm inside mole_build_lut, the post-attention norm
    and the residual inside mole_layer_forward."""
    import torch
    eps = 1e-5
    w = wl.scaled(wl.CONFIGS[name], **kw)
    ew, li, ni, ids = wl.expert_weights(w, norm=True), wl.layer_inputs(w), wl.norm_inputs(w), wl.token_ids(w)
    dv = {k: to_dev(v, w.dtype) for k, v in ew.items()}
    lut = torch.empty((w.V, w.N, w.d), dtype=dv["E"].dtype, device="cuda")
    ws = torch.empty((mb.mole_build_lut_workspace(w.V, w.d, w.D, w.N, DT[w.dtype]),), dtype=torch.uint8, device="cuda")
    mb.mole_build_lut(dv["E"], dv["W1"], None, dv["W2"], None, dv["norm_w"], eps, lut, w.V, w.d, w.D, w.N,
                      DT[w.dtype], mb.MOLE_GELU_ERF, ws)
    ids_d = torch.from_numpy(ids).cuda()
    x_d, lw_d, wr_d, sh_d = (to_dev(a, w.dtype) for a in (ni["x"], ni["ln_w"], li["W_r"], li["shared"]))
    out_d = torch.empty_like(x_d)
    err_d = torch.zeros((1,), dtype=torch.int32, device="cuda")
    mb.mole_layer_forward(lut, 0, ids_d, None, x_d, lw_d, eps, wr_d, sh_d, out_d, 0, None, None, err_d, 1, w.T, w.V, w.d,
                          w.N, DT[w.dtype])
    torch.cuda.synchronize()
    assert int(err_d.item()) == 0
    got = wl.storage_to_f64(to_host(out_d, w.dtype), w.dtype)
    ref = training_listing_layer(ew, ni["x"], ni["ln_w"], li["W_r"], li["shared"], ids, w.dtype, eps)
    tab = wl.to_storage(oracle.build_lut(ew["E"], ew["W1"], ew["W2"], norm_w=ew["norm_w"], norm_eps=eps), w.dtype)
    # The device builds its table with fp32 accumulation, so an entry can land on the neighbouring bf16
    # value (relative 2^-8); the gates sum to one, so the routed term moves by at most that fraction of the
    # largest looked-up entry.  Where residual, shared and routed terms cancel, only atol is left, hence
    # the explicit allowance.
    extra = 2.0 ** -8 * np.abs(wl.storage_to_f64(tab, w.dtype)[ids]).max() if w.dtype == wl.BF16 else 0.0
    assert_close(got, ref, w.dtype, f"listing layer end to end ({w.name} {kw})", extra_atol=extra)
    # and through the oracle's two steps, with its table stored in the same type
    s64 = lambda a: wl.storage_to_f64(a, w.dtype)
    ref2, *_ = oracle.layer_forward(tab, ids, s64(ni["x"]), s64(ni["ln_w"]), eps, s64(li["W_r"]), s64(li["shared"]))
    np.testing.assert_allclose(ref2, ref, rtol=1e-5 if w.dtype == wl.F32 else 1e-10,
                               atol=1e-5 if w.dtype == wl.F32 else 1e-11)


def test_plan_with_slot_and_staging():
    """MOLE_FLAG_DEDUP together with slot = inv on a staging buffer of the distinct rows."""
    import torch
    w = wl.scaled(wl.CONFIGS["decode410m"], V=3000, d=512, N=16, T=300, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    ids_d = torch.from_numpy(ids).cuda()
    uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(w.T, w.V) // 4,), dtype=torch.int32, device="cuda")
    mb.mole_dedup_ids(ids_d, w.T, w.V, uniq_d, inv_d, nu, err, plan)
    torch.cuda.synchronize()
    U = int(nu.item())
    staging = to_dev(table, w.dtype)[uniq_d[:U].long()].contiguous()
    h_d, wr_d, sh_d = (to_dev(li[k], w.dtype) for k in ("h", "W_r", "shared"))
    out_d = torch.empty_like(h_d)
    mb.mole_lookup_forward(staging, ids_d, inv_d, h_d, wr_d, sh_d, None, out_d, None, None, err, w.T, U, w.d, w.N,
                           DT[w.dtype], mb.MOLE_FLAG_DEDUP, plan)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    ref, _, _, _ = oracle.lookup_forward(table, ids, li["h"], li["W_r"], li["shared"])
    assert_close(wl.storage_to_f64(to_host(out_d, w.dtype), w.dtype), ref, w.dtype, "plan + slot")


@pytest.mark.parametrize("N", [16, 5])
def test_foreign_plan_is_flagged_and_ignored(N):
    """A workspace that mole_dedup_ids did not write for this T sets bit 1 of err_flag; the tokens are then
    visited in their own order and the output is the one of the call without the flag (here, with an id
    outside the table as well, both bits are reported)."""
    import torch
    w = wl.scaled(wl.CONFIGS["decode410m"], V=500, d=256, N=N, T=64, L=1)
    table, li, ids = wl.random_table(w), wl.layer_inputs(w), wl.token_ids(w)
    for bad_id, flags_want in ((False, 2), (True, 3)):
        ids = ids.copy()
        if bad_id:
            ids[5] = w.V
        ids_d = torch.from_numpy(ids).cuda()
        h_d, wr_d = to_dev(li["h"], w.dtype), to_dev(li["W_r"], w.dtype)
        out_d = torch.full_like(h_d, 7.0)
        err = torch.zeros((1,), dtype=torch.int32, device="cuda")
        junk = torch.zeros((mb.mole_dedup_workspace(w.T, w.V) // 4,), dtype=torch.int32, device="cuda")
        for runs in (0, mb.MOLE_FLAG_RUNS):
            err.zero_()
            mb.mole_lookup_forward(to_dev(table, w.dtype), ids_d, None, h_d, wr_d, None, None, out_d, None, None, err,
                                   w.T, w.V, w.d, w.N, DT[w.dtype], mb.MOLE_FLAG_DEDUP | runs, junk)
            torch.cuda.synchronize()
            assert int(err.item()) == flags_want
            ref, _, _, _ = oracle.lookup_forward(table, ids, li["h"], li["W_r"])
            assert_close(wl.storage_to_f64(to_host(out_d, w.dtype), w.dtype), ref, w.dtype, "foreign plan ignored")


@pytest.mark.parametrize("N,T", [(16, 96), (32, 5000)])
def test_hip_graph_replay_matches_eager(N, T):
    """Capture dedup + forward (two layers, per-layer launches) in a HIP graph; every replay, with eager
    work and synchronisation in between, must equal the eager result.  (16, 96): the one-workgroup dedup and the
    streaming kernel; (32, 5000): the eight-workgroup dedup and the tile kernel."""
    import torch
    w = wl.scaled(wl.CONFIGS["decode410m"], V=2000, d=1024, N=N, T=T, L=2)
    tabs = [to_dev(wl.random_table(w, l), w.dtype) for l in range(w.L)]
    lis = [wl.layer_inputs(w, l) for l in range(w.L)]
    hs = [to_dev(li["h"], w.dtype) for li in lis]
    wrs = [to_dev(li["W_r"], w.dtype) for li in lis]
    shs = [to_dev(li["shared"], w.dtype) for li in lis]
    ids_d = torch.from_numpy(wl.token_ids(w)).cuda()
    uniq_d, inv_d = torch.empty_like(ids_d), torch.empty_like(ids_d)
    nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(w.T, w.V) // 4,), dtype=torch.int32, device="cuda")
    outs = [torch.zeros_like(h) for h in hs]
    s = torch.cuda.Stream()

    def step():
        mb.mole_dedup_ids(ids_d, w.T, w.V, uniq_d, inv_d, nu, err, plan, stream=s)
        for l in range(w.L):
            mb.mole_lookup_forward(tabs[l], ids_d, None, hs[l], wrs[l], shs[l], None, outs[l], None, None, err,
                                   w.T, w.V, w.d, w.N, DT[w.dtype], mb.MOLE_FLAG_DEDUP, plan, stream=s)
    with torch.cuda.stream(s):
        step()
    s.synchronize()
    eager = [o.clone() for o in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            step()
    for rep in range(4):
        for o in outs:
            o.zero_()                                  # eager work between replays
        ids_new = torch.from_numpy(wl.token_ids(w, batch=rep)).cuda()
        ids_d.copy_(ids_new)                           # the graph reads whatever the buffers hold now
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        with torch.cuda.stream(s):
            ref_outs = [torch.zeros_like(o) for o in outs]
            mb.mole_dedup_ids(ids_d, w.T, w.V, uniq_d, inv_d, nu, err, plan, stream=s)
            for l in range(w.L):
                mb.mole_lookup_forward(tabs[l], ids_d, None, hs[l], wrs[l], shs[l], None, ref_outs[l], None, None,
                                       err, w.T, w.V, w.d, w.N, DT[w.dtype], mb.MOLE_FLAG_DEDUP, plan, stream=s)
        s.synchronize()
        for o, r in zip(outs, ref_outs):
            assert torch.equal(o.view(torch.int16), r.view(torch.int16)), f"replay {rep}"
    assert int(err.item()) == 0
    assert torch.equal(eager[0].view(torch.int16), eager[0].view(torch.int16))
