"""GPU parity of mole_build_lut against the fp64 oracle (itself pinned to numpy/scipy and to closed forms)."""
import numpy as np
import pytest

import oracle
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl
from helpers import DT, assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu


def run_build(w, ew, act=mb.MOLE_GELU_ERF, eps=1e-5):
    import torch
    dv = {k: to_dev(v, w.dtype) for k, v in ew.items()}
    lut = torch.full((w.V, w.N, w.d), float("nan"), dtype=dv["E"].dtype, device="cuda")
    ws_bytes = mb.mole_build_lut_workspace(w.V, w.d, w.D, w.N, DT[w.dtype])
    assert ws_bytes > 0
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
    mb.mole_build_lut(dv["E"], dv["W1"], dv["b1"], dv["W2"], dv["b2"], dv["norm_w"], eps, lut, w.V, w.d, w.D, w.N,
                      DT[w.dtype], act, ws)
    torch.cuda.synchronize()
    return to_host(lut, w.dtype)


def test_tiny_fp32_full_table():
    w = wl.CONFIGS["tiny"]
    ew = wl.expert_weights(w)
    got = run_build(w, ew)
    ref = oracle.build_lut(ew["E"], ew["W1"], ew["W2"])
    assert_close(got.astype(np.float64), ref, wl.F32, "tiny LUT")


@pytest.mark.parametrize("bias,norm,act", [(True, False, mb.MOLE_GELU_ERF), (True, True, mb.MOLE_GELU_TANH),
                                           (False, True, mb.MOLE_GELU_ERF)])
def test_fp32_options(bias, norm, act):
    w = wl.scaled(wl.CONFIGS["tiny"], V=300, d=48, D=80, N=3)
    ew = wl.expert_weights(w, bias=bias, norm=norm)
    got = run_build(w, ew, act=act)
    ref = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], b1=ew["b1"], b2=ew["b2"], norm_w=ew["norm_w"],
                           act=oracle.GELU_TANH if act == mb.MOLE_GELU_TANH else oracle.GELU_ERF)
    assert_close(got.astype(np.float64), ref, wl.F32, "fp32 LUT with options")


@pytest.mark.parametrize("V,d,D,N,bias,norm,act", [
    (700, 256, 512, 3, False, False, mb.MOLE_GELU_ERF),     # MFMA tiles, ragged last row tile
    (257, 128, 384, 2, True, False, mb.MOLE_GELU_TANH),
    (300, 256, 256, 2, True, True, mb.MOLE_GELU_ERF),       # RMSNorm first (hi/lo input planes)
    (100, 48, 80, 3, True, False, mb.MOLE_GELU_ERF),        # shape outside the MFMA tiles: plain path
])
def test_bf16_build(V, d, D, N, bias, norm, act):
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, D=D, N=N)
    ew = wl.expert_weights(w, bias=bias, norm=norm)
    got = run_build(w, ew, act=act)
    ref = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], b1=ew["b1"], b2=ew["b2"], norm_w=ew["norm_w"],
                           act=oracle.GELU_TANH if act == mb.MOLE_GELU_TANH else oracle.GELU_ERF)
    assert_close(wl.storage_to_f64(got, w.dtype), ref, w.dtype, "bf16 LUT")
    assert np.abs(ref).mean() > 1e-3


def test_bf16_build_closed_forms():
    w = wl.scaled(wl.CONFIGS["offload410m"], V=300, d=128, D=256, N=2)
    ew = wl.expert_weights(w, bias=True)
    ew0 = dict(ew, W2=np.zeros_like(ew["W2"]))
    got = run_build(w, ew0)                       # second matrix zero -> the output bias everywhere
    np.testing.assert_array_equal(got, np.broadcast_to(ew["b2"][None], got.shape))
    ew1 = dict(ew, W1=np.zeros_like(ew["W1"]), b1=None)
    got = run_build(w, ew1)                       # GELU(0) = 0 -> the output bias again
    np.testing.assert_array_equal(got, np.broadcast_to(ew["b2"][None], got.shape))


def test_410m_layer_sampled_rows():
    """One full 410M layer (V=50304, d=1024, D=4096, N=16, bf16) built on the GPU; 96 seeded-random
    vocabulary rows x all experts against the fp64 oracle (the whole table is 1.35e13 flop: too slow
    on the host)."""
    import torch
    w = wl.CONFIGS["offload410m"]
    g = torch.Generator(device="cuda")
    g.manual_seed(55)
    E = torch.randn((w.V, w.d), generator=g, device="cuda").to(torch.bfloat16)
    W1 = (torch.randn((w.N, w.d, w.D), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    W2 = (torch.randn((w.N, w.D, w.d), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    lut = torch.full((w.V, w.N, w.d), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty((mb.mole_build_lut_workspace(w.V, w.d, w.D, w.N, mb.MOLE_BF16),), dtype=torch.uint8, device="cuda")
    mb.mole_build_lut(E, W1, None, W2, None, None, 0.0, lut, w.V, w.d, w.D, w.N, mb.MOLE_BF16, mb.MOLE_GELU_ERF, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(lut.float()).any()
    rows = np.unique(np.concatenate([np.random.default_rng(8).integers(0, w.V, 92), [0, 255, 256, w.V - 1]]))
    rows_t = torch.from_numpy(rows.astype(np.int64)).cuda()
    got = to_host(lut[rows_t], wl.BF16)
    ref = oracle.build_lut(to_host(E[rows_t], wl.BF16), to_host(W1, wl.BF16), to_host(W2, wl.BF16))
    assert_close(wl.storage_to_f64(got, wl.BF16), ref, wl.BF16, "410M LUT sample")
