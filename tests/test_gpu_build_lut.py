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
@pytest.mark.parametrize("hidden", [None, "f16", "split"])
def test_bf16_build(monkeypatch, V, d, D, N, bias, norm, act, hidden):
    """hidden: the format the hidden activation is carried in -- chosen by the library (fp16 here, the
    values are small) or forced to either variant."""
    if hidden:
        monkeypatch.setenv("MOLE_BUILD_HIDDEN", hidden)
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, D=D, N=N)
    ew = wl.expert_weights(w, bias=bias, norm=norm)
    got = run_build(w, ew, act=act)
    ref = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], b1=ew["b1"], b2=ew["b2"], norm_w=ew["norm_w"],
                           act=oracle.GELU_TANH if act == mb.MOLE_GELU_TANH else oracle.GELU_ERF)
    assert_close(wl.storage_to_f64(got, w.dtype), ref, w.dtype, "bf16 LUT")
    assert np.abs(ref).mean() > 1e-3


def test_bf16_build_beyond_the_fp16_range():
    """Pre-activations of size ~1e4..1e5: many hidden activations exceed 65504, so an fp16 hidden plane
    would saturate.  The library must notice (its bound exceeds the limit) and carry hi + lo planes.
    Outputs here are sums of D products of size ~1e3 that partly cancel, so the comparison allows, per
    element, the error the hi + lo pair (2^-17 per value) and the fp32 accumulation (2^-24 per add) can
    leave: 2^-15 * sum_m |hidden_m * W2_m| is a generous bound for both.  Saturation would show as errors
    of order (|hidden| - 65504) * |W2|, hundreds of times larger."""
    import scipy.special
    w = wl.scaled(wl.CONFIGS["offload410m"], V=300, d=128, D=256, N=2)
    ew = wl.expert_weights(w, bias=True)
    f = lambda a: wl.storage_to_f64(a, w.dtype)
    ew["E"] = wl.to_storage(f(ew["E"]) * 6000.0, w.dtype)
    ew["W1"] = wl.to_storage(f(ew["W1"]) * 25.0, w.dtype)
    ref = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], b1=ew["b1"], b2=ew["b2"])
    pre = np.einsum("vk,jkm->vjm", f(ew["E"]), f(ew["W1"])) + f(ew["b1"])[None]
    assert (np.abs(pre) > 65504).mean() > 0.01               # the case really leaves the fp16 range
    hid = 0.5 * pre * (1.0 + scipy.special.erf(pre / np.sqrt(2.0)))
    allowance = 2.0 ** -15 * np.einsum("vjm,jmc->vjc", np.abs(hid), np.abs(f(ew["W2"])))
    clipped = np.einsum("vjm,jmc->vjc", np.clip(hid, -65504, 65504), f(ew["W2"])) + f(ew["b2"])[None]
    assert (np.abs(clipped - ref) > 100 * allowance + 1e-3 + 2e-2 * np.abs(ref)).any()   # saturation would be seen
    got = run_build(w, ew)
    assert_close(wl.storage_to_f64(got, w.dtype), ref, w.dtype, "bf16 LUT, large activations", extra_atol=allowance)
