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
def test_bf16_build(tuning, V, d, D, N, bias, norm, act, hidden):
    """hidden: the format the hidden activation is carried in -- chosen by the library (fp16 here, the
    values are small) or forced to either variant."""
    if hidden:
        tuning("MOLE_BUILD_HIDDEN", {"f16": 1, "split": 2}[hidden])
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, D=D, N=N)
    ew = wl.expert_weights(w, bias=bias, norm=norm)
    got = run_build(w, ew, act=act)
    ref = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], b1=ew["b1"], b2=ew["b2"], norm_w=ew["norm_w"],
                           act=oracle.GELU_TANH if act == mb.MOLE_GELU_TANH else oracle.GELU_ERF)
    assert_close(wl.storage_to_f64(got, w.dtype), ref, w.dtype, "bf16 LUT")
    assert np.abs(ref).mean() > 1e-3


@pytest.mark.parametrize("seed", range(10))
def test_seeded_random_shapes(tuning, seed):
    """V, d, D, N, biases, norm, activation and the hidden format drawn at random: MFMA path (both tile
    sizes, ragged row tiles) and plain path against the oracle."""
    rng = np.random.default_rng(5000 + seed)
    d = int(rng.choice([48, 64, 128, 192, 256, 320, 512]))
    D = int(rng.choice([80, 128, 256, 384, 512, 768]))
    N = int(rng.integers(1, 5))
    V = int(rng.integers(1, 900))
    bias, norm = bool(rng.integers(2)), bool(rng.integers(2))
    act = mb.MOLE_GELU_TANH if rng.integers(2) else mb.MOLE_GELU_ERF
    hidden = rng.choice(["", "f16", "split"])
    if hidden:
        tuning("MOLE_BUILD_HIDDEN", {"f16": 1, "split": 2}[str(hidden)])
    if rng.integers(2):
        tuning("MOLE_BUILD_SMALL_TILE", "1")
    w = wl.scaled(wl.CONFIGS["offload410m"], V=V, d=d, D=D, N=N, name=f"build random seed {seed}: V{V} d{d} D{D} N{N}")
    ew = wl.expert_weights(w, bias=bias, norm=norm)
    got = run_build(w, ew, act=act)
    ref = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], b1=ew["b1"], b2=ew["b2"], norm_w=ew["norm_w"],
                           act=oracle.GELU_TANH if act == mb.MOLE_GELU_TANH else oracle.GELU_ERF)
    assert_close(wl.storage_to_f64(got, w.dtype), ref, w.dtype, f"LUT ({w.name})")


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
    """One full 410M layer (V=50304, d=1024, D=4096, N=16, bf16) built on the GPU; 512 seeded-random
    vocabulary rows (plus tile-boundary rows) x all experts against the fp64 oracle (the whole table is
    1.35e13 flop: too slow on the host)."""
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
    rows = np.unique(np.concatenate([np.random.default_rng(8).integers(0, w.V, 506),
                                     [0, 255, 256, 16383, 16384, w.V - 1]]))
    rows_t = torch.from_numpy(rows.astype(np.int64)).cuda()
    got = to_host(lut[rows_t], wl.BF16)
    ref = oracle.build_lut(to_host(E[rows_t], wl.BF16), to_host(W1, wl.BF16), to_host(W2, wl.BF16))
    assert_close(wl.storage_to_f64(got, wl.BF16), ref, wl.BF16, "410M LUT sample")
