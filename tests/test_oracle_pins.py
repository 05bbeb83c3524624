"""Pins for the fp64 CPU oracle: every check compares it with something other than itself --
the training-form layer evaluated by brute force, closed forms, invariants, special cases that
reduce to library routines (numpy / scipy / torch CPU / math).  No GPU, no HIP library.
"""
import math

import numpy as np
import pytest
import scipy.special

import oracle
from paper_2503_15798_amd import workloads as wl


# --------------------------------------------------------------------------------------------
# independent numpy helpers (none of them is used by the oracle)
# --------------------------------------------------------------------------------------------
def np_gelu_erf(x):
    return 0.5 * x * (1.0 + scipy.special.erf(x / np.sqrt(2.0)))


def np_softmax(z):
    return scipy.special.softmax(z, axis=-1)


def brute_force_training_layer(E, W1, W2, W_r, h, ids, shared, b1=None, b2=None):
    """Training-phase layer (Sec. 3.2): run every expert FFN on the token's embedding and combine
    with the full-softmax gates.  Pure numpy fp64, one token at a time."""
    T, d = h.shape
    N = W1.shape[0]
    out = np.zeros((T, d))
    for t in range(T):
        e = E[ids[t]]
        g = np_softmax(h[t] @ W_r)
        acc = np.zeros(d)
        for j in range(N):
            a = e @ W1[j]
            if b1 is not None:
                a = a + b1[j]
            v = np_gelu_erf(a) @ W2[j]
            if b2 is not None:
                v = v + b2[j]
            acc += g[j] * v
        out[t] = acc + shared[t]
    return out


def tiny_case(dtype=wl.F32, bias=False, T=None):
    w = wl.CONFIGS["tiny"]
    if dtype != wl.F32:
        w = wl.scaled(w, dtype=dtype)
    ew = wl.expert_weights(w, bias=bias)
    li = wl.layer_inputs(w, T=T)
    ids = wl.token_ids(w, T=T)
    return w, ew, li, ids


# --------------------------------------------------------------------------------------------
# whole path: lookup form == training form (the re-parameterization is exact)
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bias", [False, True])
def test_lookup_equals_running_every_expert(bias):
    w, ew, li, ids = tiny_case(bias=bias)
    lut = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], b1=ew["b1"], b2=ew["b2"])
    assert lut.shape == (w.V, w.N, w.d)
    out, g, rows, err = oracle.lookup_forward(lut, ids, li["h"].astype(np.float64),
                                              li["W_r"].astype(np.float64),
                                              shared=li["shared"].astype(np.float64))
    f = lambda a: None if a is None else a.astype(np.float64)
    ref = brute_force_training_layer(f(ew["E"]), f(ew["W1"]), f(ew["W2"]), f(li["W_r"]), f(li["h"]),
                                     ids, f(li["shared"]), f(ew["b1"]), f(ew["b2"]))
    assert err == 0
    np.testing.assert_array_equal(rows, ids.astype(np.int64))
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-12)
    # the routed term alone is ~0.02 in size; check it is not hidden under the shared term
    routed = out - li["shared"].astype(np.float64)
    assert np.abs(routed).mean() > 1e-3


def test_forward_matches_torch_einsum():
    torch = pytest.importorskip("torch")
    w = wl.scaled(wl.CONFIGS["tiny"], V=97, d=24, N=5, T=33)   # d != N != T: a transposed operand fails
    tab = wl.random_table(w).astype(np.float64)
    li = {k: v.astype(np.float64) for k, v in wl.layer_inputs(w).items()}
    ids = wl.token_ids(w)
    out, g, rows, err = oracle.lookup_forward(tab, ids, li["h"], li["W_r"], li["shared"], li["residual"])
    tt = torch.from_numpy
    gt = torch.softmax(tt(li["h"]) @ tt(li["W_r"]), dim=-1)
    ref = torch.einsum("tn,tnd->td", gt, tt(tab)[tt(ids.astype(np.int64))]) + tt(li["shared"]) + tt(li["residual"])
    np.testing.assert_allclose(g, gt.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------------------------
# router + softmax
# --------------------------------------------------------------------------------------------
def test_gates_are_a_distribution_and_match_scipy():
    w = wl.scaled(wl.CONFIGS["tiny"], d=40, N=7, T=19)
    li = wl.layer_inputs(w)
    g = oracle.gates(li["h"], li["W_r"] * np.float32(20.0))
    assert g.shape == (19, 7)
    assert (g > 0).all()
    np.testing.assert_allclose(g.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    ref = np_softmax(li["h"].astype(np.float64) @ (li["W_r"] * np.float32(20.0)).astype(np.float64))
    np.testing.assert_allclose(g, ref, rtol=1e-12, atol=1e-16)
    assert np.abs(g - 1.0 / 7).max() > 0.05      # the case is not degenerate


def test_zero_router_gives_mean_of_rows():
    w = wl.scaled(wl.CONFIGS["tiny"], V=50, d=16, N=6, T=21)
    tab = wl.random_table(w).astype(np.float64)
    li = wl.layer_inputs(w)
    ids = wl.token_ids(w)
    Wr0 = np.zeros((w.d, w.N))
    out, g, _, _ = oracle.lookup_forward(tab, ids, li["h"].astype(np.float64), Wr0,
                                         shared=li["shared"].astype(np.float64))
    np.testing.assert_allclose(g, 1.0 / w.N, rtol=0, atol=1e-16)
    np.testing.assert_allclose(out, tab[ids].mean(axis=1) + li["shared"], rtol=1e-13, atol=1e-15)


def test_softmax_shift_invariance():
    """Adding one vector to every router column shifts all logits of a token equally."""
    w = wl.scaled(wl.CONFIGS["tiny"], d=32, N=5, T=17)
    li = wl.layer_inputs(w)
    h = li["h"].astype(np.float64)
    Wr = li["W_r"].astype(np.float64) * 30.0
    c = np.random.default_rng(5).standard_normal((w.d, 1))
    np.testing.assert_allclose(oracle.gates(h, Wr + c), oracle.gates(h, Wr), rtol=1e-9, atol=1e-14)


def test_large_logits_do_not_overflow():
    h = np.full((2, 4), 100.0)
    Wr = np.array([[3.0, 0.0, -3.0]] * 4)          # logits 1200, 0, -1200
    g = oracle.gates(h, Wr)
    assert np.isfinite(g).all()
    np.testing.assert_allclose(g, [[1.0, 0.0, 0.0]] * 2, atol=1e-300)


# --------------------------------------------------------------------------------------------
# gather
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_single_expert_is_a_plain_row_gather(dtype):
    w = wl.scaled(wl.CONFIGS["tiny"], V=200, d=24, N=1, T=64, dtype=dtype)
    tab = wl.random_table(w)
    li = wl.layer_inputs(w)
    ids = wl.token_ids(w)
    out, g, rows, err = oracle.lookup_forward(tab, ids, li["h"], li["W_r"])
    np.testing.assert_array_equal(g, np.ones((64, 1)))
    np.testing.assert_array_equal(out, wl.storage_to_f64(tab, dtype)[ids, 0, :])     # exact
    np.testing.assert_array_equal(rows, ids)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_saturated_router_returns_one_experts_row_exactly(dtype):
    w = wl.scaled(wl.CONFIGS["tiny"], V=300, d=16, N=4, T=16, dtype=dtype)
    tab = wl.random_table(w)
    ids = wl.token_ids(w)
    h = np.zeros((w.T, w.d), dtype=np.float32)
    star = np.arange(w.T) % w.N                      # expert chosen by token t
    kk = np.arange(w.T) % w.d                        # h[t] = unit vector e_kk
    h[np.arange(w.T), kk] = 1.0
    Wr = np.zeros((w.d, w.N), dtype=np.float32)
    for t in range(w.T):
        Wr[kk[t], star[t]] = 1.0e4                   # k and star advance together (16 % 4 == 0)
    out, g, _, _ = oracle.lookup_forward(tab, ids, wl.to_storage(h, dtype), wl.to_storage(Wr, dtype))
    onehot = np.zeros((w.T, w.N))
    onehot[np.arange(w.T), star] = 1.0
    np.testing.assert_array_equal(g, onehot)
    np.testing.assert_array_equal(out, wl.storage_to_f64(tab, dtype)[ids, star, :])


def test_row_index_uses_all_three_axes():
    """table[v,j,c] = 10000 v + 100 j + c makes any index slip (v<->j, stride N vs d) visible."""
    V, N, d, T = 13, 3, 7, 13
    tab = (10000.0 * np.arange(V)[:, None, None] + 100.0 * np.arange(N)[None, :, None]
           + np.arange(d)[None, None, :])
    ids = np.arange(T, dtype=np.int32)[::-1].copy()
    h = np.zeros((T, d))
    h[:, 0] = 1.0
    Wr = np.zeros((d, N))
    Wr[0, 2] = 5000.0
    out, g, rows, _ = oracle.lookup_forward(tab, ids, h, Wr)
    np.testing.assert_array_equal(out, tab[ids, 2, :])


def test_out_of_range_ids_give_zero_routed_term_and_flag():
    w = wl.scaled(wl.CONFIGS["tiny"], V=40, d=8, N=3, T=6)
    tab = wl.random_table(w)
    li = wl.layer_inputs(w)
    ids = np.array([0, 39, 40, -1, 5, 2**31 - 1], dtype=np.int32)
    out, g, rows, err = oracle.lookup_forward(tab, ids, li["h"], li["W_r"], shared=li["shared"])
    assert err == 1
    np.testing.assert_array_equal(rows, [0, 39, -1, -1, 5, -1])
    bad = np.array([2, 3, 5])
    np.testing.assert_array_equal(out[bad], li["shared"].astype(np.float64)[bad])
    good = np.array([0, 1, 4])
    assert (out[good] != li["shared"].astype(np.float64)[good]).any()


# --------------------------------------------------------------------------------------------
# combine / add
# --------------------------------------------------------------------------------------------
def test_linearity_and_optional_terms():
    w = wl.scaled(wl.CONFIGS["tiny"], V=64, d=12, N=4, T=20)
    tab = wl.random_table(w).astype(np.float64)
    li = {k: v.astype(np.float64) for k, v in wl.layer_inputs(w).items()}
    ids = wl.token_ids(w)
    Wr = li["W_r"] * 25.0
    routed, *_ = oracle.lookup_forward(tab, ids, li["h"], Wr)
    with_shared, *_ = oracle.lookup_forward(tab, ids, li["h"], Wr, shared=li["shared"])
    with_both, *_ = oracle.lookup_forward(tab, ids, li["h"], Wr, shared=li["shared"], residual=li["residual"])
    doubled, *_ = oracle.lookup_forward(2.0 * tab, ids, li["h"], Wr, shared=li["shared"])
    np.testing.assert_allclose(with_shared - routed, li["shared"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(with_both - with_shared, li["residual"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(doubled - li["shared"], 2.0 * routed, rtol=1e-13, atol=1e-15)
    # independent value of the routed term
    ref = np.einsum("tn,tnd->td", np_softmax(li["h"] @ Wr), tab[ids])
    np.testing.assert_allclose(routed, ref, rtol=1e-12, atol=1e-15)


def test_bf16_storage_is_widened_exactly():
    w = wl.scaled(wl.CONFIGS["tiny"], V=64, d=16, N=4, T=20, dtype=wl.BF16)
    tab = wl.random_table(w)
    li = wl.layer_inputs(w)
    ids = wl.token_ids(w)
    a, ga, *_ = oracle.lookup_forward(tab, ids, li["h"], li["W_r"], li["shared"], li["residual"])
    f = lambda x: wl.storage_to_f64(x, wl.BF16)
    b, gb, *_ = oracle.lookup_forward(f(tab), ids, f(li["h"]), f(li["W_r"]), f(li["shared"]), f(li["residual"]))
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(ga, gb)
    # and the bf16 helpers themselves: round-to-nearest-even on known patterns
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7 + 2 ** -8, -0.0, 3.140625], dtype=np.float32)
    bits = wl.f32_to_bf16_bits(x)
    np.testing.assert_array_equal(bits, [0x3F80, 0x3F80, 0x3F82, 0x8000, 0x4049])
    np.testing.assert_array_equal(wl.bf16_bits_to_f32(bits), np.array([1.0, 1.0, 1.015625, -0.0, 3.140625], np.float32))


# --------------------------------------------------------------------------------------------
# dedup
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("T,V,dist", [(1, 10, "uniform"), (256, 1024, "uniform"), (4096, 50304, "zipf"),
                                      (333, 7, "uniform")])
def test_dedup_matches_numpy_unique(T, V, dist):
    ids = wl.make_ids(T, V, seed=T + V, dist=dist)
    uniq, inv, U, err = oracle.dedup(ids, V)
    ru, rinv = np.unique(ids, return_inverse=True)
    assert err == 0 and U == len(ru)
    np.testing.assert_array_equal(uniq, ru)
    np.testing.assert_array_equal(inv, rinv)
    assert (np.diff(uniq) > 0).all()
    np.testing.assert_array_equal(uniq[inv], ids)
    assert U <= min(T, V)


def test_dedup_edge_cases():
    uniq, inv, U, err = oracle.dedup(np.zeros((0,), np.int32), 5)
    assert U == 0 and err == 0 and len(inv) == 0
    uniq, inv, U, err = oracle.dedup(np.array([4, 4, 4, 4], np.int32), 5)
    assert U == 1 and list(uniq) == [4] and list(inv) == [0, 0, 0, 0]
    uniq, inv, U, err = oracle.dedup(np.array([3, 7, -2, 3], np.int32), 5)
    assert err == 1 and list(uniq) == [3] and list(inv) == [0, -1, -1, 0]


# --------------------------------------------------------------------------------------------
# LUT build
# --------------------------------------------------------------------------------------------
def test_gelu_against_math_erf_and_known_values():
    for x in [-6.0, -1.5, -0.3, 0.0, 1e-3, 0.7, 2.0, 9.0]:
        assert oracle.gelu(x) == pytest.approx(0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0))), rel=1e-15, abs=1e-300)
        tanh_ref = 0.5 * x * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))
        assert oracle.gelu(x, oracle.GELU_TANH) == pytest.approx(tanh_ref, rel=1e-14, abs=1e-300)
    assert oracle.gelu(0.0) == 0.0
    assert oracle.gelu(1.0) == pytest.approx(0.8413447460685429, rel=1e-14)      # Phi(1)
    assert oracle.gelu(-1.0) == pytest.approx(-0.15865525393145707, rel=1e-13)   # -Phi(-1)
    assert abs(oracle.gelu(1.0) - oracle.gelu(1.0, oracle.GELU_TANH)) > 1e-5     # the two forms differ


def test_build_lut_matches_numpy_matmul_and_layout():
    w = wl.scaled(wl.CONFIGS["tiny"], V=37, d=12, D=20, N=3)     # all sizes distinct
    ew = {k: (None if v is None else v.astype(np.float64)) for k, v in wl.expert_weights(w, bias=True).items()}
    lut = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], b1=ew["b1"], b2=ew["b2"])
    assert lut.shape == (37, 3, 12)
    for j in range(w.N):
        ref = np_gelu_erf(ew["E"] @ ew["W1"][j] + ew["b1"][j]) @ ew["W2"][j] + ew["b2"][j]
        np.testing.assert_allclose(lut[:, j, :], ref, rtol=1e-12, atol=1e-15)
    # tanh form and a row subset
    sub = np.array([36, 0, 5, 5], dtype=np.int32)
    lut_t = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], act=oracle.GELU_TANH, rows=sub)
    a = ew["E"][sub] @ ew["W1"][1]
    ref = (0.5 * a * (1 + np.tanh(np.sqrt(2 / np.pi) * (a + 0.044715 * a ** 3)))) @ ew["W2"][1]
    np.testing.assert_allclose(lut_t[:, 1, :], ref, rtol=1e-12, atol=1e-15)


def test_build_lut_closed_forms():
    w = wl.scaled(wl.CONFIGS["tiny"], V=9, d=8, D=16, N=2)
    ew = {k: (None if v is None else v.astype(np.float64)) for k, v in wl.expert_weights(w, bias=True).items()}
    # second matrix zero -> every entry is the output bias
    lut = oracle.build_lut(ew["E"], ew["W1"], np.zeros_like(ew["W2"]), b1=ew["b1"], b2=ew["b2"])
    np.testing.assert_array_equal(lut, np.broadcast_to(ew["b2"][None], lut.shape))
    # first matrix and bias zero -> GELU(0) = 0 -> again the output bias
    lut = oracle.build_lut(ew["E"], np.zeros_like(ew["W1"]), ew["W2"], b1=None, b2=ew["b2"])
    np.testing.assert_array_equal(lut, np.broadcast_to(ew["b2"][None], lut.shape))
    # no biases, zero embedding row -> zero entry
    E0 = ew["E"].copy()
    E0[4] = 0.0
    lut = oracle.build_lut(E0, ew["W1"], ew["W2"])
    assert (lut[4] == 0.0).all() and (lut[3] != 0.0).any()


def test_build_lut_optional_rmsnorm():
    w = wl.scaled(wl.CONFIGS["tiny"], V=11, d=10, D=14, N=2)
    ew = {k: (None if v is None else v.astype(np.float64)) for k, v in wl.expert_weights(w, norm=True).items()}
    eps = 1e-5
    lut = oracle.build_lut(ew["E"], ew["W1"], ew["W2"], norm_w=ew["norm_w"], norm_eps=eps)
    x = ew["E"] / np.sqrt((ew["E"] ** 2).mean(axis=1, keepdims=True) + eps) * ew["norm_w"]
    for j in range(w.N):
        np.testing.assert_allclose(lut[:, j, :], np_gelu_erf(x @ ew["W1"][j]) @ ew["W2"][j], rtol=1e-12, atol=1e-15)
    plain = oracle.build_lut(ew["E"], ew["W1"], ew["W2"])
    assert np.abs(plain - lut).max() > 1e-4


# --------------------------------------------------------------------------------------------
# a planted mistake must be caught: the same checks fail on deliberately wrong variants
# (the variants live here, on the CPU, as numpy code)
# --------------------------------------------------------------------------------------------
# --------------------------------------------------------------------------------------------
# the layer from the post-attention state (inference listing): norm -> router -> lookup -> adds
# --------------------------------------------------------------------------------------------
def fused_case(dtype=np.float64, T=29, V=83, d=40, N=6, seed=3):
    rng = np.random.default_rng(seed)
    tab = rng.standard_normal((V, N, d))
    x = rng.standard_normal((T, d)) * 3.0 + 0.5
    ln_w = rng.uniform(0.5, 1.5, size=d)
    W_r = rng.standard_normal((d, N)) * 0.4
    shared = rng.standard_normal((T, d))
    ids = rng.integers(0, V, size=T).astype(np.int32)
    return tab, ids, x, ln_w, W_r, shared


def test_layer_forward_matches_torch_rmsnorm_softmax_einsum():
    """Independent evaluation with torch CPU ops in fp64, in the order of the inference listing."""
    import torch
    tab, ids, x, ln_w, W_r, shared = fused_case()
    eps = 1e-5
    out, g, hn, rows, err = oracle.layer_forward(tab, ids, x, ln_w, eps, W_r, shared)
    xt = torch.from_numpy(x)
    hn_t = xt * torch.rsqrt(xt.pow(2).mean(-1, keepdim=True) + eps) * torch.from_numpy(ln_w)
    g_t = torch.softmax(hn_t @ torch.from_numpy(W_r), dim=-1)
    looked = torch.from_numpy(tab)[torch.from_numpy(ids).long()]                   # [T,N,d]
    out_t = xt + torch.from_numpy(shared) + (looked * g_t.unsqueeze(-1)).sum(dim=1)
    assert err == 0 and np.array_equal(rows, ids)
    np.testing.assert_allclose(hn, hn_t.numpy(), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(g, g_t.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(out, out_t.numpy(), rtol=1e-12, atol=1e-13)


def test_layer_forward_is_the_pinned_forward_after_a_numpy_norm():
    tab, ids, x, ln_w, W_r, shared = fused_case(seed=8)
    eps = 1e-6
    out, g, hn, _, _ = oracle.layer_forward(tab, ids, x, ln_w, eps, W_r, shared)
    hn_np = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + eps) * ln_w
    ref, g_ref, _, _ = oracle.lookup_forward(tab, ids, hn_np, W_r, shared, residual=x)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g, g_ref, rtol=1e-12, atol=1e-15)
    # without shared: the term is simply absent
    out2, *_ = oracle.layer_forward(tab, ids, x, ln_w, eps, W_r, None)
    np.testing.assert_allclose(out2, out - shared, rtol=1e-12, atol=1e-12)


def test_layer_forward_invariants():
    tab, ids, x, ln_w, W_r, shared = fused_case(seed=21)
    # eps = 0: the normed state, hence the gates, do not change when a token's state is scaled
    scale = np.linspace(0.1, 40.0, x.shape[0])[:, None]
    _, g1, hn1, _, _ = oracle.layer_forward(tab, ids, x, ln_w, 0.0, W_r, shared)
    _, g2, hn2, _, _ = oracle.layer_forward(tab, ids, x * scale, ln_w, 0.0, W_r, shared)
    np.testing.assert_allclose(hn1, hn2, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g1, g2, rtol=1e-11, atol=1e-15)
    # unit weight, eps = 0: every normed row has mean square exactly 1
    _, _, hn3, _, _ = oracle.layer_forward(tab, ids, x, np.ones_like(ln_w), 0.0, W_r, shared)
    np.testing.assert_allclose((hn3 * hn3).mean(axis=1), 1.0, rtol=1e-13)
    # a huge eps switches the router off: uniform gates, so out = x + shared + mean of the rows
    out4, g4, _, _, _ = oracle.layer_forward(tab, ids, x, ln_w, 1e30, W_r, shared)
    np.testing.assert_allclose(g4, 1.0 / tab.shape[1], rtol=1e-9)
    np.testing.assert_allclose(out4, x + shared + tab[ids].mean(axis=1), rtol=1e-9, atol=1e-9)
    # an id outside the table: routed term zero, flagged
    bad = ids.copy()
    bad[3] = tab.shape[0]
    out5, _, _, rows5, err5 = oracle.layer_forward(tab, bad, x, ln_w, 1e-5, W_r, shared)
    assert err5 == 1 and rows5[3] == -1
    np.testing.assert_allclose(out5[3], x[3] + shared[3], rtol=0, atol=0)


def test_layer_forward_pins_catch_planted_mistakes():
    tab, ids, x, ln_w, W_r, shared = fused_case(seed=30)
    eps = 1e-5
    good, *_ = oracle.layer_forward(tab, ids, x, ln_w, eps, W_r, shared)
    rms = np.sqrt((x * x).mean(axis=1, keepdims=True) + eps)

    def layer(hn, res):
        return res + shared + np.einsum("tn,tnd->td", np_softmax(hn @ W_r), tab[ids])
    wrong = {
        "router on the un-normed state": layer(x, x),
        "norm weight dropped": layer(x / rms, x),
        "normed state as residual": layer(x / rms * ln_w, x / rms * ln_w),
        "mean subtracted (LayerNorm)": layer((x - x.mean(1, keepdims=True)) / rms * ln_w, x),
        "sum instead of mean of squares": layer(x / np.sqrt((x * x).sum(1, keepdims=True) + eps) * ln_w, x),
        "residual dropped": layer(x / rms * ln_w, 0 * x),
    }
    for name, bad in wrong.items():
        assert not np.allclose(good, bad, rtol=1e-9, atol=1e-12), name


# --------------------------------------------------------------------------------------------
# shared expert (two-matrix FFN on the router's input) and the layer that evaluates it itself
# --------------------------------------------------------------------------------------------
def np_shared_ffn(x, W1, W2, b1=None, b2=None):
    a = x @ W1.T
    if b1 is not None:
        a = a + b1
    out = np_gelu_erf(a) @ W2.T
    return out if b2 is None else out + b2


def _ffn_case(T=7, d=12, D=20, bias=True, seed=3):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    W1, W2 = rng.standard_normal((D, d)) * 0.3, rng.standard_normal((d, D)) * 0.3
    b1, b2 = (rng.standard_normal(D) * 0.2, rng.standard_normal(d) * 0.2) if bias else (None, None)
    return x, W1, W2, b1, b2


@pytest.mark.parametrize("bias", [False, True])
def test_shared_ffn_matches_numpy_matmul(bias):
    """All sizes distinct (T, d, D = 7, 12, 20), so a transposed operand or a swapped bias cannot pass."""
    x, W1, W2, b1, b2 = _ffn_case(bias=bias)
    np.testing.assert_allclose(oracle.shared_ffn(x, W1, W2, b1, b2), np_shared_ffn(x, W1, W2, b1, b2), rtol=1e-12,
                               atol=1e-13)
    # tanh form against its textbook formula
    a = x @ W1.T + (0 if b1 is None else b1)
    th = 0.5 * a * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (a + 0.044715 * a ** 3)))
    want = th @ W2.T + (0 if b2 is None else b2)
    np.testing.assert_allclose(oracle.shared_ffn(x, W1, W2, b1, b2, act=oracle.GELU_TANH), want, rtol=1e-12, atol=1e-13)


def test_shared_ffn_closed_forms():
    x, W1, W2, b1, b2 = _ffn_case()
    T, d = x.shape
    # second matrix zero: the output is its bias, whatever the input
    np.testing.assert_array_equal(oracle.shared_ffn(x, W1, np.zeros_like(W2), b1, b2), np.tile(b2, (T, 1)))
    # zero input and no first bias: GELU(0) = 0, again only the second bias is left
    np.testing.assert_array_equal(oracle.shared_ffn(np.zeros_like(x), W1, W2, None, b2), np.tile(b2, (T, 1)))
    # zero input with a first bias: one row GELU(b1) @ W2.T + b2 for every token, GELU from math.erf
    g = np.array([0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in b1])
    np.testing.assert_allclose(oracle.shared_ffn(np.zeros_like(x), W1, W2, b1, b2), np.tile(g @ W2.T + b2, (T, 1)),
                               rtol=1e-12, atol=1e-14)
    # linear in the second matrix, and tokens are independent
    np.testing.assert_allclose(oracle.shared_ffn(x, W1, 2.0 * W2, b1, None), 2.0 * oracle.shared_ffn(x, W1, W2, b1, None),
                               rtol=1e-13)
    np.testing.assert_array_equal(oracle.shared_ffn(x[2:5], W1, W2, b1, b2), oracle.shared_ffn(x, W1, W2, b1, b2)[2:5])
    # bf16 storage is widened exactly
    xb, W1b, W2b = (wl.to_storage(a, wl.BF16) for a in (x, W1, W2))
    f = lambda a: wl.storage_to_f64(a, wl.BF16)
    np.testing.assert_allclose(oracle.shared_ffn(xb, W1b, W2b), np_shared_ffn(f(xb), f(W1b), f(W2b)), rtol=1e-12,
                               atol=1e-13)


def test_layer_with_shared_ffn_is_the_layer_equation():
    """sum_j g_j v_j + FFN_shared(h) + residual with every term from an independent numpy expression."""
    rng = np.random.default_rng(8)
    V, N, d, D, T = 30, 5, 12, 20, 9
    table = rng.standard_normal((V, N, d))
    ids = rng.integers(0, V, T).astype(np.int32)
    h, res = rng.standard_normal((T, d)), rng.standard_normal((T, d))
    W_r = rng.standard_normal((d, N)) * 0.5
    _, W1, W2, b1, b2 = _ffn_case(T=T, d=d, D=D, seed=9)
    out, g, rows, err = oracle.layer_with_shared_ffn(table, ids, h, W_r, W1, W2, b1, b2, residual=res)
    gates = np_softmax(h @ W_r)
    want = np.einsum("tn,tnd->td", gates, table[ids]) + np_shared_ffn(h, W1, W2, b1, b2) + res
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g, gates, rtol=1e-12)
    np.testing.assert_array_equal(rows, ids)
    assert err == 0
    # the shared expert reads the router's input (the normed state), not the residual
    assert not np.allclose(out, np.einsum("tn,tnd->td", gates, table[ids]) + np_shared_ffn(res, W1, W2, b1, b2) + res)


def test_shared_ffn_pins_catch_planted_mistakes():
    """Wrong variants of the shared expert, written in numpy, must fail the comparison the right one passes."""
    x, W1, W2, b1, b2 = _ffn_case(T=6, d=8, D=8)        # square, so that transposed variants are well-formed
    ref = oracle.shared_ffn(x, W1, W2, b1, b2)
    wrong = {
        "first matrix transposed": np_gelu_erf(x @ W1 + b1) @ W2.T + b2,
        "second matrix transposed": np_gelu_erf(x @ W1.T + b1) @ W2 + b2,
        "no activation": (x @ W1.T + b1) @ W2.T + b2,
        "activation after the second matrix": np_gelu_erf((x @ W1.T + b1) @ W2.T + b2),
        "first bias after the activation": (np_gelu_erf(x @ W1.T) + b1) @ W2.T + b2,
        "second bias dropped": np_gelu_erf(x @ W1.T + b1) @ W2.T,
        "gated (SwiGLU-like) form": (np_gelu_erf(x @ W1.T + b1) * (x @ W1.T)) @ W2.T + b2,
    }
    np.testing.assert_allclose(ref, np_shared_ffn(x, W1, W2, b1, b2), rtol=1e-12, atol=1e-13)
    for name, val in wrong.items():
        assert not np.allclose(ref, val, rtol=1e-6, atol=1e-8), name


def test_pins_catch_planted_mistakes():
    w = wl.scaled(wl.CONFIGS["tiny"], V=97, d=24, N=5, T=33)
    tab = wl.random_table(w).astype(np.float64)
    li = {k: v.astype(np.float64) for k, v in wl.layer_inputs(w).items()}
    li["W_r"] *= 25.0
    ids = wl.token_ids(w)
    good, *_ = oracle.lookup_forward(tab, ids, li["h"], li["W_r"], li["shared"])
    g = np_softmax(li["h"] @ li["W_r"])
    wrong_variants = {
        "dropped shared": np.einsum("tn,tnd->td", g, tab[ids]),
        "uniform gates": tab[ids].mean(axis=1) + li["shared"],
        "reversed experts": np.einsum("tn,tnd->td", g[:, ::-1], tab[ids]) + li["shared"],
        "wrong sign": -np.einsum("tn,tnd->td", g, tab[ids]) + li["shared"],
        "row off by one": np.einsum("tn,tnd->td", g, tab[(ids + 1) % w.V]) + li["shared"],
        "no max-subtraction, exp of negated logits": np.einsum(
            "tn,tnd->td", np_softmax(-(li["h"] @ li["W_r"])), tab[ids]) + li["shared"],
    }
    for name, bad in wrong_variants.items():
        assert not np.allclose(good, bad, rtol=1e-9, atol=1e-12), name
