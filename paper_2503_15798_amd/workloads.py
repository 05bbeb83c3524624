"""Seeded synthetic inputs for the MoLE lookup-expert layer.

This module only *generates input bits* (tables, router weights, hidden states,
token ids) and converts between storage formats.  It holds none of the method's
arithmetic (no router, no softmax, no combine, no FFN) so that both the CPU
oracle's tests and the HIP path's tests can draw identical inputs from it
without sharing any of the computation under test.

Shapes follow the paper's model table (Table 2: 160M d=768, 410M d=1024,
D_r=4d, N in {4,16}, plus N=32 from the expert-count ablation, Table 6) and its
data setup (Sec. 5.1: GPT-NeoX tokenizer, ~50k vocabulary -> Pythia's padded
V=50304).  The paper's real inputs (Pile text, trained tables) are not
available; a truncated Zipf(s=1.1) law over V stands in for the unigram
distribution and N(0, sigma) values stand in for trained tables.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"


# ----------------------------------------------------------------------------
# storage-format helpers (bf16 is carried as uint16 bit patterns in numpy)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = np.isnan(x)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp32/fp64 values -> storage array of `dtype` (float32 array or uint16 bf16 bits)."""
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Storage array -> the exact values it encodes, as fp64."""
    if dtype == F32:
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == BF16:
        return bf16_bits_to_f32(x).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


# ----------------------------------------------------------------------------
# token-id distributions
# ----------------------------------------------------------------------------
def zipf_cdf(V: int, s: float = 1.1) -> np.ndarray:
    """CDF of the truncated Zipf law p(k) ~ k^-s, k = 1..V (rank 1 is the most frequent)."""
    w = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def zipf_ids(T: int, V: int, seed: int, s: float = 1.1, permute: bool = True) -> np.ndarray:
    """T ids with Zipf(s) rank frequencies; rank k maps to id perm[k-1] (seeded) so that
    the frequent rows are scattered over the table instead of sitting at its start."""
    rng = np.random.default_rng(seed)
    perm = rng.permutation(V) if permute else np.arange(V)
    u = rng.random(T)
    rank0 = np.searchsorted(zipf_cdf(V, s), u, side="left")
    rank0 = np.minimum(rank0, V - 1)
    return perm[rank0].astype(np.int32)


def uniform_ids(T: int, V: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(0, V, size=T, dtype=np.int64).astype(np.int32)


def make_ids(T: int, V: int, seed: int, dist: str) -> np.ndarray:
    if dist == "zipf":
        return zipf_ids(T, V, seed)
    if dist == "uniform":
        return uniform_ids(T, V, seed)
    raise ValueError(f"unknown id distribution {dist!r}")


# ----------------------------------------------------------------------------
# workload descriptions
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    V: int          # vocabulary size (rows of the table)
    d: int          # hidden size
    N: int          # routed experts (all active)
    D: int          # routed-expert hidden size D_r
    L: int          # MoLE layers sharing one id batch
    T: int          # tokens per call
    dtype: str      # storage dtype of tables / activations
    ids: str        # "zipf" | "uniform"
    seed: int
    lut_sigma: float = 0.05

    @property
    def row_elems(self) -> int:
        return self.N * self.d

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2


# The five benchmark configurations, plus the batch-size / id-distribution variants they name.
CONFIGS: Dict[str, Workload] = {
    "tiny":           Workload("tiny", 1024, 64, 4, 256, 1, 256, F32, "uniform", 0),
    "decode160m":     Workload("decode160m", 50304, 768, 16, 3072, 12, 64, BF16, "zipf", 2),
    "decode410m_t1":  Workload("decode410m_t1", 50304, 1024, 16, 4096, 24, 1, BF16, "zipf", 3),
    "decode410m_t32": Workload("decode410m_t32", 50304, 1024, 16, 4096, 24, 32, BF16, "zipf", 3),
    "decode410m":     Workload("decode410m", 50304, 1024, 16, 4096, 24, 256, BF16, "zipf", 3),
    "prefill410m":    Workload("prefill410m", 50304, 1024, 32, 4096, 1, 16384, BF16, "zipf", 4),
    "prefill410m_uniform": Workload("prefill410m_uniform", 50304, 1024, 32, 4096, 1, 16384, BF16, "uniform", 4),
    "offload410m":    Workload("offload410m", 50304, 1024, 16, 4096, 24, 32, BF16, "zipf", 5),
    # further shapes of the paper: the 1B model with 4 experts (model table) and the expert-count ablation
    "decode1b_4e":    Workload("decode1b_4e", 50304, 2048, 4, 8192, 16, 256, BF16, "zipf", 6),
    "decode410m_n2":  Workload("decode410m_n2", 50304, 1024, 2, 4096, 24, 256, BF16, "zipf", 7),
    "decode410m_n4":  Workload("decode410m_n4", 50304, 1024, 4, 4096, 24, 256, BF16, "zipf", 7),
    "decode410m_n8":  Workload("decode410m_n8", 50304, 1024, 8, 4096, 24, 256, BF16, "zipf", 7),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some sizes replaced (parity tests shrink V / T / L)."""
    return replace(w, **kw)


# ----------------------------------------------------------------------------
# host-side tensors (numpy; small and medium sizes)
# ----------------------------------------------------------------------------
def _normal(rng: np.random.Generator, shape, sigma: float) -> np.ndarray:
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def expert_weights(w: Workload, seed: Optional[int] = None, bias: bool = False,
                   norm: bool = False) -> Dict[str, np.ndarray]:
    """Embedding matrix E [V,d] ~N(0,1) and N two-matrix expert FFNs (d -> D -> d),
    W1 [N,d,D], W2 [N,D,d] ~N(0,0.02), in storage dtype.  Optional biases / RMSNorm weight."""
    rng = np.random.default_rng((w.seed if seed is None else seed) * 7919 + 11)
    out = {
        "E": to_storage(_normal(rng, (w.V, w.d), 1.0), w.dtype),
        "W1": to_storage(_normal(rng, (w.N, w.d, w.D), 0.02), w.dtype),
        "W2": to_storage(_normal(rng, (w.N, w.D, w.d), 0.02), w.dtype),
        "b1": None, "b2": None, "norm_w": None,
    }
    if bias:
        out["b1"] = to_storage(_normal(rng, (w.N, w.D), 0.1), w.dtype)
        out["b2"] = to_storage(_normal(rng, (w.N, w.d), 0.1), w.dtype)
    if norm:
        out["norm_w"] = to_storage(1.0 + _normal(rng, (w.d,), 0.1), w.dtype)
    return out


def random_table(w: Workload, layer: int = 0) -> np.ndarray:
    """A synthetic table [V,N,d] ~N(0, lut_sigma) in storage dtype (stand-in for a trained LUT)."""
    rng = np.random.default_rng(w.seed * 1000003 + 101 * layer + 1)
    return to_storage(_normal(rng, (w.V, w.N, w.d), w.lut_sigma), w.dtype)


def layer_inputs(w: Workload, layer: int = 0, T: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Per-layer activations: router weight W_r [d,N] ~N(0,0.02), router input h [T,d] ~N(0,1),
    shared-FFN output [T,d] ~N(0,1), residual [T,d] ~N(0,1); all in storage dtype."""
    T = w.T if T is None else T
    rng = np.random.default_rng(w.seed * 1000003 + 101 * layer + 2)
    return {
        "W_r": to_storage(_normal(rng, (w.d, w.N), 0.02), w.dtype),
        "h": to_storage(_normal(rng, (T, w.d), 1.0), w.dtype),
        "shared": to_storage(_normal(rng, (T, w.d), 1.0), w.dtype),
        "residual": to_storage(_normal(rng, (T, w.d), 1.0), w.dtype),
    }


def shared_ffn_weights(w: Workload, D_s: int, layer: int = 0, bias: bool = True) -> Dict[str, np.ndarray]:
    """Shared expert of a layer: W1 [D_s, d] and W2 [d, D_s] ~N(0, 0.02), stored as a linear layer stores its
    weight ([out, in]); optional biases b1 [D_s], b2 [d] ~N(0, 0.1); storage dtype."""
    rng = np.random.default_rng(w.seed * 1000003 + 101 * layer + 4)
    out = {
        "W1": to_storage(_normal(rng, (D_s, w.d), 0.02), w.dtype),
        "W2": to_storage(_normal(rng, (w.d, D_s), 0.02), w.dtype),
        "b1": None, "b2": None,
    }
    if bias:
        out["b1"] = to_storage(_normal(rng, (D_s,), 0.1), w.dtype)
        out["b2"] = to_storage(_normal(rng, (w.d,), 0.1), w.dtype)
    return out


def norm_inputs(w: Workload, layer: int = 0, T: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Inputs of the layer taken from the post-attention state: x [T,d] ~N(0,1) times a per-token scale
    drawn log-uniformly from [1/8, 8] (so that a norm in front of the router matters), and the norm
    weight ln_w [d] ~U(0.5, 1.5); storage dtype."""
    T = w.T if T is None else T
    rng = np.random.default_rng(w.seed * 1000003 + 101 * layer + 3)
    scale = np.exp2(rng.uniform(-3.0, 3.0, size=(T, 1)))
    return {
        "x": to_storage(_normal(rng, (T, w.d), 1.0) * scale, w.dtype),
        "ln_w": to_storage(rng.uniform(0.5, 1.5, size=(w.d,)), w.dtype),
    }


def token_ids(w: Workload, batch: int = 0, T: Optional[int] = None) -> np.ndarray:
    """Batch `batch` of token ids for the workload (different batches rotate through the table)."""
    T = w.T if T is None else T
    return make_ids(T, w.V, w.seed * 7919 + 13 * batch, w.ids)


# ----------------------------------------------------------------------------
# device-side tensors for tables too large to build on the host (torch, lazily imported)
# ----------------------------------------------------------------------------
def device_table(w: Workload, layer: int, device, out=None):
    """bf16/fp32 table [V,N,d] ~N(0, lut_sigma) generated on `device` from a seeded generator.
    Returns a torch tensor; pass `out` to fill an existing tensor (e.g. a slice of [L,V,N,d])."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(w.seed * 1000003 + 101 * layer + 1)
    tdt = torch.float32 if w.dtype == F32 else torch.bfloat16
    if out is None:
        out = torch.empty((w.V, w.N, w.d), dtype=tdt, device=device)
    # normal_ on bf16 draws in fp32 and rounds; chunk to bound the temporary
    out.normal_(0.0, w.lut_sigma, generator=g)
    return out
