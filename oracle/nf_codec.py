"""NormalFloat (NF4 / NF3) block quantisation of a lookup table -- CPU oracle of the codec.

TEST INFRASTRUCTURE ONLY (see oracle/mole_oracle.c).  Shares nothing with the HIP path: the code-book
is derived here from scipy's normal quantile function; the library carries its own table from its own
generator.

What the MoLE paper fixes (Sec. 5.5 and Table 8): the 16-bit tables are post-training quantised to the
NF4 and NF3 data types of the QLoRA paper with token-wise blocks of 768 and 128 elements, which brings
storage and per-token traffic to 25.3 % and 19.5 %.  Those ratios pin the scale widths:
(4 + 32/768)/16 = 25.26 % (one 32-bit absmax per block) and (3 + 16/128)/16 = 19.53 % (16-bit absmax).

The NF-k data type, as the QLoRA paper defines it: 2^k levels that are quantiles of N(0,1) normalised
to [-1, 1], asymmetric so that 0 is a level: the quantiles of a positive range with 2^(k-1)+1 points
and of a negative range with 2^(k-1) points are united and the duplicate zero dropped.  The quantile of
probability 1 is infinite, so the outermost one is taken at delta < 1: the cumulative probabilities of
the positive range run evenly from 1/2 to delta, those of the negative range evenly from 1/2 down to
1 - delta, and the levels are divided by the quantile at delta.  delta is half a step short of 1, where
a step is 1/(2^k - 1) when the zero shared by both halves is counted once and 1/2^k when it is counted
twice; the data type takes the mean of the two: delta = 1 - (1/(2 (2^k - 1)) + 1/(2 2^k)) / 2
(0.9677083 for k = 4).  PIN: the QLoRA paper prints the sixteen NF4 values in its appendix on the exact
values of the data type (tests/golden/nf4_levels.txt); this construction reproduces them to fp32
rounding, a delta of 1 - 1/(2 2^k) or 1 - 1/(2 (2^k - 1)) alone misses them in the third decimal.  No
NF3 table is printed anywhere: its values are the same construction at k = 3, PARITY UNPINNED beyond
the structure (exact -1, 0, +1, 3 negative and 4 positive levels, evenly spaced in probability).

Quantisation rule (both sides take every decision in fp32):
    s    = max |x| over the block (exact; for a bf16 table it is itself a bf16 value, so a 16-bit scale
           loses nothing)
    xn   = fp32(x) / s          (IEEE fp32 division; xn = 0 when s == 0)
    code = number of midpoints m_i < xn, m_i = fp32((level_i + level_{i+1}) / 2)   (a tie goes down)
    x^   = level[code] * s      (fp32 product)
Packing: NF4 -- two codes per byte, element 2i in the low nibble.  NF3 -- every 8 consecutive elements
form a 24-bit word (element e in bits 3e..3e+2); per row the low 16 bits of all words come first
(little-endian, d/4 bytes), then their high 8 bits (d/8 bytes).
"""
from __future__ import annotations

from typing import Tuple

import numpy as np
import scipy.stats


def codebook(bits: int) -> np.ndarray:
    """The 2^bits NF levels, ascending, as float32."""
    if bits not in (2, 3, 4, 5, 6, 7, 8):
        raise ValueError("bits out of range")
    half = 2 ** (bits - 1)
    n = 2 ** bits
    delta = 1.0 - (1.0 / (2.0 * (n - 1)) + 1.0 / (2.0 * n)) / 2.0
    pos = scipy.stats.norm.ppf(np.linspace(0.5, delta, half + 1))        # 0 ... Q(delta): 2^(k-1)+1 points
    neg = scipy.stats.norm.ppf(np.linspace(1.0 - delta, 0.5, half))[:-1]  # -Q(delta) ... : its zero dropped
    levels = np.concatenate([neg, pos]) / pos[-1]
    levels[half - 1] = 0.0
    assert len(levels) == 2 ** bits
    return levels.astype(np.float32)


def midpoints(bits: int) -> np.ndarray:
    lv = codebook(bits).astype(np.float64)
    return ((lv[:-1] + lv[1:]) / 2.0).astype(np.float32)


def quantize(table_f32: np.ndarray, bits: int, block: int) -> Tuple[np.ndarray, np.ndarray]:
    """table [..., d] float32 (exact widening of the stored values) -> (codes [..., d] uint8,
    scales [..., d/block] float32)."""
    x = np.ascontiguousarray(table_f32, dtype=np.float32)
    d = x.shape[-1]
    if d % block:
        raise ValueError("block must divide d")
    xb = x.reshape(x.shape[:-1] + (d // block, block))
    s = np.abs(xb).max(axis=-1).astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        xn = np.where(s[..., None] > 0, xb / s[..., None], np.float32(0)).astype(np.float32)
    mids = midpoints(bits)
    codes = (xn[..., None] > mids).sum(axis=-1).astype(np.uint8)
    return codes.reshape(x.shape), s


def dequantize(codes: np.ndarray, scales: np.ndarray, bits: int, block: int) -> np.ndarray:
    """-> float32 [..., d]: level[code] * scale, product in fp32."""
    lv = codebook(bits)
    d = codes.shape[-1]
    v = lv[codes].reshape(codes.shape[:-1] + (d // block, block)) * scales[..., None].astype(np.float32)
    return v.reshape(codes.shape).astype(np.float32)


def pack(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes [..., d] -> bytes [..., d*bits/8] in the layout described in the module docstring."""
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    d = c.shape[-1]
    if bits == 4:
        return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)
    if bits == 3:
        g = c.reshape(c.shape[:-1] + (d // 8, 8)).astype(np.uint32)
        word = np.zeros(g.shape[:-1], dtype=np.uint32)
        for e in range(8):
            word |= g[..., e] << np.uint32(3 * e)
        lo16 = np.stack([(word & 0xFF), (word >> 8) & 0xFF], axis=-1).reshape(c.shape[:-1] + (d // 4,))
        hi8 = (word >> 16) & 0xFF
        return np.concatenate([lo16, hi8], axis=-1).astype(np.uint8)
    raise ValueError("packing is defined for 3 and 4 bits")


def unpack(packed: np.ndarray, bits: int, d: int) -> np.ndarray:
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    out = np.zeros(p.shape[:-1] + (d,), dtype=np.uint8)
    if bits == 4:
        out[..., 0::2] = p & 15
        out[..., 1::2] = p >> 4
        return out
    if bits == 3:
        lo16, hi8 = p[..., : d // 4].astype(np.uint32), p[..., d // 4:].astype(np.uint32)
        word = lo16[..., 0::2] | (lo16[..., 1::2] << 8) | (hi8 << 16)
        for e in range(8):
            out[..., e::8] = ((word >> np.uint32(3 * e)) & 7).astype(np.uint8)
        return out
    raise ValueError("packing is defined for 3 and 4 bits")


def table_bytes(rows: int, N: int, d: int, bits: int, block: int, scale_bytes: int) -> int:
    return rows * N * (d * bits // 8 + (d // block) * scale_bytes)
