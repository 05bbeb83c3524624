"""Pins of the NF4 / NF3 codec oracle (oracle/nf_codec.py) and of the library's level table -- no GPU.
The oracle derives its levels from scipy's normal quantile function; the library carries a table from
its own generator (standard-library inverse CDF).  Neither may be checked against itself: the NF4 values
are held against the table the data type's own paper prints (tests/golden/nf4_levels.txt)."""
import os

import numpy as np
import pytest
import scipy.optimize
import scipy.stats

from oracle import nf_codec as nf
from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl


GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "nf4_levels.txt")


def printed_nf4_levels():
    with open(GOLDEN) as f:
        return np.array([float(line) for line in f if line.strip() and not line.startswith("#")])


def test_nf4_levels_are_the_printed_ones():
    """The data type's own paper prints the sixteen NF4 values; the oracle's construction must land on them
    (they were produced in float32 there, hence a few float32 roundings of slack, 1e-6).  The two plausible
    misreadings of the outermost quantile miss them by 2e-3 and more."""
    printed = printed_nf4_levels()
    assert printed.shape == (16,)
    np.testing.assert_allclose(nf.codebook(4).astype(np.float64), printed, rtol=0, atol=1e-6)
    for delta in (1 - 1 / 32, 1 - 1 / 30):                     # a step of 1/16, or of 1/15, alone
        pos = scipy.stats.norm.ppf(np.linspace(0.5, delta, 9))
        neg = scipy.stats.norm.ppf(np.linspace(1 - delta, 0.5, 8))[:-1]
        wrong = np.concatenate([neg, pos]) / pos[-1]
        assert np.abs(wrong - printed).max() > 1.5e-3


@pytest.mark.parametrize("bits", [4, 3])
def test_levels_follow_the_definition(bits):
    lv = nf.codebook(bits).astype(np.float64)
    n, half = 2 ** bits, 2 ** (bits - 1)
    assert len(lv) == n and (np.diff(lv) > 0).all()
    assert lv[0] == -1.0 and lv[-1] == 1.0 and lv[half - 1] == 0.0           # exact -1, 0, +1
    assert (lv < 0).sum() == half - 1 and (lv > 0).sum() == half            # asymmetric: one more positive level
    # the levels are evenly spaced in probability on each side (that is what "quantiles" means); the
    # outermost probability is not assumed here but recovered from the printed NF4 table: the printed
    # second-highest level fixes the quantile the levels were divided by
    printed = printed_nf4_levels()
    f = lambda top: (scipy.stats.norm.cdf(printed[-2] * top) - 0.5) * 8 / 7 + 0.5 - scipy.stats.norm.cdf(top)
    top4 = scipy.optimize.brentq(f, 1.0, 3.0)
    delta4 = scipy.stats.norm.cdf(top4)                                       # 0.96771 from the printed values
    assert abs(delta4 - (1 - (1 / 30 + 1 / 32) / 2)) < 2e-6
    delta = 1 - (1 / (2 * (n - 1)) + 1 / (2 * n)) / 2                         # the same rule at this width
    top = scipy.stats.norm.ppf(delta)
    p = scipy.stats.norm.cdf(lv * top)
    np.testing.assert_allclose(np.diff(p[half - 1:]), (delta - 0.5) / half, rtol=2e-6)
    np.testing.assert_allclose(np.diff(p[:half]), (delta - 0.5) / (half - 1), rtol=2e-6)
    np.testing.assert_allclose(p[-1], delta, rtol=1e-7)
    np.testing.assert_allclose(p[0], 1 - delta, rtol=1e-6)


@pytest.mark.parametrize("bits", [4, 3])
def test_library_table_equals_the_oracle_levels(bits):
    """Two independent derivations (scipy ppf vs. the library's generator) give the same fp32 levels."""
    lib_levels = np.array(mb.mole_nf_codebook(bits), dtype=np.float32)
    np.testing.assert_array_equal(lib_levels, nf.codebook(bits))
    assert mb.mole_nf_codebook(5) == []


@pytest.mark.parametrize("bits,block", [(4, 768), (3, 128), (4, 64), (3, 16)])
def test_quantise_picks_the_nearest_level(bits, block):
    rng = np.random.default_rng(bits * 100 + block)
    x = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(rng.standard_normal((5, 3, 768)).astype(np.float32) * 0.05))
    codes, scales = nf.quantize(x, bits, block)
    assert codes.max() < 2 ** bits and scales.shape == (5, 3, 768 // block)
    np.testing.assert_array_equal(scales, np.abs(x.reshape(5, 3, -1, block)).max(axis=-1))   # exact absmax
    lv = nf.codebook(bits).astype(np.float64)
    xn = (x.reshape(5, 3, -1, block).astype(np.float64) / scales[..., None]).reshape(x.shape)
    nearest = np.abs(xn[..., None] - lv).argmin(axis=-1)
    # brute-force nearest level in fp64; only elements within fp32 rounding of a midpoint may differ
    mids = (lv[:-1] + lv[1:]) / 2
    margin = np.abs(xn[..., None] - mids).min(axis=-1)
    differ = codes != nearest
    assert differ.mean() < 1e-3 and (margin[differ] < 1e-6).all()
    # the element that defines the block's scale maps to -1 or +1
    dq = nf.dequantize(codes, scales, bits, block)
    top = np.abs(x.reshape(5, 3, -1, block)).argmax(axis=-1)
    np.testing.assert_array_equal(np.take_along_axis(dq.reshape(5, 3, -1, block), top[..., None], -1)[..., 0],
                                  np.take_along_axis(x.reshape(5, 3, -1, block), top[..., None], -1)[..., 0])
    # error bound: half the widest gap between levels, times the scale
    gap = np.diff(lv).max() / 2
    assert (np.abs(dq - x).reshape(5, 3, -1, block) <= gap * scales[..., None] * (1 + 1e-6)).all()


def test_special_blocks():
    x = np.zeros((1, 1, 64), np.float32)
    codes, scales = nf.quantize(x, 4, 64)
    assert (scales == 0).all() and (codes == 7).all()                 # zero block: scale 0, the zero level
    assert (nf.dequantize(codes, scales, 4, 64) == 0).all()
    lv = nf.codebook(4)
    x = np.tile(lv * np.float32(2.5), 4)[None, None, :].astype(np.float32)              # exactly on the levels
    codes, scales = nf.quantize(x, 4, 64)
    np.testing.assert_array_equal(codes[0, 0, :16], np.arange(16))
    np.testing.assert_allclose(nf.dequantize(codes, scales, 4, 64), x, rtol=1e-6)
    # a tie (value exactly on a midpoint) goes to the lower level
    m = nf.midpoints(3)
    x = np.tile(np.concatenate([m, [1.0]]).astype(np.float32), 2)[None, None, :]
    codes, _ = nf.quantize(x, 3, 16)
    np.testing.assert_array_equal(codes[0, 0, :7], np.arange(7))


@pytest.mark.parametrize("bits", [4, 3])
def test_pack_unpack_roundtrip_and_layout(bits):
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 2 ** bits, size=(3, 2, 64), dtype=np.uint8)
    packed = nf.pack(codes, bits)
    assert packed.shape == (3, 2, 64 * bits // 8)
    np.testing.assert_array_equal(nf.unpack(packed, bits, 64), codes)
    one = np.zeros((1, 1, 16), np.uint8)
    if bits == 4:
        one[0, 0, 0], one[0, 0, 1], one[0, 0, 15] = 0xA, 0x3, 0xF
        p = nf.pack(one, 4)[0, 0]
        assert p[0] == 0x3A and p[7] == 0xF0                          # element 2i in the low nibble
    else:
        one[0, 0, 0], one[0, 0, 3], one[0, 0, 7], one[0, 0, 9] = 0b101, 0b011, 0b110, 0b111
        p = nf.pack(one, 3)[0, 0]
        # elements 0..7 -> word 0 = 5 | 3 << 9 | 6 << 21; element 9 -> word 1 = 7 << 3
        w0, w1 = 5 | (3 << 9) | (6 << 21), 7 << 3
        assert list(p[:4]) == [w0 & 0xFF, (w0 >> 8) & 0xFF, w1 & 0xFF, (w1 >> 8) & 0xFF]   # low 16 bits of each word
        assert list(p[4:]) == [w0 >> 16, w1 >> 16]                                        # then the high 8 bits


def test_size_ratios_of_the_paper():
    full = 50304 * 4 * 768 * 2
    assert abs(nf.table_bytes(50304, 4, 768, 4, 768, 4) / full - 0.253) < 0.001      # Sec. 5.5
    assert abs(nf.table_bytes(50304, 4, 768, 3, 128, 2) / full - 0.195) < 0.001
