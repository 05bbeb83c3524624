"""LUT files (host-only calls of the library; no GPU): the bytes on disk are checked against the format
the header documents by parsing them here with struct / numpy, and row reads against plain numpy
indexing of the source tables -- copies and gathers, so everything is bit-exact."""
import os
import struct

import numpy as np
import pytest
import torch

from paper_2503_15798_amd import binding as mb


def tables(L, V, N, d, dtype, seed):
    rng = np.random.default_rng(seed)
    if dtype == mb.MOLE_BF16:
        return rng.integers(0, 1 << 16, size=(L, V, N, d), dtype=np.uint16)
    if dtype == mb.MOLE_U8:
        return rng.integers(0, 256, size=(L, V, N, d), dtype=np.uint8)      # raw bytes (quantised tables)
    return rng.standard_normal((L, V, N, d)).astype(np.float32)


def as_tensor(a):
    """numpy array -> torch CPU tensor sharing nothing (the binding takes tensors or addresses)."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy())
    return torch.from_numpy(a.copy())


ELEM_BYTES = {mb.MOLE_F32: 4, mb.MOLE_BF16: 2, mb.MOLE_U8: 1}
TORCH_DT = {mb.MOLE_F32: torch.float32, mb.MOLE_BF16: torch.int16, mb.MOLE_U8: torch.uint8}


def write_file(path, tab, dtype, layout, threads=3):
    L, V, N, d = tab.shape
    f = mb.mole_lut_file_create(path, dtype, layout, L, V, N, d)
    try:
        for l in range(L):
            mb.mole_lut_file_write_layer(f, l, as_tensor(tab[l]), threads)
    finally:
        mb.mole_lut_file_close(f)


@pytest.mark.parametrize("dtype", [mb.MOLE_BF16, mb.MOLE_F32, mb.MOLE_U8])
@pytest.mark.parametrize("layout", [mb.MOLE_LAYOUT_LAYER_MAJOR, mb.MOLE_LAYOUT_ID_MAJOR])
def test_bytes_on_disk_follow_the_documented_format(tmp_path, dtype, layout):
    L, V, N, d = 3, 37, 4, 24
    tab = tables(L, V, N, d, dtype, seed=11)
    path = str(tmp_path / "t.molelut")
    write_file(path, tab, dtype, layout)
    raw = open(path, "rb").read()
    eb = ELEM_BYTES[dtype]
    assert len(raw) == 4096 + L * V * N * d * eb
    magic, ver, hb, dt, lay, v, l, n, dd, zero, pb = struct.unpack_from("<8sIIIIqiiiIQ", raw, 0)
    assert magic == b"MOLELUT\0" and ver == 1 and hb == 4096 and dt == dtype and lay == layout
    assert (v, l, n, dd, zero, pb) == (V, L, N, d, 0, L * V * N * d * eb)
    assert raw[56:4096] == bytes(4096 - 56)
    payload = np.frombuffer(raw, dtype=tab.dtype, offset=4096)
    want = tab if layout == mb.MOLE_LAYOUT_LAYER_MAJOR else tab.transpose(1, 0, 2, 3)
    assert np.array_equal(payload.reshape(want.shape), want)


@pytest.mark.parametrize("dtype", [mb.MOLE_BF16, mb.MOLE_F32, mb.MOLE_U8])
@pytest.mark.parametrize("layout", [mb.MOLE_LAYOUT_LAYER_MAJOR, mb.MOLE_LAYOUT_ID_MAJOR])
@pytest.mark.parametrize("threads", [1, 5])
def test_read_rows_is_a_gather_of_all_layers(tmp_path, dtype, layout, threads):
    L, V, N, d = 4, 101, 2, 40
    tab = tables(L, V, N, d, dtype, seed=5)
    path = str(tmp_path / "t.molelut")
    write_file(path, tab, dtype, layout)
    f, desc = mb.mole_lut_file_open(path)
    try:
        assert (desc.dtype, desc.layout, desc.L, desc.N, desc.d, desc.V) == (dtype, layout, L, N, d, V)
        ids = np.array([0, V - 1, 7, 7, 50, 3, 99, 0, 1], dtype=np.int32)
        dst = torch.full((len(ids), L, N, d), 7, dtype=TORCH_DT[dtype])
        mb.mole_lut_file_read_rows(f, torch.from_numpy(ids), len(ids), dst, threads)
        got = dst.numpy().view(tab.dtype)
        want = tab[:, ids].transpose(1, 0, 2, 3)            # [n, L, N, d]
        assert np.array_equal(got, want)
        # the mapping shows the same payload
        addr = mb.mole_lut_file_payload(f)
        import ctypes
        nelem = L * V * N * d
        ctype = {mb.MOLE_BF16: ctypes.c_uint16, mb.MOLE_F32: ctypes.c_float, mb.MOLE_U8: ctypes.c_uint8}[dtype]
        mapped = np.ctypeslib.as_array((ctype * nelem).from_address(addr))
        want_all = tab if layout == mb.MOLE_LAYOUT_LAYER_MAJOR else tab.transpose(1, 0, 2, 3)
        assert np.array_equal(mapped.reshape(want_all.shape), want_all)
        del mapped
        # n = 0 reads nothing
        mb.mole_lut_file_read_rows(f, None, 0, None, threads)
    finally:
        mb.mole_lut_file_close(f)


def test_errors(tmp_path):
    L, V, N, d = 2, 10, 2, 8
    tab = tables(L, V, N, d, mb.MOLE_BF16, seed=1)
    path = str(tmp_path / "t.molelut")
    write_file(path, tab, mb.MOLE_BF16, mb.MOLE_LAYOUT_ID_MAJOR)

    with pytest.raises(mb.MoleError) as e:
        mb.mole_lut_file_open(str(tmp_path / "missing.molelut"))
    assert e.value.status == mb.MOLE_EIO
    with pytest.raises(mb.MoleError) as e:
        mb.mole_lut_file_create(str(tmp_path / "no_such_dir" / "x"), mb.MOLE_BF16, 0, L, V, N, d)
    assert e.value.status == mb.MOLE_EIO
    for bad in (dict(dtype=9), dict(layout=2), dict(L=0), dict(V=0), dict(N=0), dict(d=0)):
        a = dict(dtype=mb.MOLE_BF16, layout=0, L=L, V=V, N=N, d=d)
        a.update(bad)
        with pytest.raises(mb.MoleError) as e:
            mb.mole_lut_file_create(str(tmp_path / "bad"), **a)
        assert e.value.status == mb.MOLE_EINVAL

    f, _ = mb.mole_lut_file_open(path)
    try:
        dst = torch.zeros((2, L, N, d), dtype=torch.int16)
        for ids in ([0, V], [-1, 0]):
            with pytest.raises(mb.MoleError) as e:
                mb.mole_lut_file_read_rows(f, torch.tensor(ids, dtype=torch.int32), 2, dst, 2)
            assert e.value.status == mb.MOLE_EINVAL and "outside" in e.value.message
        assert not dst.any()                                # nothing was read
        with pytest.raises(mb.MoleError) as e:              # opened read-only
            mb.mole_lut_file_write_layer(f, 0, as_tensor(tab[0]), 1)
        assert e.value.status == mb.MOLE_EINVAL
    finally:
        mb.mole_lut_file_close(f)
    mb.mole_lut_file_close(None)                            # no-op

    raw = open(path, "rb").read()
    trunc = str(tmp_path / "trunc.molelut")
    open(trunc, "wb").write(raw[:-16])
    with pytest.raises(mb.MoleError) as e:
        mb.mole_lut_file_open(trunc)
    assert e.value.status == mb.MOLE_EINVAL and "payload size" in e.value.message
    badmagic = str(tmp_path / "magic.molelut")
    open(badmagic, "wb").write(b"NOTALUT\0" + raw[8:])
    with pytest.raises(mb.MoleError) as e:
        mb.mole_lut_file_open(badmagic)
    assert e.value.status == mb.MOLE_EINVAL
    # a crafted header whose size product wraps around 2^64 back to the real payload size: L * V * N * d * 2 =
    # 64 * (10 + 2^58) = 640 + 2^64.  It must be refused, not mapped as a table of 2^58 rows.
    wrap = str(tmp_path / "wrap.molelut")
    assert struct.unpack_from("<q", raw, 24)[0] == V
    open(wrap, "wb").write(raw[:24] + struct.pack("<q", V + (1 << 58)) + raw[32:])
    with pytest.raises(mb.MoleError) as e:
        mb.mole_lut_file_open(wrap)
    assert e.value.status == mb.MOLE_EINVAL and "too large" in e.value.message
    short = str(tmp_path / "short.molelut")
    open(short, "wb").write(raw[:100])
    with pytest.raises(mb.MoleError) as e:
        mb.mole_lut_file_open(short)
    assert e.value.status == mb.MOLE_EIO

    f = mb.mole_lut_file_create(str(tmp_path / "w.molelut"), mb.MOLE_BF16, 0, L, V, N, d)
    try:
        with pytest.raises(mb.MoleError):
            mb.mole_lut_file_write_layer(f, L, as_tensor(tab[0]), 1)
        with pytest.raises(mb.MoleError):
            mb.mole_lut_file_write_layer(f, 0, None, 1)
    finally:
        mb.mole_lut_file_close(f)
