"""ctypes binding of libmole.so: one Python function per C entry point, same names.

Argument marshalling only -- every step of the path runs in the library's HIP kernels.
Tensor arguments are torch tensors living on the GPU (or pinned host tensors where the
header allows host memory); their data pointers are passed through unchanged.  There is
no CPU fallback: if the library is missing, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
# MOLE_LIB overrides the library file (used to compare differently compiled builds)
LIB_PATH = os.environ.get("MOLE_LIB") or os.path.join(_HERE, "libmole.so")

MOLE_OK, MOLE_EINVAL, MOLE_EUNSUPPORTED, MOLE_EWORKSPACE, MOLE_EHIP, MOLE_EIO = range(6)
MOLE_F32, MOLE_BF16, MOLE_U8 = 0, 1, 2
MOLE_GELU_ERF, MOLE_GELU_TANH = 0, 1
MOLE_FLAG_DEDUP = 1
MOLE_FLAG_RUNS = 2
MOLE_LAYOUT_LAYER_MAJOR, MOLE_LAYOUT_ID_MAJOR = 0, 1
MOLE_NOALLOC_MAX_T = 16384

_STATUS_NAMES = {0: "MOLE_OK", 1: "MOLE_EINVAL", 2: "MOLE_EUNSUPPORTED", 3: "MOLE_EWORKSPACE", 4: "MOLE_EHIP",
                 5: "MOLE_EIO"}

# every symbol include/mole.h declares
EXPORTS = ("mole_last_error", "mole_version", "mole_build_lut_workspace", "mole_build_lut",
           "mole_dedup_workspace", "mole_dedup_ids", "mole_lookup_forward",
           "mole_lookup_forward_layers", "mole_set_tuning", "mole_layer_forward", "mole_offload_fetch", "mole_offload_fetch_idmajor",
           "mole_lut_file_create", "mole_lut_file_open", "mole_lut_file_payload", "mole_lut_file_write_layer",
           "mole_lut_file_read_rows", "mole_lut_file_close", "mole_nf_codebook", "mole_nf_codes_bytes",
           "mole_nf_scales_bytes", "mole_quantize_lut", "mole_lookup_forward_nf", "mole_offload_fetch_nf",
           "mole_layer_forward_nf", "mole_lookup_forward_noalloc", "mole_shared_ffn_workspace",
           "mole_shared_ffn_forward", "mole_dedup_forward_workspace", "mole_dedup_forward")


class LutDesc(ctypes.Structure):
    """mole_lut_desc of include/mole.h."""
    _fields_ = [("dtype", ctypes.c_int32), ("layout", ctypes.c_int32), ("L", ctypes.c_int32),
                ("N", ctypes.c_int32), ("d", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("V", ctypes.c_int64)]


class MoleError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


_lib = None


def lib() -> ctypes.CDLL:
    """Load libmole.so (built in-tree by paper_2503_15798_amd.build); raise if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2503_15798_amd.build` "
                          "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    c_void, c_i32, c_i64, c_sz, c_f, c_u = (ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t,
                                            ctypes.c_float, ctypes.c_uint)
    L.mole_last_error.restype = ctypes.c_char_p
    L.mole_last_error.argtypes = []
    L.mole_version.restype = c_i32
    L.mole_version.argtypes = []
    L.mole_build_lut_workspace.restype = c_sz
    L.mole_build_lut_workspace.argtypes = [c_i64, c_i32, c_i32, c_i32, c_i32]
    L.mole_build_lut.restype = c_i32
    L.mole_build_lut.argtypes = [c_void] * 6 + [c_f, c_void, c_i64, c_i32, c_i32, c_i32, c_i32, c_i32,
                                                c_void, c_sz, c_void]
    L.mole_dedup_workspace.restype = c_sz
    L.mole_dedup_workspace.argtypes = [c_i32, c_i64]
    L.mole_dedup_ids.restype = c_i32
    L.mole_dedup_ids.argtypes = [c_void, c_i32, c_i64, c_void, c_void, c_void, c_void, c_void, c_sz, c_void]
    L.mole_lookup_forward.restype = c_i32
    L.mole_lookup_forward.argtypes = [c_void] * 11 + [c_i32, c_i64, c_i32, c_i32, c_i32, c_u, c_void, c_sz, c_void]
    L.mole_lookup_forward_layers.restype = c_i32
    L.mole_lookup_forward_layers.argtypes = ([c_void, c_i64] + [c_void] * 7 + [c_i64] + [c_void] * 3 +
                                             [c_i32, c_i32, c_i64, c_i32, c_i32, c_i32, c_u, c_void, c_sz, c_void])
    L.mole_lookup_forward_noalloc.restype = c_i32
    L.mole_lookup_forward_noalloc.argtypes = [c_void] * 8 + [c_i32, c_i64, c_i32, c_i32, c_i32, c_void]
    L.mole_shared_ffn_workspace.restype = c_sz
    L.mole_shared_ffn_workspace.argtypes = [c_i32, c_i32, c_i32, c_i32]
    L.mole_shared_ffn_forward.restype = c_i32
    L.mole_shared_ffn_forward.argtypes = [c_void] * 13 + [c_i32, c_i64, c_i32, c_i32, c_i32, c_i32, c_i32, c_void, c_sz,
                                                          c_void]
    L.mole_set_tuning.restype = c_i32
    L.mole_set_tuning.argtypes = [ctypes.c_char_p, c_i32]
    L.mole_layer_forward.restype = c_i32
    L.mole_layer_forward.argtypes = ([c_void, c_i64, c_void, c_void, c_void, c_void, c_f, c_void, c_void, c_void,
                                      c_i64, c_void, c_void, c_void] +
                                     [c_i32, c_i32, c_i64, c_i32, c_i32, c_i32, c_u, c_void, c_sz, c_void])
    L.mole_dedup_forward_workspace.restype = c_sz
    L.mole_dedup_forward_workspace.argtypes = [c_i32, c_i64, c_i32, c_i32]
    L.mole_dedup_forward.restype = c_i32
    L.mole_dedup_forward.argtypes = ([c_void, c_i64, c_void, c_void, c_void, c_f, c_void, c_void, c_void, c_void, c_i64] +
                                     [c_void] * 4 + [c_i32, c_i32, c_i64, c_i32, c_i32, c_i32, c_void, c_sz, c_void])
    L.mole_offload_fetch.restype = c_i32
    L.mole_offload_fetch.argtypes = [c_void, c_i64, c_void, c_void, c_void, c_i64, c_void,
                                     c_i32, c_i32, c_i64, c_i32, c_i32, c_i32, c_void]
    L.mole_offload_fetch_idmajor.restype = c_i32
    L.mole_offload_fetch_idmajor.argtypes = [c_void, c_void, c_void, c_void, c_i64, c_void,
                                             c_i32, c_i32, c_i64, c_i32, c_i32, c_i32, c_void]
    L.mole_offload_fetch_nf.restype = c_i32
    L.mole_offload_fetch_nf.argtypes = [c_void, c_i64, c_void, c_i64, c_void, c_void, c_void, c_i64, c_void, c_i64,
                                        c_void, c_i32, c_i32, c_i64, c_i32, c_i32, c_i32, c_i32, c_i32, c_void]
    L.mole_lut_file_create.restype = c_i32
    L.mole_lut_file_create.argtypes = [ctypes.c_char_p, ctypes.POINTER(LutDesc), ctypes.POINTER(c_void)]
    L.mole_lut_file_open.restype = c_i32
    L.mole_lut_file_open.argtypes = [ctypes.c_char_p, ctypes.POINTER(c_void), ctypes.POINTER(LutDesc)]
    L.mole_lut_file_payload.restype = c_void
    L.mole_lut_file_payload.argtypes = [c_void]
    L.mole_lut_file_write_layer.restype = c_i32
    L.mole_lut_file_write_layer.argtypes = [c_void, c_i32, c_void, c_i32]
    L.mole_lut_file_read_rows.restype = c_i32
    L.mole_lut_file_read_rows.argtypes = [c_void, c_void, c_i32, c_void, c_i32]
    L.mole_lut_file_close.restype = c_i32
    L.mole_lut_file_close.argtypes = [c_void]
    L.mole_nf_codebook.restype = c_i32
    L.mole_nf_codebook.argtypes = [c_i32, c_void]
    L.mole_nf_codes_bytes.restype = c_sz
    L.mole_nf_codes_bytes.argtypes = [c_i64, c_i32, c_i32, c_i32]
    L.mole_nf_scales_bytes.restype = c_sz
    L.mole_nf_scales_bytes.argtypes = [c_i64, c_i32, c_i32, c_i32, c_i32]
    L.mole_quantize_lut.restype = c_i32
    L.mole_quantize_lut.argtypes = [c_void, c_void, c_void, c_i64, c_i32, c_i32, c_i32, c_i32, c_i32, c_void]
    L.mole_lookup_forward_nf.restype = c_i32
    L.mole_lookup_forward_nf.argtypes = ([c_void, c_i64, c_void, c_i64] + [c_void] * 7 + [c_i64] + [c_void] * 3 +
                                         [c_i32, c_i32, c_i64, c_i32, c_i32, c_i32, c_i32, c_i32, c_u, c_void, c_sz,
                                          c_void])
    L.mole_layer_forward_nf.restype = c_i32
    L.mole_layer_forward_nf.argtypes = ([c_void, c_i64, c_void, c_i64, c_void, c_void, c_void, c_void, ctypes.c_float,
                                         c_void, c_void, c_void, c_i64, c_void, c_void, c_void] +
                                        [c_i32, c_i32, c_i64, c_i32, c_i32, c_i32, c_i32, c_i32, c_u, c_void, c_sz,
                                         c_void])
    _lib = L
    return L


def _ptr(t) -> Optional[int]:
    """Raw address of a tensor's storage (None stays NULL).  Integers pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("libmole takes dense row-major tensors")
    return t.data_ptr()


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int) -> None:
    if status != MOLE_OK:
        raise MoleError(status, lib().mole_last_error().decode())


def mole_last_error() -> str:
    return lib().mole_last_error().decode()


def mole_version() -> int:
    return lib().mole_version()


def mole_build_lut_workspace(V: int, d: int, D: int, N: int, dtype: int) -> int:
    return lib().mole_build_lut_workspace(V, d, D, N, dtype)


def mole_build_lut(E, W1, b1, W2, b2, norm_w, norm_eps: float, LUT, V: int, d: int, D: int, N: int,
                   dtype: int, act: int, workspace, stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().mole_build_lut(_ptr(E), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _ptr(norm_w), norm_eps,
                                _ptr(LUT), V, d, D, N, dtype, act, _ptr(workspace), wb, _stream(stream)))


def mole_dedup_workspace(T: int, V: int) -> int:
    return lib().mole_dedup_workspace(T, V)


def mole_dedup_ids(ids, T: int, V: int, uniq, inv, n_uniq, err_flag, workspace, stream=None,
                   workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().mole_dedup_ids(_ptr(ids), T, V, _ptr(uniq), _ptr(inv), _ptr(n_uniq), _ptr(err_flag),
                                _ptr(workspace), wb, _stream(stream)))


def mole_lookup_forward(table, ids, slot, h, W_r, shared_out, residual, out, gates_dbg, rows_dbg, err_flag,
                        T: int, rows: int, d: int, N: int, dtype: int, flags: int = 0, workspace=None,
                        stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().mole_lookup_forward(_ptr(table), _ptr(ids), _ptr(slot), _ptr(h), _ptr(W_r), _ptr(shared_out),
                                     _ptr(residual), _ptr(out), _ptr(gates_dbg), _ptr(rows_dbg), _ptr(err_flag),
                                     T, rows, d, N, dtype, flags, _ptr(workspace), wb, _stream(stream)))


def mole_lookup_forward_layers(table, table_stride: int, ids, slot, h, W_r, shared_out, residual, out,
                               act_stride: int, gates_dbg, rows_dbg, err_flag, L: int, T: int, rows: int,
                               d: int, N: int, dtype: int, flags: int = 0, workspace=None, stream=None,
                               workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().mole_lookup_forward_layers(_ptr(table), table_stride, _ptr(ids), _ptr(slot), _ptr(h), _ptr(W_r),
                                            _ptr(shared_out), _ptr(residual), _ptr(out), act_stride,
                                            _ptr(gates_dbg), _ptr(rows_dbg), _ptr(err_flag), L, T, rows, d, N,
                                            dtype, flags, _ptr(workspace), wb, _stream(stream)))


def mole_lookup_forward_noalloc(table, ids, h, W_r, shared_out, residual, out, err_flag, T: int, V: int, d: int, N: int,
                                dtype: int, stream=None) -> None:
    _check(lib().mole_lookup_forward_noalloc(_ptr(table), _ptr(ids), _ptr(h), _ptr(W_r), _ptr(shared_out),
                                             _ptr(residual), _ptr(out), _ptr(err_flag), T, V, d, N, dtype,
                                             _stream(stream)))


def mole_shared_ffn_workspace(T: int, d: int, D_s: int, N: int) -> int:
    return lib().mole_shared_ffn_workspace(T, d, D_s, N)


def mole_shared_ffn_forward(table, ids, slot, h, W_r, W1, b1, W2, b2, residual, out, gates_dbg, err_flag, T: int,
                            rows: int, d: int, D_s: int, N: int, dtype: int, act: int, workspace, stream=None,
                            workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().mole_shared_ffn_forward(_ptr(table), _ptr(ids), _ptr(slot), _ptr(h), _ptr(W_r), _ptr(W1), _ptr(b1),
                                         _ptr(W2), _ptr(b2), _ptr(residual), _ptr(out), _ptr(gates_dbg), _ptr(err_flag),
                                         T, rows, d, D_s, N, dtype, act, _ptr(workspace), wb, _stream(stream)))


def mole_set_tuning(name: str, value: int) -> None:
    _check(lib().mole_set_tuning(name.encode(), value))


def mole_layer_forward(table, table_stride: int, ids, slot, x, ln_w, ln_eps: float, W_r, shared_out, out,
                       act_stride: int, gates_dbg, rows_dbg, err_flag, L: int, T: int, rows: int, d: int, N: int,
                       dtype: int, flags: int = 0, workspace=None, stream=None,
                       workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().mole_layer_forward(_ptr(table), table_stride, _ptr(ids), _ptr(slot), _ptr(x), _ptr(ln_w), ln_eps,
                                    _ptr(W_r), _ptr(shared_out), _ptr(out), act_stride, _ptr(gates_dbg),
                                    _ptr(rows_dbg), _ptr(err_flag), L, T, rows, d, N, dtype, flags,
                                    _ptr(workspace), wb, _stream(stream)))


def mole_dedup_forward_workspace(T: int, V: int, N: int, L: int = 1) -> int:
    return lib().mole_dedup_forward_workspace(T, V, N, L)


def mole_dedup_forward(table, table_stride: int, ids, h, ln_w, ln_eps: float, W_r, shared_out, residual, out,
                       act_stride: int, uniq, inv, n_uniq, err_flag, L: int, T: int, V: int, d: int, N: int, dtype: int,
                       workspace, stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().mole_dedup_forward(_ptr(table), table_stride, _ptr(ids), _ptr(h), _ptr(ln_w), ln_eps, _ptr(W_r),
                                    _ptr(shared_out), _ptr(residual), _ptr(out), act_stride, _ptr(uniq), _ptr(inv),
                                    _ptr(n_uniq), _ptr(err_flag), L, T, V, d, N, dtype, _ptr(workspace), wb,
                                    _stream(stream)))


def mole_offload_fetch(host_table, host_layer_stride: int, uniq, n_uniq, staging, staging_layer_stride: int,
                       err_flag, L: int, U_cap: int, V: int, d: int, N: int, dtype: int, stream=None) -> None:
    _check(lib().mole_offload_fetch(_ptr(host_table), host_layer_stride, _ptr(uniq), _ptr(n_uniq), _ptr(staging),
                                    staging_layer_stride, _ptr(err_flag), L, U_cap, V, d, N, dtype,
                                    _stream(stream)))


def mole_offload_fetch_idmajor(host_table, uniq, n_uniq, staging, staging_layer_stride: int, err_flag, L: int,
                               U_cap: int, V: int, d: int, N: int, dtype: int, stream=None) -> None:
    _check(lib().mole_offload_fetch_idmajor(_ptr(host_table), _ptr(uniq), _ptr(n_uniq), _ptr(staging),
                                            staging_layer_stride, _ptr(err_flag), L, U_cap, V, d, N, dtype,
                                            _stream(stream)))


def mole_offload_fetch_nf(host_codes, host_codes_stride: int, host_scales, host_scales_stride: int, uniq, n_uniq,
                          staging_codes, staging_codes_stride: int, staging_scales, staging_scales_stride: int,
                          err_flag, L: int, U_cap: int, V: int, d: int, N: int, bits: int, block: int,
                          scale_bytes: int, stream=None) -> None:
    _check(lib().mole_offload_fetch_nf(_ptr(host_codes), host_codes_stride, _ptr(host_scales), host_scales_stride,
                                       _ptr(uniq), _ptr(n_uniq), _ptr(staging_codes), staging_codes_stride,
                                       _ptr(staging_scales), staging_scales_stride, _ptr(err_flag), L, U_cap, V, d, N,
                                       bits, block, scale_bytes, _stream(stream)))


def mole_lut_file_create(path: str, dtype: int, layout: int, L: int, V: int, N: int, d: int) -> int:
    """-> handle (an integer holding the mole_lut_file pointer)."""
    desc = LutDesc(dtype, layout, L, N, d, 0, V)
    handle = ctypes.c_void_p()
    _check(lib().mole_lut_file_create(os.fsencode(path), ctypes.byref(desc), ctypes.byref(handle)))
    return handle.value


def mole_lut_file_open(path: str):
    """-> (handle, LutDesc)."""
    desc = LutDesc()
    handle = ctypes.c_void_p()
    _check(lib().mole_lut_file_open(os.fsencode(path), ctypes.byref(handle), ctypes.byref(desc)))
    return handle.value, desc


def mole_lut_file_payload(handle: int) -> Optional[int]:
    """Address of the mapped table (host memory)."""
    return lib().mole_lut_file_payload(handle)


def mole_lut_file_write_layer(handle: int, layer: int, src_host, threads: int = 8) -> None:
    _check(lib().mole_lut_file_write_layer(handle, layer, _ptr(src_host), threads))


def mole_lut_file_read_rows(handle: int, ids_host, n: int, dst_host, threads: int = 8) -> None:
    _check(lib().mole_lut_file_read_rows(handle, _ptr(ids_host), n, _ptr(dst_host), threads))


def mole_lut_file_close(handle: Optional[int]) -> None:
    _check(lib().mole_lut_file_close(handle))


def mole_nf_codebook(bits: int):
    """The 2^bits NF levels as a list of floats (empty for an unsupported width)."""
    buf = (ctypes.c_float * 16)()
    n = lib().mole_nf_codebook(bits, ctypes.cast(buf, ctypes.c_void_p))
    return [buf[i] for i in range(n)]


def mole_nf_codes_bytes(rows: int, N: int, d: int, bits: int) -> int:
    return lib().mole_nf_codes_bytes(rows, N, d, bits)


def mole_nf_scales_bytes(rows: int, N: int, d: int, block: int, scale_bytes: int) -> int:
    return lib().mole_nf_scales_bytes(rows, N, d, block, scale_bytes)


def mole_quantize_lut(table, codes, scales, rows: int, N: int, d: int, bits: int, block: int, scale_bytes: int,
                      stream=None) -> None:
    _check(lib().mole_quantize_lut(_ptr(table), _ptr(codes), _ptr(scales), rows, N, d, bits, block, scale_bytes,
                                   _stream(stream)))


def mole_lookup_forward_nf(codes, codes_stride: int, scales, scales_stride: int, ids, slot, h, W_r, shared_out,
                           residual, out, act_stride: int, gates_dbg, rows_dbg, err_flag, L: int, T: int, rows: int,
                           d: int, N: int, bits: int, block: int, scale_bytes: int, flags: int = 0, workspace=None,
                           stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().mole_lookup_forward_nf(_ptr(codes), codes_stride, _ptr(scales), scales_stride, _ptr(ids), _ptr(slot),
                                        _ptr(h), _ptr(W_r), _ptr(shared_out), _ptr(residual), _ptr(out), act_stride,
                                        _ptr(gates_dbg), _ptr(rows_dbg), _ptr(err_flag), L, T, rows, d, N, bits, block,
                                        scale_bytes, flags, _ptr(workspace), wb, _stream(stream)))


def mole_layer_forward_nf(codes, codes_stride: int, scales, scales_stride: int, ids, slot, x, ln_w, ln_eps: float,
                          W_r, shared_out, out, act_stride: int, gates_dbg, rows_dbg, err_flag, L: int, T: int, rows: int,
                          d: int, N: int, bits: int, block: int, scale_bytes: int, flags: int = 0, workspace=None,
                          stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().mole_layer_forward_nf(_ptr(codes), codes_stride, _ptr(scales), scales_stride, _ptr(ids), _ptr(slot),
                                       _ptr(x), _ptr(ln_w), ln_eps, _ptr(W_r), _ptr(shared_out), _ptr(out), act_stride,
                                       _ptr(gates_dbg), _ptr(rows_dbg), _ptr(err_flag), L, T, rows, d, N, bits, block,
                                       scale_bytes, flags, _ptr(workspace), wb, _stream(stream)))
