"""ctypes front-end of the fp64 CPU oracle (oracle/mole_oracle.c).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
CPU-baseline leg may import this; the product package never does.  Nothing here
touches the HIP library, and the arithmetic all lives in the C file.

Tensors are numpy arrays in storage format: float32, float64, or uint16 holding
bfloat16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mole_oracle.c")
_LIB = os.path.join(_HERE, "libmole_oracle.so")

GELU_ERF, GELU_TANH = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE arithmetic: no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.mole_oracle_gelu.restype = ctypes.c_double
        _lib.mole_oracle_gelu.argtypes = [ctypes.c_double, ctypes.c_int]
    return _lib


def threads() -> int:
    """Number of threads the oracle's parallel loops use (OpenMP default = visible cores)."""
    n = os.environ.get("OMP_NUM_THREADS")
    if n:
        return int(n.split(",")[0])
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def _code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    if a.dtype == np.float64:
        return 2
    raise TypeError(f"unsupported storage dtype {a.dtype}")


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _same(*arrs) -> int:
    codes = {_code(a) for a in arrs if a is not None}
    if len(codes) != 1:
        raise TypeError("tensors that share a dtype argument must have one storage dtype")
    return codes.pop()


def gelu(x: float, act: int = GELU_ERF) -> float:
    return float(lib().mole_oracle_gelu(float(x), int(act)))


def gates(h: np.ndarray, W_r: np.ndarray) -> np.ndarray:
    """Router equation: softmax over all N experts of h @ W_r.  h [T,d], W_r [d,N] -> [T,N] fp64."""
    T, d = h.shape
    d2, N = W_r.shape
    assert d == d2
    h = np.ascontiguousarray(h)
    W_r = np.ascontiguousarray(W_r)
    g = np.empty((T, N), dtype=np.float64)
    rc = lib().mole_oracle_gates(_p(h), _code(h), _p(W_r), _code(W_r),
                                 ctypes.c_int64(T), d, N, _p(g))
    if rc:
        raise RuntimeError(f"mole_oracle_gates rc={rc}")
    return g


def lookup_forward(table: np.ndarray, ids: np.ndarray, h: np.ndarray, W_r: np.ndarray,
                   shared: Optional[np.ndarray] = None, residual: Optional[np.ndarray] = None
                   ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """Inference-layer equation.  Returns (out [T,d] fp64, gates [T,N] fp64, rows [T] int64, err)."""
    V, N, d = table.shape
    T = int(ids.shape[0])
    assert h.shape == (T, d) and W_r.shape == (d, N)
    table = np.ascontiguousarray(table)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    h, W_r = np.ascontiguousarray(h), np.ascontiguousarray(W_r)
    shared = None if shared is None else np.ascontiguousarray(shared)
    residual = None if residual is None else np.ascontiguousarray(residual)
    act = _same(h, W_r, shared, residual)
    out = np.empty((T, d), dtype=np.float64)
    g = np.empty((T, N), dtype=np.float64)
    rows = np.empty((T,), dtype=np.int64)
    err = ctypes.c_int32(0)
    rc = lib().mole_oracle_lookup_forward(
        _p(table), _code(table), _p(ids), _p(h), _p(W_r), _p(shared), _p(residual), act,
        ctypes.c_int64(T), ctypes.c_int64(V), d, N, _p(out), _p(g), _p(rows), ctypes.byref(err))
    if rc:
        raise RuntimeError(f"mole_oracle_lookup_forward rc={rc}")
    return out, g, rows, int(err.value)


def layer_forward(table: np.ndarray, ids: np.ndarray, x: np.ndarray, ln_w: np.ndarray, eps: float,
                  W_r: np.ndarray, shared: Optional[np.ndarray] = None
                  ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray, int]:
    """MoLE part of the inference listing from the post-attention state x (norm, router, lookup, adds).
    Returns (out [T,d], gates [T,N], hn [T,d] (the normed state), rows [T], err)."""
    V, N, d = table.shape
    T = int(ids.shape[0])
    assert x.shape == (T, d) and W_r.shape == (d, N) and ln_w.shape == (d,)
    table = np.ascontiguousarray(table)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    x, W_r, ln_w = np.ascontiguousarray(x), np.ascontiguousarray(W_r), np.ascontiguousarray(ln_w)
    shared = None if shared is None else np.ascontiguousarray(shared)
    act = _same(x, W_r, ln_w, shared)
    out = np.empty((T, d), dtype=np.float64)
    g = np.empty((T, N), dtype=np.float64)
    hn = np.empty((T, d), dtype=np.float64)
    rows = np.empty((T,), dtype=np.int64)
    err = ctypes.c_int32(0)
    rc = lib().mole_oracle_layer_forward(
        _p(table), _code(table), _p(ids), _p(x), _p(ln_w), ctypes.c_double(eps), _p(W_r), _p(shared), act,
        ctypes.c_int64(T), ctypes.c_int64(V), d, N, _p(out), _p(g), _p(hn), _p(rows), ctypes.byref(err))
    if rc:
        raise RuntimeError(f"mole_oracle_layer_forward rc={rc}")
    return out, g, hn, rows, int(err.value)


def dedup(ids: np.ndarray, V: int) -> Tuple[np.ndarray, np.ndarray, int, int]:
    """Canonical dedup map.  Returns (uniq [U] ascending, inv [T], U, err)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T = int(ids.shape[0])
    uniq = np.empty((max(T, 1),), dtype=np.int32)
    inv = np.empty((max(T, 1),), dtype=np.int32)
    U = ctypes.c_int32(0)
    err = ctypes.c_int32(0)
    rc = lib().mole_oracle_dedup(_p(ids), ctypes.c_int64(T), ctypes.c_int64(V),
                                 _p(uniq), _p(inv), ctypes.byref(U), ctypes.byref(err))
    if rc:
        raise RuntimeError(f"mole_oracle_dedup rc={rc}")
    return uniq[:U.value].copy(), inv[:T].copy(), int(U.value), int(err.value)


def build_lut(E: np.ndarray, W1: np.ndarray, W2: np.ndarray,
              b1: Optional[np.ndarray] = None, b2: Optional[np.ndarray] = None,
              norm_w: Optional[np.ndarray] = None, norm_eps: float = 1e-5,
              act: int = GELU_ERF, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """LUT entry equation for the vocabulary rows in `rows` (all rows when None).
    E [V,d], W1 [N,d,D], W2 [N,D,d] -> [n_rows, N, d] fp64."""
    V, d = E.shape
    N, d2, D = W1.shape
    assert d2 == d and W2.shape == (N, D, d)
    arrs = [np.ascontiguousarray(a) if a is not None else None for a in (E, W1, b1, W2, b2, norm_w)]
    E, W1, b1, W2, b2, norm_w = arrs
    dt = _same(*arrs)
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        n_rows = int(rows.shape[0])
    else:
        n_rows = V
    out = np.empty((n_rows, N, d), dtype=np.float64)
    rc = lib().mole_oracle_build_lut(
        _p(E), _p(W1), _p(b1), _p(W2), _p(b2), _p(norm_w), ctypes.c_double(norm_eps), dt,
        ctypes.c_int64(V), d, D, N, int(act), _p(rows), ctypes.c_int64(n_rows), _p(out))
    if rc:
        raise RuntimeError(f"mole_oracle_build_lut rc={rc}")
    return out


def shared_ffn(x: np.ndarray, W1: np.ndarray, W2: np.ndarray, b1: Optional[np.ndarray] = None,
               b2: Optional[np.ndarray] = None, act: int = GELU_ERF) -> np.ndarray:
    """Shared expert: GELU(x @ W1.T + b1) @ W2.T + b2.  x [T,d], W1 [D,d], W2 [d,D] (linear-layer weights as
    stored, [out, in]) -> [T,d] fp64."""
    T, d = x.shape
    D, d2 = W1.shape
    assert d2 == d and W2.shape == (d, D)
    arrs = [np.ascontiguousarray(a) if a is not None else None for a in (x, W1, b1, W2, b2)]
    x, W1, b1, W2, b2 = arrs
    dt = _same(*arrs)
    out = np.empty((T, d), dtype=np.float64)
    rc = lib().mole_oracle_shared_ffn(_p(x), _p(W1), _p(b1), _p(W2), _p(b2), dt, ctypes.c_int64(T), d, D, int(act),
                                      _p(out))
    if rc:
        raise RuntimeError(f"mole_oracle_shared_ffn rc={rc}")
    return out


def _f64(a: Optional[np.ndarray]) -> Optional[np.ndarray]:
    """Storage array (float32, float64 or bf16 bits) widened exactly to fp64."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def layer_with_shared_ffn(table: np.ndarray, ids: np.ndarray, h: np.ndarray, W_r: np.ndarray,
                          W1: np.ndarray, W2: np.ndarray, b1: Optional[np.ndarray] = None,
                          b2: Optional[np.ndarray] = None, residual: Optional[np.ndarray] = None,
                          act: int = GELU_ERF) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """Inference-layer equation with the shared expert evaluated here: sum_j g_j v_j + FFN_shared(h) + residual.
    The shared term stays in fp64 between the two steps.  Returns (out, gates, rows, err)."""
    h64 = _f64(h)      # widened once: the C loops then read doubles instead of converting per multiply
    shared = shared_ffn(h64, _f64(W1), _f64(W2), _f64(b1), _f64(b2), act)
    return lookup_forward(table, ids, h64, _f64(W_r), shared, _f64(residual))
