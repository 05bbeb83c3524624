"""Shared helpers of the test-suite: numpy storage arrays <-> torch device tensors, tolerances."""
import numpy as np

from paper_2503_15798_amd import binding as mb
from paper_2503_15798_amd import workloads as wl

# Tolerances of the comparison |gpu - ref| <= atol + rtol * |ref| (element by element).
# bf16 storage with fp32 accumulation; fp32 throughout.
TOL = {wl.BF16: dict(rtol=2e-2, atol=1e-3), wl.F32: dict(rtol=1e-5, atol=1e-6)}
DT = {wl.F32: mb.MOLE_F32, wl.BF16: mb.MOLE_BF16}


def to_dev(a, dtype, device="cuda"):
    """numpy storage array (float32, or uint16 bf16 bits) -> torch tensor on the device."""
    import torch
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if dtype == wl.BF16 and a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_host(t, dtype):
    """torch tensor -> numpy storage array (uint16 bits for bf16)."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def assert_close(got_f64, ref_f64, dtype, what="", extra_atol=0.0):
    """extra_atol: an absolute allowance a test derives for an error source outside the forward itself
    (e.g. one storage ulp of an independently built table)."""
    tol = TOL[dtype]
    err = np.abs(got_f64 - ref_f64)
    lim = tol["atol"] + extra_atol + tol["rtol"] * np.abs(ref_f64)
    bad = err > lim
    if bad.any():
        i = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; worst at {i}: "
                             f"got {got_f64[i]!r}, ref {ref_f64[i]!r}, |err| {err[i]:.3e} > {lim[i]:.3e}")


def gathered_rows(tab_d, ids):
    """(rows [U, N, d] storage array on the host, inv [T] int32) for the distinct in-range ids of a batch:
    the rows of a device table that a forward over `ids` looks up, copied back by plain indexing (no
    library call), and the position of every token's row among them.  Lets the oracle run on tables that
    exist only on the device."""
    import torch
    ids = np.asarray(ids)
    uniq, inv = np.unique(ids, return_inverse=True)
    rows = tab_d[torch.from_numpy(uniq.astype(np.int64)).to(tab_d.device)]
    dtype = wl.BF16 if rows.dtype == torch.bfloat16 else wl.F32
    return to_host(rows, dtype), inv.astype(np.int32)
