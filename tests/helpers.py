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


def folded_router(ln_w, W_r, dtype, d):
    """(unit norm weight, router weight with the norm weight folded in and rounded to the storage type):
    what mole_fold_router_norm stores, computed on the host -- the product of two stored values rounded
    once has the same bits either way.  The outputs of the fused-norm calls are compared with the oracle
    on these (the rounding of the folded weight shifts the gates within their tolerance, which can exceed
    atol on an output where state, shared and routed terms cancel)."""
    import numpy as np
    from paper_2503_15798_amd import workloads as wl
    folded = wl.to_storage(wl.storage_to_f64(ln_w, dtype)[:, None] * wl.storage_to_f64(W_r, dtype), dtype)
    return wl.to_storage(np.ones(d), dtype), folded


def fold_gate_allowance(x, ln_w, W_r, eps, dtype, ref_g):
    """Absolute allowance [T, N] on the gates of a fused-norm call against the layer with the UNFOLDED norm
    weight: every element of the folded weight carries an independent rounding error of at most one unit
    roundoff u of the storage type (standard deviation at most u |w| / sqrt 3), so logit j of a token
    moves by a sum of d independent terms; six standard deviations of it, and |dg_j| <= 2 g_j max_j |dz_j|
    to first order."""
    import numpy as np
    from paper_2503_15798_amd import workloads as wl
    u = 2.0 ** -9 if dtype == wl.BF16 else 2.0 ** -24
    x64 = wl.storage_to_f64(x, dtype)
    xn = x64 / np.sqrt((x64 ** 2).mean(axis=1, keepdims=True) + eps)
    wf = wl.storage_to_f64(ln_w, dtype)[:, None] * wl.storage_to_f64(W_r, dtype)
    dz = 6.0 * u / np.sqrt(3.0) * np.sqrt((xn ** 2) @ (wf ** 2))
    return 2.0 * dz.max(axis=1, keepdims=True) * ref_g
