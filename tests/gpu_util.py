"""Shared helpers of the GPU parity tests (they call the HIP library through the binding)."""
import numpy as np
import pytest
import torch


def require_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def dev(a, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if bf16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def host(t):
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


def say(*a):
    print(*a, flush=True)


def oracle_mask32(oracle, u_np, k):
    """The oracle's own thresholds and lifetimes for a score tensor [B,Gu,n].  The thresholds are rounded to fp32, the
    precision the kernels store them in, and widened back: the gates clip(u - tau) and the membership of a key in the
    strictly fractional set (a floating-point value deciding an integer) are then taken from the same numbers on both
    sides, and none of them comes from the GPU."""
    tau64, death = oracle.mask_all(u_np, k)
    return tau64.astype(np.float32).astype(np.float64), death


def kink_keys(u_np, tau_ref, tau_gpu):
    """Boolean [B,Gu,n]: keys whose membership in the fractional set {tau_T < u_j < tau_T + 1} could differ for some
    prefix T between the reference thresholds and the GPU's (both fp32 values).  The two arrays agree except where the
    fp64 roots straddle an fp32 rounding boundary, so the set is almost always empty; the du of such a key differs by
    one term of its sum and is compared at a looser bar by the callers."""
    B, Gu, n = u_np.shape
    out = np.zeros((B, Gu, n), bool)
    tg = tau_gpu.astype(np.float64)
    for b, g, T in zip(*np.nonzero(tg != tau_ref)):
        lo, hi = sorted((tg[b, g, T], tau_ref[b, g, T]))
        z = u_np[b, g, : T + 1].astype(np.float64)
        out[b, g, : T + 1] |= ((z >= lo) & (z <= hi)) | ((z - 1.0 >= lo) & (z - 1.0 <= hi))
    return out


def check_mask_against(tau_gpu, death_gpu, tau_ref, death_ref):
    """thresholds within 1e-5 (relative to max(1,|ref|)), lifetimes bit-exact"""
    np.testing.assert_array_equal(death_gpu, death_ref)
    err = np.abs(tau_gpu.astype(np.float64) - tau_ref) / np.maximum(1.0, np.abs(tau_ref))
    assert err.max() <= 1e-5, err.max()
