"""sparsek_mask_static (the entry point that allocates nothing) against sparsek_mask, through the raw C ABI.

Both run the same kernels, so thresholds and lifetimes must agree bit for bit (the bar for integer work, and tighter
than the 1e-5 bar of the thresholds).  Two calls in a row share the library's built-in scratch array; the second is
smaller, so stale contents of the first would show.
"""
import ctypes

import numpy as np
import pytest
import torch

import paper_2406_16747_amd as spk
from gpu_util import require_gpu, say

pytestmark = pytest.mark.gpu


def both(L, u, k):
    B, Gu, n = u.shape
    cfg = spk.SparsekCfg(B=B, H=Gu, Gu=Gu, n=n, d=64, k=k, w=1, dtype=spk.F32, gate_mode=0, softmax_scale=1.0)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # every buffer exists before the call under test
    tau_a, tau_b = torch.empty_like(u), torch.full_like(u, float("nan"))
    death_a = torch.empty(u.shape, dtype=torch.int32, device=u.device)
    death_b = torch.full(u.shape, -7, dtype=torch.int32, device=u.device)
    ws = torch.empty(L.sparsek_mask_workspace_bytes(ctypes.byref(cfg)), dtype=torch.uint8, device=u.device)
    assert L.sparsek_mask(ctypes.byref(cfg), p(u), p(tau_a), p(death_a), p(ws), ws.numel(), st) == 0
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = L.sparsek_mask_static(ctypes.byref(cfg), p(u), p(tau_b), p(death_b), st)
    assert rc == 0, L.sparsek_strerror(rc)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return (tau_a, death_a), (tau_b, death_b)


def test_static_scratch_entry_point_matches_sparsek_mask():
    require_gpu()
    L = spk.lib()
    g = torch.Generator(device="cpu").manual_seed(77)
    for (B, Gu, n, k) in ((2, 3, 9000, 300), (1, 2, 1500, 64)):  # second call smaller: fewer rows, fewer super-blocks
        say("mask_static case", B, Gu, n, k)
        u = torch.randn((B, Gu, n), generator=g, dtype=torch.float32).cuda()
        (tau_a, death_a), (tau_b, death_b) = both(L, u, k)
        assert torch.equal(death_a, death_b)
        assert torch.equal(tau_a, tau_b)
        assert not torch.isnan(tau_b).any()


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    require_gpu()
    L = spk.lib()
    one = ctypes.c_void_p(256)  # never dereferenced: the size check comes first
    null = ctypes.c_void_p(0)
    big = spk.SparsekCfg(B=1, H=4000, Gu=4000, n=2048 * 8, d=64, k=16, w=1, dtype=spk.F32, gate_mode=0, softmax_scale=1.0)
    assert L.sparsek_mask_workspace_bytes(ctypes.byref(big)) > 65536
    assert L.sparsek_mask_static(ctypes.byref(big), one, one, one, null) == -6
    assert b"scratch" in L.sparsek_strerror(-6)
    bad = spk.SparsekCfg(B=1, H=2, Gu=3, n=100, d=64, k=16, w=1, dtype=spk.F32, gate_mode=0, softmax_scale=1.0)
    assert L.sparsek_mask_static(ctypes.byref(bad), one, one, one, null) == -1
    ok = spk.SparsekCfg(B=1, H=2, Gu=2, n=100, d=64, k=16, w=1, dtype=spk.F32, gate_mode=0, softmax_scale=1.0)
    assert L.sparsek_mask_static(ctypes.byref(ok), null, one, one, null) == -1
