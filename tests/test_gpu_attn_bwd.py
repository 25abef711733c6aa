"""GPU parity of sparsek_attn_bwd (gradients with respect to q, k, v) against the CPU oracle.

Bars: |g - ref| <= 1e-2 max|ref| per tensor for bf16 storage (outputs are rounded to bf16, the
stored bf16 O enters D = dO.O with relative error 2^-9), <= 2e-4 max|ref| for fp32.  The reference
is computed from the oracle's own thresholds (rounded to fp32, the precision the kernels keep them in) and lifetimes.
"""
import numpy as np
import pytest
import torch

import paper_2406_16747_amd as spk
from paper_2406_16747_amd import synth
from gpu_util import check_mask_against, dev, host, kink_keys, oracle_mask32, require_gpu, say

pytestmark = pytest.mark.gpu


def run_bwd(oracle, inp, gate_mode, heads=None):
    B, H, n, d, k, w, Gu = (inp[x] for x in ("B", "H", "n", "d", "k", "w", "Gu"))
    bf16 = inp["dtype"] == "bf16"
    u = dev(inp["u"])
    Q, K, V, dO = (dev(inp[x], bf16) for x in ("Q", "K", "V", "dO"))
    tau, death = spk.sparsek_mask(u, k)
    o, lse = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, k, w, gate_mode, inp["scale"])
    dq, dk, dv = spk.sparsek_attn_bwd(Q, K, V, u, tau, death, o, lse, dO, k, w, gate_mode, inp["scale"])
    torch.cuda.synchronize()
    got = [host(x) for x in (dq, dk, dv)]
    tau_r, death_r = oracle_mask32(oracle, inp["u"], k)
    check_mask_against(host(tau), host(death), tau_r, death_r)
    ref = oracle.attn_bwd(inp["Q32"], inp["K32"], inp["V32"], inp["u"], tau_r, death_r,
                          inp["dO32"], k, w, gate_mode, inp["scale"])
    worst = 0.0
    common = max(np.abs(r).max() for r in ref)
    for name, g, r in zip(("dq", "dk", "dv"), got, ref):
        assert np.isfinite(g).all(), name
        # a tensor whose exact gradient (nearly) vanishes, e.g. dq with a single key, is held to the others' scale
        scale = max(np.abs(r).max(), 1e-3 * common)
        err = np.abs(g - r).max()
        tol = (1e-2 if bf16 else 2e-4) * scale
        assert err <= tol + 1e-30, (name, err, scale, np.unravel_index(np.abs(g - r).argmax(), g.shape))
        worst = max(worst, err / max(scale, 1e-30))
    return worst


@pytest.mark.parametrize("n,d,k,w,Gu,dtype", [
    (200, 64, 12, 9, 1, "bf16"), (333, 128, 20, 0, 1, "bf16"), (520, 64, 30, 40, 2, "bf16"),
    (300, 32, 10, 7, 2, "fp32"), (90, 64, 100, 5, 1, "bf16"), (150, 64, 0, 5, 1, "bf16"), (64, 64, 3, 70, 1, "bf16"),
    (1, 64, 4, 4, 1, "bf16"), (257, 128, 16, 16, 1, "fp32"),
])
@pytest.mark.parametrize("gate_mode", [0, 1, 2, 3])
def test_attn_bwd_small(oracle, n, d, k, w, Gu, dtype, gate_mode):
    require_gpu()
    say("attn_bwd", n, d, k, w, Gu, dtype, gate_mode)
    inp = synth.make(3, Gu=Gu, seed=n + k, with_dO=True, B=2, H=2, n=n, d=d, k=k, w=w, dtype=dtype,
                     qk_div=float(np.sqrt(d)) / 4)
    run_bwd(oracle, inp, gate_mode)


def test_attn_bwd_config3_recipe_reduced(oracle):
    """Config 3 recipe (drifting scores, k=w=512 at n=8192 scaled down 4x), one batch, 2 heads."""
    require_gpu()
    say("attn_bwd config 3 reduced")
    inp = synth.make(3, with_dO=True, B=1, H=2, n=2048, k=128, w=128)
    run_bwd(oracle, inp, 0)


@pytest.mark.parametrize("n,d,k,w,Gu,gate_mode", [
    # a top-k list that spans two metadata segments of the dQ kernel and many blocks of selected keys
    (2600, 128, 1500, 256, 1, 0), (2600, 128, 1500, 256, 1, 1),
    # d = 64 with one score row per head, ragged tail, window narrower than a query tile
    (1500, 64, 300, 40, 2, 0), (1500, 64, 300, 40, 2, 3),
    # selection only (w = 0) and window only (k = 0) on the MFMA path
    (1100, 128, 200, 0, 1, 0), (1100, 64, 0, 300, 1, 2),
])
def test_attn_bwd_medium(oracle, n, d, k, w, Gu, gate_mode):
    require_gpu()
    say("attn_bwd medium", n, d, k, w, Gu, gate_mode)
    inp = synth.make(3, Gu=Gu, seed=3 * n + k, with_dO=True, B=1, H=2, n=n, d=d, k=k, w=w, dtype="bf16",
                     qk_div=float(np.sqrt(d)) / 2)
    run_bwd(oracle, inp, gate_mode)


@pytest.mark.parametrize("gate_mode", [0, 1, 3])
def test_one_call_backward_equals_the_two_parts(oracle, gate_mode):
    """sparsek_bwd = sparsek_attn_bwd + sparsek_mask_bwd, bit for bit (dq, dk, dv; du accumulates with atomics
    across heads, so it is compared to rounding), and all four gradients of the one call against the oracle."""
    require_gpu()
    say("one-call backward", gate_mode)
    inp = synth.make(3, seed=77, with_dO=True, B=2, H=2, n=700, d=64, k=40, w=30, dtype="bf16", qk_div=2.0)
    u = dev(inp["u"])
    Q, K, V, dO = (dev(inp[x], True) for x in ("Q", "K", "V", "dO"))
    tau, death = spk.sparsek_mask(u, 40)
    o, lse = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, 40, 30, gate_mode, 1.0)
    dq, dk, dv = spk.sparsek_attn_bwd(Q, K, V, u, tau, death, o, lse, dO, 40, 30, gate_mode, 1.0)
    du = spk.sparsek_mask_bwd(Q, K, V, u, tau, death, o, lse, dO, 40, 30, gate_mode, 1.0)
    dq2, dk2, dv2, du2 = spk.sparsek_bwd(Q, K, V, u, tau, death, o, lse, dO, 40, 30, gate_mode, 1.0)
    torch.cuda.synchronize()
    for a, b in ((dq, dq2), (dk, dk2), (dv, dv2)):
        assert torch.equal(a, b)
    scale = float(du.abs().max())
    assert scale > 0 and float((du - du2).abs().max()) <= 1e-5 * scale
    tau_r, death_r = oracle_mask32(oracle, inp["u"], 40)
    check_mask_against(host(tau), host(death), tau_r, death_r)
    kink = kink_keys(inp["u"], tau_r, host(tau))
    assert kink.sum() <= 4
    args = (inp["Q32"], inp["K32"], inp["V32"], inp["u"], tau_r, death_r, inp["dO32"], 40, 30, gate_mode, 1.0)
    ref = list(oracle.attn_bwd(*args)) + [oracle.mask_bwd(*args)[0]]
    for name, g, r in zip(("dq", "dk", "dv", "du"), (dq2, dk2, dv2, du2), ref):
        rs = np.abs(r).max()
        diff = np.abs(host(g) - r)
        if name == "du":
            diff = diff[~kink]
        assert rs > 0 and diff.max() <= 1e-2 * rs, (name, diff.max(), rs)


def test_one_call_backward_fp32_generic_path(oracle):
    """sparsek_bwd on the generic (fp32) kernels against the oracle's two gradients."""
    require_gpu()
    say("one-call backward fp32")
    inp = synth.make(3, seed=91, with_dO=True, B=1, H=2, n=300, d=32, k=24, w=20, dtype="fp32", qk_div=2.0)
    u = dev(inp["u"])
    Q, K, V, dO = (dev(inp[x], False) for x in ("Q", "K", "V", "dO"))
    tau, death = spk.sparsek_mask(u, 24)
    o, lse = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, 24, 20, 0, inp["scale"])
    got = [host(x) for x in spk.sparsek_bwd(Q, K, V, u, tau, death, o, lse, dO, 24, 20, 0, inp["scale"])]
    tau_r, death_r = oracle_mask32(oracle, inp["u"], 24)
    check_mask_against(host(tau), host(death), tau_r, death_r)
    assert not kink_keys(inp["u"], tau_r, host(tau)).any()
    ref = list(oracle.attn_bwd(inp["Q32"], inp["K32"], inp["V32"], inp["u"], tau_r, death_r, inp["dO32"], 24, 20, 0,
                               inp["scale"]))
    ref.append(oracle.mask_bwd(inp["Q32"], inp["K32"], inp["V32"], inp["u"], tau_r, death_r, inp["dO32"], 24, 20, 0,
                               inp["scale"])[0])
    for name, g, r in zip(("dq", "dk", "dv", "du"), got, ref):
        scale = np.abs(r).max()
        assert scale > 0 and np.abs(g - r).max() <= 2e-4 * scale, (name, np.abs(g - r).max(), scale)
