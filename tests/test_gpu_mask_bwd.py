"""GPU parity of sparsek_mask_bwd (gradient w.r.t. the scores) against the CPU oracle.

The reference is computed from the oracle's own thresholds and lifetimes (nothing of the GPU's
enters it); the thresholds are rounded to fp32, the precision the kernels keep them in, because
the membership of a key in the strictly fractional set S* is decided from them.  Keys whose
membership could differ where the two sides' fp32 thresholds differ are listed (almost always
none), must be few, and are held to a looser bar.  Bars: |du - ref| <= 1e-2 max|ref| for
bf16 tensors (the stored bf16 output O enters dO.O with relative error 2^-9), 2e-4 max|ref|
for fp32.  The sum of du over a row must vanish (rows of the SPARSEK Jacobian sum to 0).
"""
import numpy as np
import pytest
import torch

import paper_2406_16747_amd as spk
from paper_2406_16747_amd import synth
from gpu_util import check_mask_against, dev, host, kink_keys, oracle_mask32, require_gpu, say

pytestmark = pytest.mark.gpu


def run_bwd(oracle, inp, gate_mode, heads_all=True):
    B, H, n, d, k, w, Gu = (inp[x] for x in ("B", "H", "n", "d", "k", "w", "Gu"))
    bf16 = inp["dtype"] == "bf16"
    u = dev(inp["u"])
    Q, K, V, dO = (dev(inp[x], bf16) for x in ("Q", "K", "V", "dO"))
    tau, death = spk.sparsek_mask(u, k)
    o, lse = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, k, w, gate_mode, 1.0)
    du = spk.sparsek_mask_bwd(Q, K, V, u, tau, death, o, lse, dO, k, w, gate_mode, 1.0)
    torch.cuda.synchronize()
    du = host(du)
    assert np.isfinite(du).all()
    tau_r, death_r = oracle_mask32(oracle, inp["u"], k)
    check_mask_against(host(tau), host(death), tau_r, death_r)
    ref, _ = oracle.mask_bwd(inp["Q32"], inp["K32"], inp["V32"], inp["u"], tau_r, death_r, inp["dO32"], k, w,
                             gate_mode, 1.0)
    kink = kink_keys(inp["u"], tau_r, host(tau))
    assert kink.sum() <= 4, kink.sum()
    scale = np.abs(ref).max()
    diff = np.abs(du - ref)
    err = diff[~kink].max()
    tol = (1e-2 if bf16 else 2e-4) * scale
    assert err <= tol + 1e-30, (err, scale)
    assert diff.max() <= 0.2 * scale + 1e-30
    if scale > 0:
        assert np.abs(du.sum(-1)).max() <= 1e-3 * scale * np.sqrt(n)
    return err / max(scale, 1e-30), scale


@pytest.mark.parametrize("n,d,k,w,Gu,dtype", [
    (200, 64, 12, 9, 1, "bf16"), (333, 128, 20, 0, 1, "bf16"), (520, 64, 30, 40, 2, "bf16"),
    (300, 32, 10, 7, 2, "fp32"), (90, 64, 100, 5, 1, "bf16"), (150, 64, 0, 5, 1, "bf16"), (64, 64, 3, 70, 1, "bf16"),
    # more than 1024 candidates per query block: the compaction runs over several segments
    (2500, 64, 1150, 40, 1, "bf16"), (1700, 128, 300, 1000, 1, "bf16"),
])
@pytest.mark.parametrize("gate_mode", [0, 1, 2, 3])
def test_mask_bwd_small(oracle, n, d, k, w, Gu, dtype, gate_mode):
    require_gpu()
    say("mask_bwd", n, d, k, w, Gu, dtype, gate_mode)
    inp = synth.make(3, Gu=Gu, seed=n + k, with_dO=True, B=2, H=2, n=n, d=d, k=k, w=w, dtype=dtype,
                     qk_div=float(np.sqrt(d)) / 4)
    rel, scale = run_bwd(oracle, inp, gate_mode)
    if gate_mode == 2 or k == 0 or n <= w or k >= n:
        assert scale == 0.0


def test_mask_bwd_config3_recipe_reduced(oracle):
    """Config 3 recipe (drifting scores, k=w=512 at n=8192 scaled down 4x), one batch, 2 heads."""
    require_gpu()
    say("mask_bwd config 3 reduced")
    inp = synth.make(3, with_dO=True, B=1, H=2, n=2048, k=128, w=128)
    run_bwd(oracle, inp, 0)


def test_straight_through_forward_is_the_ungated_forward_and_has_a_gradient(oracle):
    """gate_mode 3 (straight-through, Sec. 3.4): the forward skips the gates (bit-identical to
    mode 2); the score gradient is that of the oracle's mode 3, and differs from the soft one."""
    require_gpu()
    say("mask_bwd straight-through")
    inp = synth.make(3, with_dO=True, B=1, H=2, n=1536, k=96, w=64, seed=5)
    B, H, n, d, k, w = (inp[x] for x in ("B", "H", "n", "d", "k", "w"))
    u = dev(inp["u"])
    Q, K, V, dO = (dev(inp[x], True) for x in ("Q", "K", "V", "dO"))
    tau, death = spk.sparsek_mask(u, k)
    o2, lse2 = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, k, w, 2, 1.0)
    o3, lse3 = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, k, w, 3, 1.0)
    assert torch.equal(o2, o3) and torch.equal(lse2, lse3)
    rel3, scale3 = run_bwd(oracle, inp, 3)
    assert scale3 > 0
    du3 = host(spk.sparsek_mask_bwd(Q, K, V, u, tau, death, o3, lse3, dO, k, w, 3, 1.0))
    o0, lse0 = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, k, w, 0, 1.0)
    du0 = host(spk.sparsek_mask_bwd(Q, K, V, u, tau, death, o0, lse0, dO, k, w, 0, 1.0))
    assert np.abs(du3 - du0).max() > 1e-2 * scale3


def test_two_runs_agree_du_at_rounding_level_the_other_gradients_bitwise():
    """du adds the heads of a score group and the query blocks with fp32 atomics, so its bits depend on the order
    in which workgroups arrive: two runs may differ at rounding level (1e-5 of the gradient's scale allowed).  dq,
    dk and dv use no atomics and must be bitwise equal."""
    require_gpu()
    say("backward run twice")
    inp = synth.make(3, with_dO=True, B=2, H=4, n=2048, k=128, w=128, seed=21)
    k, w = inp["k"], inp["w"]
    u = dev(inp["u"])
    Q, K, V, dO = (dev(inp[x], True) for x in ("Q", "K", "V", "dO"))
    tau, death = spk.sparsek_mask(u, k)
    o, lse = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, k, w, 0, 1.0)
    du_a = spk.sparsek_mask_bwd(Q, K, V, u, tau, death, o, lse, dO, k, w, 0, 1.0).clone()
    g_a = [t.clone() for t in spk.sparsek_attn_bwd(Q, K, V, u, tau, death, o, lse, dO, k, w, 0, 1.0)]
    du_b = spk.sparsek_mask_bwd(Q, K, V, u, tau, death, o, lse, dO, k, w, 0, 1.0)
    g_b = spk.sparsek_attn_bwd(Q, K, V, u, tau, death, o, lse, dO, k, w, 0, 1.0)
    torch.cuda.synchronize()
    scale = float(du_a.abs().max())
    assert scale > 0
    assert float((du_a - du_b).abs().max()) <= 1e-5 * scale
    for a, b in zip(g_a, g_b):
        assert torch.equal(a, b)
