"""GPU parity of the decode step (sparsek_decode_init/load/step/status) against the oracle.

The oracle's decode is "row t of the prefill attention over the whole history", so these
tests also check the paper's claim that incremental evaluation with a k+w cache gives
exactly the full-history result.
"""
import numpy as np
import pytest
import torch

import paper_2406_16747_amd as spk
from paper_2406_16747_amd import synth
from gpu_util import dev, host, require_gpu, say

pytestmark = pytest.mark.gpu


def history(rng, B, H, Gu, n, d, dtype, ties=False):
    div = np.float32(np.sqrt(d) / 4.0)  # moderately peaky softmax
    out = {}
    for name in ("Q", "K", "V"):
        x = rng.standard_normal((B, H, n, d), dtype=np.float32) / (div if name != "V" else np.float32(1))
        out[name], out[name + "32"] = synth._store(x, dtype)
    u = rng.standard_normal((B, Gu, n), dtype=np.float32)
    if ties:
        u = (np.round(u * 3) / 3).astype(np.float32)
    out["u"] = u
    return out


def run_decode(oracle, B, H, Gu, d, k, w, n_ctx, steps, dtype="bf16", gate_mode=0, ties=False, cand_cap=0,
               seed=0, check_heads=None):
    rng = np.random.default_rng(seed)
    n = n_ctx + steps
    hist = history(rng, B, H, Gu, n, d, dtype, ties)
    bf16 = dtype == "bf16"
    tdt = torch.bfloat16 if bf16 else torch.float32
    Q, K, V = (dev(hist[x], bf16) for x in ("Q", "K", "V"))
    u = dev(hist["u"])
    state = spk.DecodeState(B, H, Gu, d, k, w, tdt, gate_mode, 1.0, cand_cap)
    state.buf.fill_(255)  # NaN patterns everywhere: init/load must not rely on fresh memory
    if n_ctx == 0:
        spk.sparsek_decode_init(state)
    else:
        u_ctx = u[:, :, :n_ctx].contiguous()
        tau, death = spk.sparsek_mask(u_ctx, k)
        spk.sparsek_decode_load(state, K[:, :, :n_ctx].contiguous(), V[:, :, :n_ctx].contiguous(), u_ctx, tau, death)
    outs = []
    for s in range(steps):
        t = n_ctx + s
        o = spk.sparsek_decode_step(state, Q[:, :, t].contiguous(), K[:, :, t].contiguous(),
                                    V[:, :, t].contiguous(), u[:, :, t].contiguous())
        outs.append(o)
    torch.cuda.synchronize()
    og = np.stack([host(o) for o in outs], axis=2)  # [B,H,steps,d]
    flags = spk.sparsek_decode_status(state)
    heads = check_heads or [(b, h) for b in range(B) for h in range(H)]
    worst = 0.0
    for (b, h) in heads:
        g = 0 if Gu == 1 else h
        ref = oracle.decode_bydef(hist["Q32"][b, h, n_ctx:], hist["K32"][b, h], hist["V32"][b, h], hist["u"][b, g],
                                  n_ctx, k, w, gate_mode, 1.0)
        err = np.abs(og[b, h] - ref).max()
        scale = np.abs(ref).max()
        worst = max(worst, err / scale)
        if bf16:
            assert err <= 1e-2 * max(1.0, scale) and err <= scale * 2.0 ** -7, (b, h, err, scale)
        else:
            assert err <= 2e-5 * scale, (b, h, err, scale)
    return state, og, flags, hist


@pytest.mark.parametrize("Gu", [1, 2])
@pytest.mark.parametrize("k,w", [(8, 6), (5, 0), (0, 7), (1, 1), (40, 3)])
def test_decode_from_empty(oracle, k, w, Gu):
    require_gpu()
    say("decode from empty", k, w, Gu)
    _, _, flags, _ = run_decode(oracle, 2, 2, Gu, 64, k, w, 0, 90, ties=(k == 5), seed=k * 10 + w)
    assert not flags.any()


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("fp32", 32), ("bf16", 64)])
@pytest.mark.parametrize("gate_mode", [0, 1, 2, 3])
def test_decode_after_prefill(oracle, dtype, d, gate_mode):
    require_gpu()
    say("decode after prefill", dtype, d, gate_mode)
    _, _, flags, _ = run_decode(oracle, 1, 3, 3 if d == 64 else 1, d, 24, 20, 400, 60, dtype, gate_mode, seed=d)
    assert not flags.any()


@pytest.mark.parametrize("n_ctx", [1, 5, 19, 20, 21, 44, 45])
def test_decode_load_boundaries(oracle, n_ctx):
    """Contexts shorter than w, than k+w, and just past them."""
    require_gpu()
    say("decode boundaries", n_ctx)
    run_decode(oracle, 1, 2, 1, 64, 25, 20, n_ctx, 30, seed=n_ctx)


def test_decode_step_equals_prefill_row_on_gpu(oracle):
    """Sec. 3.4: recurrent evaluation gives the same result as the one-shot one."""
    require_gpu()
    B, H, Gu, d, k, w, n_ctx, steps = 1, 2, 1, 128, 32, 32, 700, 50
    state, og, _, hist = run_decode(oracle, B, H, Gu, d, k, w, n_ctx, steps, seed=3)
    Q, K, V = (dev(hist[x], True) for x in ("Q", "K", "V"))
    u = dev(hist["u"])
    tau, death = spk.sparsek_mask(u, k)
    o_pre = host(spk.sparsek_attn_fwd(Q, K, V, u, tau, death, k, w, 0, 1.0, return_lse=False))
    err = np.abs(o_pre[:, :, n_ctx:] - og).max()
    assert err <= 2.0 ** -7 * np.abs(og).max()


def test_decode_snapshot_and_replay(oracle):
    require_gpu()
    rng = np.random.default_rng(9)
    B, H, Gu, d, k, w = 2, 2, 1, 64, 10, 8
    hist = history(rng, B, H, Gu, 120, d, "bf16")
    Q, K, V = (dev(hist[x], True) for x in ("Q", "K", "V"))
    u = dev(hist["u"])
    state = spk.DecodeState(B, H, Gu, d, k, w, torch.bfloat16)
    spk.sparsek_decode_init(state)

    def go(a, b):
        return [spk.sparsek_decode_step(state, Q[:, :, t].contiguous(), K[:, :, t].contiguous(),
                                        V[:, :, t].contiguous(), u[:, :, t].contiguous()).clone() for t in range(a, b)]

    go(0, 70)
    snap = state.buf.clone()
    first = go(70, 120)
    state.buf.copy_(snap)
    second = go(70, 120)
    for a, b in zip(first, second):
        assert torch.equal(a, b)


def test_decode_candidate_overflow_sets_status(oracle):
    """All-equal scores keep every key above tau; a small candidate capacity must overflow,
    set bit 0 of the row's status word and keep running."""
    require_gpu()
    B, H, Gu, d, k, w = 1, 1, 1, 64, 4, 2
    state = spk.DecodeState(B, H, Gu, d, k, w, torch.bfloat16, cand_cap=8)
    spk.sparsek_decode_init(state)
    g = torch.Generator(device="cuda").manual_seed(1)
    for t in range(40):
        x = torch.randn(3, B, H, d, device="cuda", generator=g).bfloat16()
        o = spk.sparsek_decode_step(state, x[0], x[1], x[2], torch.full((B, Gu), 0.5, device="cuda"))
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
    assert spk.sparsek_decode_status(state)[0] & 1
