"""Parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times: thresholds / lifetimes of whole score rows against the oracle, attention
outputs on sampled heads and query spans (the oracle computes any row on its own), decode on
sampled heads over all 256 steps.  Configs 4 and 5 are drawn on the device (same
distributions as the host recipe) and the sampled slices are copied back for the oracle.
The kernels deal heads to the chip's 8 partitions by index, so the sampled heads of configs 4 and 5
cover every residue modulo 8 and the last head.  Every prefill config runs a second time with q
boosted 8x (peaky softmax: a wrong gate or index cannot average out).  Gradient references come
from the oracle's own thresholds and lifetimes.
"""
import math

import numpy as np
import pytest
import torch

import paper_2406_16747_amd as spk
from paper_2406_16747_amd import synth
from gpu_util import dev, host, kink_keys, oracle_mask32, require_gpu, say

pytestmark = pytest.mark.gpu


def check_mask_rows(oracle, u_np, tau_g, death_g, k, rows):
    for (b, g) in rows:
        tau_r = oracle.tau_prefixes(u_np[b, g], k)[0]
        death_r = oracle.death(u_np[b, g], k)
        np.testing.assert_array_equal(death_g[b, g], death_r)
        err = np.abs(tau_g[b, g].astype(np.float64) - tau_r) / np.maximum(1.0, np.abs(tau_r))
        assert err.max() <= 1e-5, (b, g, err.max())
        yield (b, g), tau_r, death_r


def check_attn_spans(oracle, q32, k32, v32, u_row, tau_r, death_r, o_g, lse_g, k, w, mode, spans):
    for (a, e) in spans:
        o_r, lse_r = oracle.attn_rows(q32, k32, v32, u_row, tau_r, death_r, k, w, mode, 1.0, a, e)
        err = np.abs(o_g[a:e] - o_r).max()
        ref = np.abs(o_r).max()
        assert err <= 1e-2 and err <= ref * 2.0 ** -7 + 1e-6, (a, err, ref)
        np.testing.assert_allclose(lse_g[a:e], lse_r, atol=2e-3, rtol=1e-4)


def test_config2_full(oracle):
    require_gpu()
    say("config 2 full: B=8 H=12 n=4096 d=64 k=w=256")
    inp = synth.make(2)
    k, w, n = inp["k"], inp["w"], inp["n"]
    u = dev(inp["u"])
    Q, K, V = (dev(inp[x], True) for x in ("Q", "K", "V"))
    tau, death = spk.sparsek_mask(u, k)
    o, lse = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, k, w, 0, 1.0)
    torch.cuda.synchronize()
    tau_g, death_g, o_g, lse_g = host(tau), host(death), host(o), host(lse)
    for (b, g), tau_r, death_r in check_mask_rows(oracle, inp["u"], tau_g, death_g, k, [(b, 0) for b in range(8)]):
        if b in (0, 5):
            for h in (0, 11) if b == 0 else (7,):
                check_attn_spans(oracle, inp["Q32"][b, h], inp["K32"][b, h], inp["V32"][b, h], inp["u"][b, 0], tau_r,
                                 death_r, o_g[b, h], lse_g[b, h], k, w, 0, [(0, n)] if (b, h) == (0, 0) else
                                 [(0, 300), (2000, 2200), (3900, n)])
    say("  peaky pass (q x 8)")
    Q8 = (Q.float() * 8.0).bfloat16()
    o, lse = spk.sparsek_attn_fwd(Q8, K, V, u, tau, death, k, w, 0, 1.0)
    torch.cuda.synchronize()
    o_g, lse_g = host(o), host(lse)
    for (b, h) in ((3, 2), (7, 9)):
        tau_r, death_r = oracle.tau_prefixes(inp["u"][b, 0], k)[0], oracle.death(inp["u"][b, 0], k)
        check_attn_spans(oracle, inp["Q32"][b, h] * np.float32(8), inp["K32"][b, h], inp["V32"][b, h], inp["u"][b, 0],
                         tau_r, death_r, o_g[b, h], lse_g[b, h], k, w, 0, [(0, 300), (500, 700), (2000, 2200), (3900, n)])


def test_config3_full_forward_and_du(oracle):
    require_gpu()
    say("config 3 full: B=4 H=16 n=8192 d=128 k=w=512, forward + du + dq, dk, dv")
    inp = synth.make(3, with_dO=True)
    k, w, n = inp["k"], inp["w"], inp["n"]
    u = dev(inp["u"])
    Q, K, V, dO = (dev(inp[x], True) for x in ("Q", "K", "V", "dO"))
    tau, death = spk.sparsek_mask(u, k)
    o, lse = spk.sparsek_attn_fwd(Q, K, V, u, tau, death, k, w, 0, 1.0)
    du = spk.sparsek_mask_bwd(Q, K, V, u, tau, death, o, lse, dO, k, w, 0, 1.0)
    torch.cuda.synchronize()
    tau_g, death_g, o_g, lse_g, du_g = host(tau), host(death), host(o), host(lse), host(du)
    for (b, g), tau_r, death_r in check_mask_rows(oracle, inp["u"], tau_g, death_g, k, [(b, 0) for b in range(4)]):
        if b == 1:
            for h in (0, 9):
                check_attn_spans(oracle, inp["Q32"][b, h], inp["K32"][b, h], inp["V32"][b, h], inp["u"][b, 0], tau_r,
                                 death_r, o_g[b, h], lse_g[b, h], k, w, 0, [(0, 200), (1000, 1150), (8000, n)])
    tau_r32, death_r = oracle_mask32(oracle, inp["u"], k)
    kink = kink_keys(inp["u"], tau_r32, tau_g)
    assert kink.sum() <= 8, kink.sum()
    # du of two batch elements (all 16 heads add into a score row), from the oracle's own thresholds
    for b in (2, 0):
        say("  oracle du for batch element", b)
        ref, _ = oracle.mask_bwd(inp["Q32"][b:b + 1], inp["K32"][b:b + 1], inp["V32"][b:b + 1], inp["u"][b:b + 1],
                                 tau_r32[b:b + 1], death_r[b:b + 1], inp["dO32"][b:b + 1], k, w, 0, 1.0)
        scale = np.abs(ref).max()
        diff = np.abs(du_g[b] - ref[0])
        assert scale > 0 and diff[~kink[b]].max() <= 1e-2 * scale, (b, diff.max(), scale)
    # dQ, dK, dV of one batch element (the gates held fixed)
    b = 2
    dq, dk, dv = spk.sparsek_attn_bwd(Q, K, V, u, tau, death, o, lse, dO, k, w, 0, 1.0)
    torch.cuda.synchronize()
    say("  oracle dq, dk, dv for batch element", b)
    refs = oracle.attn_bwd(inp["Q32"][b:b + 1], inp["K32"][b:b + 1], inp["V32"][b:b + 1], inp["u"][b:b + 1],
                           tau_r32[b:b + 1], death_r[b:b + 1], inp["dO32"][b:b + 1], k, w, 0, 1.0)
    for name, g, r in zip(("dq", "dk", "dv"), (dq, dk, dv), refs):
        g = host(g[b])
        scale = np.abs(r).max()
        err = np.abs(g - r[0]).max()
        assert np.isfinite(g).all() and scale > 0 and err <= 1e-2 * scale, (name, err, scale)
    say("  peaky pass (q x 8)")
    Q8 = (Q.float() * 8.0).bfloat16()
    o, lse = spk.sparsek_attn_fwd(Q8, K, V, u, tau, death, k, w, 0, 1.0)
    torch.cuda.synchronize()
    for (b, h) in ((0, 5), (3, 15)):
        check_attn_spans(oracle, inp["Q32"][b, h] * np.float32(8), inp["K32"][b, h], inp["V32"][b, h], inp["u"][b, 0],
                         oracle.tau_prefixes(inp["u"][b, 0], k)[0], death_r[b, 0], host(o[b, h]), host(lse[b, h]), k, w,
                         0, [(0, 200), (1000, 1150), (4090, 4230), (8000, n)])


def device_recipe(B, H, Gu, n, d, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    div = math.sqrt(d)
    q, k, v = ((torch.randn((B, H, n, d), device="cuda", generator=g) / div).bfloat16() for _ in range(3))
    u = torch.randn((B, Gu, n), device="cuda", generator=g)
    return q, k, v, u


@pytest.mark.parametrize("Gu", [1, 32])
def test_config4_full(oracle, Gu):
    require_gpu()
    say("config 4 full: B=1 H=32 n=32768 d=128 k=w=1024, Gu =", Gu)
    B, H, n, d, k, w = 1, 32, 32768, 128, 1024, 1024
    q, kk, v, u = device_recipe(B, H, Gu, n, d, 1004)
    tau, death = spk.sparsek_mask(u, k)
    o, lse = spk.sparsek_attn_fwd(q, kk, v, u, tau, death, k, w, 0, 1.0)
    torch.cuda.synchronize()
    u_np, tau_g, death_g = host(u), host(tau), host(death)
    heads = [0, 9, 18, 27, 4, 13, 22, 31]  # every residue modulo 8, and the last head
    spans = [(0, 130), (1000, 1100), (2040, 2180), (16380, 16520), (32640, n)]
    rows = [(0, 0)] if Gu == 1 else [(0, h) for h in heads]
    masks = {}
    for (b, g), tau_r, death_r in check_mask_rows(oracle, u_np, tau_g, death_g, k, rows):
        masks[g] = (tau_r, death_r)
    for h in heads:
        g = 0 if Gu == 1 else h
        say("  head", h)
        check_attn_spans(oracle, host(q[0, h]), host(kk[0, h]), host(v[0, h]), u_np[0, g], masks[g][0], masks[g][1],
                         host(o[0, h]), host(lse[0, h]), k, w, 0, spans)
    say("  peaky pass (q x 8)")
    q8 = (q.float() * 8.0).bfloat16()
    o, lse = spk.sparsek_attn_fwd(q8, kk, v, u, tau, death, k, w, 0, 1.0)
    torch.cuda.synchronize()
    for h in (9, 22, 31):
        g = 0 if Gu == 1 else h
        check_attn_spans(oracle, host(q8[0, h]), host(kk[0, h]), host(v[0, h]), u_np[0, g], masks[g][0], masks[g][1],
                         host(o[0, h]), host(lse[0, h]), k, w, 0, spans)


def test_config5_full_decode(oracle):
    require_gpu()
    say("config 5 full: decode B=64 H=32 d=128 k=w=1024, context 32768, 256 steps")
    B, H, Gu, d, k, w, n_ctx, steps = 64, 32, 1, 128, 1024, 1024, 32768, 256
    g = torch.Generator(device="cuda")
    g.manual_seed(1005)
    div = math.sqrt(d)
    K = torch.empty(B, H, n_ctx, d, device="cuda", dtype=torch.bfloat16)
    V = torch.empty_like(K)
    for b in range(B):
        K[b] = (torch.randn(H, n_ctx, d, device="cuda", generator=g) / div).bfloat16()
        V[b] = (torch.randn(H, n_ctx, d, device="cuda", generator=g) / div).bfloat16()
    u = torch.randn(B, Gu, n_ctx, device="cuda", generator=g)
    # batch elements spread over the batch, heads over every residue modulo 8 and the last head
    sample = [(0, 0), (9, 1), (18, 10), (27, 19), (37, 4), (45, 13), (54, 22), (63, 31)]
    hist = {s: (host(K[s[0], s[1]]), host(V[s[0], s[1]]), host(u[s[0], 0])) for s in sample}
    tau, death = spk.sparsek_mask(u, k)
    state = spk.DecodeState(B, H, Gu, d, k, w, torch.bfloat16)
    spk.sparsek_decode_load(state, K, V, u, tau, death)
    torch.cuda.synchronize()
    del K, V
    qs, ks, vs = ((torch.randn(steps, B, H, d, device="cuda", generator=g) / div).bfloat16() for _ in range(3))
    us = torch.randn(steps, B, Gu, device="cuda", generator=g)
    outs = torch.empty(steps, B, H, d, device="cuda", dtype=torch.bfloat16)
    for s in range(steps):
        spk.sparsek_decode_step(state, qs[s], ks[s], vs[s], us[s], out=outs[s])
    torch.cuda.synchronize()
    assert not spk.sparsek_decode_status(state).any()
    for (b, h) in sample:
        say("  oracle decode for head", b, h)
        Kh, Vh, uh = hist[(b, h)]
        K_full = np.concatenate([Kh, host(ks[:, b, h])])
        V_full = np.concatenate([Vh, host(vs[:, b, h])])
        u_full = np.concatenate([uh, host(us[:, b, 0])])
        ref = oracle.decode_bydef(host(qs[:, b, h]), K_full, V_full, u_full, n_ctx, k, w, 0, 1.0)
        got = host(outs[:, b, h])
        err = np.abs(got - ref).max()
        scale = np.abs(ref).max()
        assert err <= 1e-2 and err <= scale * 2.0 ** -7, (b, h, err, scale)


def test_chunked_prefill_at_bench_shape(oracle):
    """The chunk leg of bench.py (H=32 d=128 k=w=1024, chunks of 8192) over a 32K sequence: sampled
    query spans of two heads against the oracle's attention on the whole sequence; the retained set
    stays within its capacity, far below the sequence length."""
    require_gpu()
    say("chunked prefill at the bench shape: H=32 n=32768 d=128 k=w=1024, chunks of 8192")
    B, H, n, d, k, w, c = 1, 32, 32768, 128, 1024, 1024, 8192
    g = torch.Generator(device="cuda")
    g.manual_seed(2204)
    div = math.sqrt(d)
    q, kk, v = ((torch.randn(B, H, n, d, device="cuda", generator=g) / div).bfloat16() for _ in range(3))
    u = torch.randn(B, 1, n, device="cuda", generator=g)
    st = spk.ChunkState(B, H, 1, d, k, w, spk.BF16, c, 0, 1.0)
    outs = []
    for p in range(0, n, c):
        outs.append(spk.sparsek_chunk_prefill(st, q[:, :, p:p + c].contiguous(), kk[:, :, p:p + c].contiguous(),
                                              v[:, :, p:p + c].contiguous(), u[:, :, p:p + c].contiguous()))
    o = torch.cat(outs, 2)
    torch.cuda.synchronize()
    counts, flags = spk.sparsek_chunk_status(st)
    assert not flags.any() and counts.max() < 6144
    u_np = host(u)
    tau_r = oracle.tau_prefixes(u_np[0, 0], k)[0]
    death_r = oracle.death(u_np[0, 0], k)
    for h in (3, 30):
        o_g = host(o[0, h])
        q32, k32, v32 = host(q[0, h]), host(kk[0, h]), host(v[0, h])
        for (a, e) in [(0, 150), (8100, 8300), (16384, 16500), (24500, 24600), (32700, n)]:
            o_r, _ = oracle.attn_rows(q32, k32, v32, u_np[0, 0], tau_r, death_r, k, w, 0, 1.0, a, e)
            err = np.abs(o_g[a:e] - o_r).max()
            ref = np.abs(o_r).max()
            assert err <= 1e-2 and err <= ref * 2.0 ** -7 + 1e-6, (h, a, err, ref)



def test_chunk_training_at_bench_shape(oracle):
    """Forward + backward of the second of two 8192-token chunks at the bench's head shape (H=32 d=128
    k=w=1024): dq, dk, dv of two heads and du against the oracle's full-sequence backward with the
    upstream gradient masked to that chunk (du sums over all heads, so it is checked on a run with the
    two heads alone)."""
    require_gpu()
    say("chunk training at the bench shape: H=32 (then 2) n=16384 d=128 k=w=1024, chunks of 8192")
    B, H, n, d, k, w, c = 1, 32, 16384, 128, 1024, 1024, 8192
    g = torch.Generator(device="cuda")
    g.manual_seed(2304)
    div = math.sqrt(d)
    q, kk, v = ((torch.randn(B, H, n, d, device="cuda", generator=g) / div).bfloat16() for _ in range(3))
    dO = torch.randn(B, H, n, d, device="cuda", generator=g).bfloat16()
    u = torch.randn(B, 1, n, device="cuda", generator=g)
    heads = [5, 28]

    def run(hsel):
        qs, ks, vs, ds = (x[:, hsel].contiguous() for x in (q, kk, v, dO))
        st = spk.ChunkState(B, len(hsel), 1, d, k, w, spk.BF16, c, 0, 1.0)
        res = None
        for p in range(0, n, c):
            qc = qs[:, :, p:p + c].contiguous()
            o = spk.sparsek_chunk_prefill(st, qc, ks[:, :, p:p + c].contiguous(), vs[:, :, p:p + c].contiguous(),
                                          u[:, :, p:p + c].contiguous())
            res = spk.sparsek_chunk_bwd(st, qc, o, ds[:, :, p:p + c].contiguous())
        torch.cuda.synchronize()
        return [host(x) for x in res]

    full = run(list(range(H)))   # the launch shape bench.py times
    two = run(heads)             # du of the two heads alone
    sl = slice(c, n)
    q32, k32, v32 = (host(x[:, heads]) for x in (q, kk, v))
    dO_m = host(dO[:, heads])
    dO_m[:, :, :c] = 0.0
    u_np = host(u)
    tau64, death = oracle.mask_all(u_np, k)
    say("  oracle backward of 2 heads over 16384 positions")
    rq, rk, rv = oracle.attn_bwd(q32, k32, v32, u_np, tau64, death, dO_m, k, w, 0, 1.0)
    ru, _ = oracle.mask_bwd(q32, k32, v32, u_np, tau64, death, dO_m, k, w, 0, 1.0)
    for name, gi, r in (("dq", 0, rq), ("dk", 1, rk), ("dv", 2, rv)):
        r = r[:, :, sl]
        scale = np.abs(r).max()
        for got in (full[gi][:, heads], two[gi]):
            err = np.abs(got - r).max()
            assert np.isfinite(got).all() and scale > 0 and err <= 1e-2 * scale, (name, err, scale)
    r = ru[:, :, sl]
    scale = np.abs(r).max()
    err = np.abs(two[3] - r).max()
    assert scale > 0 and err <= 1e-2 * scale, ("du", err, scale)
    assert np.isfinite(full[3]).all()
