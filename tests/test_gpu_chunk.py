"""GPU parity of the chunk-wise recurrent prefill (fixed-size scored cache) against the CPU oracle.

The paper's claim is that chunked processing gives exactly the result of the unchunked
computation, so the reference is the oracle's attention on the WHOLE sequence; the chunked GPU
path is fed the same sequence in pieces.  Bars as for the prefill attention (bf16: max abs err
<= 1e-2 and <= 2^-7 max|ref|; fp32: <= 2e-5 max|ref|).  The retained set must stay within its
capacity with the overflow flag clear.
"""
import numpy as np
import pytest
import torch

import paper_2406_16747_amd as spk
from paper_2406_16747_amd import synth
from gpu_util import dev, host, require_gpu, say

pytestmark = pytest.mark.gpu


def run_chunked(inp, chunks, gate_mode=0, cand_cap=0, chunk_max=None):
    B, H, n, d, k, w, Gu = (inp[x] for x in ("B", "H", "n", "d", "k", "w", "Gu"))
    bf16 = inp["dtype"] == "bf16"
    q, kk, v = (dev(inp[x], bf16) for x in ("Q", "K", "V"))
    u = dev(inp["u"])
    st = spk.ChunkState(B, H, Gu, d, k, w, spk.BF16 if bf16 else spk.F32, chunk_max or max(chunks), gate_mode, inp["scale"],
                        cand_cap)
    outs, pos = [], 0
    for c in chunks:
        sl = slice(pos, pos + c)
        outs.append(spk.sparsek_chunk_prefill(st, q[:, :, sl].contiguous(), kk[:, :, sl].contiguous(),
                                              v[:, :, sl].contiguous(), u[:, :, sl].contiguous()))
        pos += c
    assert pos == n
    torch.cuda.synchronize()
    counts, flags = spk.sparsek_chunk_status(st)
    return host(torch.cat(outs, 2)), counts, flags


def compare(oracle, inp, o_g, gate_mode=0):
    B, H, n, d, k, w, Gu = (inp[x] for x in ("B", "H", "n", "d", "k", "w", "Gu"))
    bf16 = inp["dtype"] == "bf16"
    assert np.isfinite(o_g).all()
    tau, death = oracle.mask_all(inp["u"], k)
    o_r, _, _ = oracle.attn_fwd(inp["Q32"], inp["K32"], inp["V32"], inp["u"], tau, death, k, w, gate_mode, inp["scale"])
    for b in range(B):
        for h in range(H):
            err = np.abs(o_g[b, h] - o_r[b, h]).max(axis=1)
            ref = np.abs(o_r[b, h]).max()
            i = int(err.argmax())
            if bf16:
                assert err[i] <= 1e-2, (b, h, i, err[i])
                assert err[i] <= ref * 2.0 ** -7 + 1e-6, (b, h, i, err[i], ref)
            else:
                assert err[i] <= 2e-5 * max(ref, 1e-3), (b, h, i, err[i], ref)


def split(n, c):
    return [c] * (n // c) + ([n % c] if n % c else [])


@pytest.mark.parametrize("n,d,k,w,Gu,dtype,chunk", [
    (1000, 64, 20, 16, 1, "bf16", 256), (700, 128, 64, 50, 1, "bf16", 128), (900, 64, 32, 40, 2, "bf16", 300),
    (600, 32, 24, 10, 1, "fp32", 200), (500, 64, 0, 33, 1, "bf16", 128), (640, 128, 48, 0, 1, "bf16", 160),
    (300, 64, 400, 30, 1, "bf16", 100), (260, 64, 16, 300, 1, "bf16", 70),
])
def test_chunked_equals_unchunked(oracle, n, d, k, w, Gu, dtype, chunk):
    require_gpu()
    say("chunked prefill", n, d, k, w, Gu, dtype, chunk)
    inp = synth.make(3, Gu=Gu, seed=n + k + w, B=2, H=2, n=n, d=d, k=k, w=w, dtype=dtype, qk_div=float(np.sqrt(d)) / 4)
    o_g, counts, flags = run_chunked(inp, split(n, chunk))
    compare(oracle, inp, o_g)
    assert not flags.any()
    assert (counts <= k + w + 4 * max(k, 16) + 127).all() and (counts >= min(n, w)).all()


@pytest.mark.parametrize("gate_mode", [1, 2, 3])
def test_chunked_gate_modes_and_uneven_chunks(oracle, gate_mode):
    require_gpu()
    say("chunked prefill modes", gate_mode)
    inp = synth.make(3, seed=77, B=1, H=3, Gu=1, n=777, d=64, k=40, w=24, qk_div=2.0)
    o_g, _, flags = run_chunked(inp, [1, 130, 2, 300, 64, 280], gate_mode, chunk_max=512)
    compare(oracle, inp, o_g, gate_mode)
    assert not flags.any()


def test_chunked_longer_sequence_constant_state(oracle):
    """Config 3 recipe scaled down (k=w=128), 4096 tokens in chunks of 512: the retained set stays
    near k + w + (support outside the top-k), far below the sequence length."""
    require_gpu()
    say("chunked prefill long")
    inp = synth.make(3, B=1, H=2, n=4096, k=128, w=128)
    o_g, counts, flags = run_chunked(inp, split(4096, 512))
    compare(oracle, inp, o_g)
    assert not flags.any()
    assert counts.max() < 1024


def test_overflow_sets_the_flag(oracle):
    """Nearly equal scores keep every key above the threshold: with a small candidate capacity the
    oldest unselected ones are dropped, the flag is raised, outputs stay finite."""
    require_gpu()
    say("chunked prefill overflow")
    inp = synth.make(3, seed=5, B=1, H=1, n=1500, d=64, k=16, w=16)
    rng = np.random.default_rng(1)
    inp["u"] = (1e-3 * rng.standard_normal((1, 1, 1500))).astype(np.float32)
    o_g, counts, flags = run_chunked(inp, split(1500, 250), cand_cap=64)
    assert np.isfinite(o_g).all()
    assert flags.all()
    assert (counts <= 128).all()


@pytest.mark.parametrize("d,dtype,Gu", [(128, "bf16", 1), (64, "bf16", 2), (32, "fp32", 1)])
def test_chunks_then_decode(oracle, d, dtype, Gu):
    """Chunked prefill over the context, hand-over, then single-token decode: every decode output is
    the corresponding row of the oracle's attention over the whole history."""
    require_gpu()
    say("chunks then decode", d, dtype, Gu)
    B, H, k, w, n_ctx, steps = 1, 2, 24, 20, 600, 40
    n = n_ctx + steps
    inp = synth.make(3, Gu=Gu, seed=d + Gu, B=B, H=H, n=n, d=d, k=k, w=w, dtype=dtype, qk_div=float(np.sqrt(d)) / 4)
    bf16 = dtype == "bf16"
    Q, K, V = (dev(inp[x], bf16) for x in ("Q", "K", "V"))
    u = dev(inp["u"])
    st = spk.ChunkState(B, H, Gu, d, k, w, spk.BF16 if bf16 else spk.F32, 256, 0, inp["scale"])
    pos = 0
    for c in (256, 256, 88):
        sl = slice(pos, pos + c)
        spk.sparsek_chunk_prefill(st, Q[:, :, sl].contiguous(), K[:, :, sl].contiguous(), V[:, :, sl].contiguous(),
                                  u[:, :, sl].contiguous())
        pos += c
    assert pos == n_ctx
    ds = spk.DecodeState(B, H, Gu, d, k, w, torch.bfloat16 if bf16 else torch.float32, 0, inp["scale"])
    ds.buf.fill_(255)
    spk.sparsek_chunk_to_decode(st, n_ctx, ds)
    outs = []
    for t in range(n_ctx, n):
        outs.append(spk.sparsek_decode_step(ds, Q[:, :, t].contiguous(), K[:, :, t].contiguous(), V[:, :, t].contiguous(),
                                            u[:, :, t].contiguous()))
    torch.cuda.synchronize()
    og = np.stack([host(o) for o in outs], axis=2)
    assert not spk.sparsek_decode_status(ds).any()
    for b in range(B):
        for h in range(H):
            g = 0 if Gu == 1 else h
            ref = oracle.decode_bydef(inp["Q32"][b, h, n_ctx:], inp["K32"][b, h], inp["V32"][b, h], inp["u"][b, g], n_ctx, k,
                                      w, 0, inp["scale"])
            err = np.abs(og[b, h] - ref).max()
            scale = np.abs(ref).max()
            if bf16:
                assert err <= 1e-2 * max(1.0, scale) and err <= scale * 2.0 ** -7, (b, h, err, scale)
            else:
                assert err <= 2e-5 * scale, (b, h, err, scale)
    # too early a hand-over is refused
    st2 = spk.ChunkState(B, H, Gu, d, k, w, spk.BF16 if bf16 else spk.F32, 256, 0, inp["scale"])
    with pytest.raises(Exception):
        spk.sparsek_chunk_to_decode(st2, k + w - 1, ds)
