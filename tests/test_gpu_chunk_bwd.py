"""GPU parity of sparsek_chunk_bwd: training with chunk-wise recurrence, the cache's gradient stopped.

With the retained keys of earlier chunks held constant, the gradient of L_c = sum(dO_c * O_c) with
respect to chunk c's own q, k, v and scores is the gradient of the unchunked operator for an upstream
gradient that is zero outside the chunk's rows, read at the chunk's positions (the chunked forward
equals the unchunked one, and O_c depends on the chunk's keys only through the chunk's rows).  So the
reference is the oracle's full-sequence attn_bwd / mask_bwd with dO masked to the chunk.
Bars as for sparsek_attn_bwd and sparsek_mask_bwd: 1e-2 of max|ref| per tensor (bf16 storage).
"""
import numpy as np
import pytest
import torch

import paper_2406_16747_amd as spk
from paper_2406_16747_amd import synth
from gpu_util import dev, host, require_gpu, say

pytestmark = pytest.mark.gpu


def run_case(oracle, inp, chunks, gate_mode):
    B, H, n, d, k, w, Gu = (inp[x] for x in ("B", "H", "n", "d", "k", "w", "Gu"))
    q, kk, v, dO = (dev(inp[x], True) for x in ("Q", "K", "V", "dO"))
    u = dev(inp["u"])
    st = spk.ChunkState(B, H, Gu, d, k, w, spk.BF16, max(chunks), gate_mode, inp["scale"], 0)
    tau64, death = oracle.mask_all(inp["u"], k)
    pos = 0
    for ci, c in enumerate(chunks):
        sl = slice(pos, pos + c)
        qc, dOc = q[:, :, sl].contiguous(), dO[:, :, sl].contiguous()
        o = spk.sparsek_chunk_prefill(st, qc, kk[:, :, sl].contiguous(), v[:, :, sl].contiguous(),
                                      u[:, :, sl].contiguous())
        dq, dk, dv, du = spk.sparsek_chunk_bwd(st, qc, o, dOc)
        torch.cuda.synchronize()
        got = {"dq": host(dq), "dk": host(dk), "dv": host(dv), "du": host(du)}
        for name, g in got.items():
            assert np.isfinite(g).all(), (name, ci)
        dO_m = np.zeros_like(inp["dO32"])
        dO_m[:, :, sl] = inp["dO32"][:, :, sl]
        rq, rk, rv = oracle.attn_bwd(inp["Q32"], inp["K32"], inp["V32"], inp["u"], tau64, death, dO_m, k, w,
                                     2 if gate_mode == 3 else gate_mode, inp["scale"])
        ru, _ = oracle.mask_bwd(inp["Q32"], inp["K32"], inp["V32"], inp["u"], tau64, death, dO_m, k, w, gate_mode,
                                inp["scale"])
        ref = {"dq": rq[:, :, sl], "dk": rk[:, :, sl], "dv": rv[:, :, sl], "du": ru[:, :, sl]}
        common = max(np.abs(ref[x]).max() for x in ("dq", "dk", "dv"))
        for name in ("dq", "dk", "dv", "du"):
            r, g = ref[name], got[name]
            scale = np.abs(r).max() if name == "du" else max(np.abs(r).max(), 1e-3 * common)
            err = np.abs(g - r).max()
            if name == "du" and scale == 0.0:
                # no soft gate in reach of this chunk's queries: the exact gradient is zero; the kernel forms it as
                # a difference of fp64 prefix sums, which may leave rounding noise of the order 1e-16 of their size
                assert err <= 1e-12 * common, (name, ci, err)
                continue
            assert err <= 1e-2 * scale + 1e-30, (name, ci, err, scale, np.unravel_index(np.abs(g - r).argmax(), g.shape))
        pos += c
    counts, flags = spk.sparsek_chunk_status(st)
    assert (flags == 0).all()


@pytest.mark.parametrize("n,d,k,w,Gu,chunks,gate_mode", [
    (900, 64, 32, 40, 1, [300, 300, 300], 0),
    (1000, 128, 48, 64, 1, [256, 256, 256, 232], 0),
    (1000, 128, 48, 64, 2, [400, 600], 1),
    (800, 64, 40, 0, 1, [200, 200, 400], 0),
    (700, 64, 24, 30, 1, [350, 350], 3),
    (600, 128, 16, 20, 1, [128, 472], 2),
    (900, 128, 40, 50, 2, [77, 500, 323], 0),
    (520, 64, 600, 8, 1, [260, 260], 0),
])
def test_chunk_bwd_equals_masked_full_backward(oracle, n, d, k, w, Gu, chunks, gate_mode):
    require_gpu()
    say("chunk bwd", n, d, k, w, Gu, chunks, gate_mode)
    inp = synth.make(3, Gu=Gu, seed=n + k + w, with_dO=True, B=1, H=2, n=n, d=d, k=k, w=w, dtype="bf16",
                     qk_div=float(np.sqrt(d)) / 4)
    run_case(oracle, inp, chunks, gate_mode)
