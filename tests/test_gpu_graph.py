"""The hot path under HIP graph capture: the entry points are plain kernel launches on the caller's stream (no
allocation, no memset or copy nodes, no synchronisation), so a step can be captured once and replayed.  Each test
replays its graph several times on new inputs, with eager work and synchronisation between the replays, and compares
every replay bit for bit with the eager call on the same inputs (the eager path is what the parity tests check
against the oracle; thresholds, lifetimes, outputs and decode states are deterministic)."""
import numpy as np
import pytest
import torch

import paper_2406_16747_amd as spk
from paper_2406_16747_amd import synth
from gpu_util import dev, require_gpu, say

pytestmark = pytest.mark.gpu


def draw(seed, B, H, n, d, k, w, dtype):
    inp = synth.make(1, seed=seed, B=B, H=H, n=n, d=d, k=k, w=w, dtype=dtype, qk_div=float(np.sqrt(d)))
    bf16 = dtype == "bf16"
    return dev(inp["u"]), dev(inp["Q"], bf16), dev(inp["K"], bf16), dev(inp["V"], bf16)


@pytest.mark.parametrize("B,H,n,d,k,w,dtype", [(1, 1, 1024, 64, 64, 64, "fp32"), (2, 4, 1500, 128, 200, 130, "bf16")])
def test_prefill_step_replays_as_a_graph(B, H, n, d, k, w, dtype):
    require_gpu()
    say("graph: prefill step", B, H, n, d, k, w, dtype)
    u, q, kk, v = draw(100, B, H, n, d, k, w, dtype)
    mask_ws = spk.sparsek_mask_workspace(u, k)
    # warm-up on a side stream, as capture needs, then capture one step: mask + attention
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        t, dth = spk.sparsek_mask(u, k, ws=mask_ws)
        spk.sparsek_attn_fwd(q, kk, v, u, t, dth, k, w, 0, 1.0)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        tau_g, death_g = spk.sparsek_mask(u, k, ws=mask_ws)
        o_g, lse_g = spk.sparsek_attn_fwd(q, kk, v, u, tau_g, death_g, k, w, 0, 1.0)
    for rep in range(4):
        u2, q2, k2, v2 = draw(200 + rep, B, H, n, d, k, w, dtype)
        for dst, src in ((u, u2), (q, q2), (kk, k2), (v, v2)):
            dst.copy_(src)
        g.replay()
        torch.cuda.synchronize()
        tau_e, death_e = spk.sparsek_mask(u2, k)       # eager work between the replays
        o_e, lse_e = spk.sparsek_attn_fwd(q2, k2, v2, u2, tau_e, death_e, k, w, 0, 1.0)
        torch.cuda.synchronize()
        assert torch.equal(tau_g, tau_e) and torch.equal(death_g, death_e), rep
        assert torch.equal(o_g, o_e) and torch.equal(lse_g, lse_e), rep
        assert spk.sparsek_mask_status(u, k, mask_ws) == 0


def test_decode_step_replays_as_a_graph():
    require_gpu()
    say("graph: decode step")
    B, H, d, k, w, n0, steps = 2, 4, 128, 48, 40, 300, 6
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    rnd = lambda *shape: torch.randn(*shape, device="cuda", generator=gen)
    u0 = rnd(B, 1, n0)
    k0, v0 = ((rnd(B, H, n0, d) / d ** 0.5).bfloat16() for _ in range(2))
    tau0, death0 = spk.sparsek_mask(u0, k)

    def fresh():
        st = spk.DecodeState(B, H, 1, d, k, w, torch.bfloat16)
        spk.sparsek_decode_load(st, k0, v0, u0, tau0, death0)
        return st

    new = [((rnd(B, H, d) / d ** 0.5).bfloat16(), (rnd(B, H, d) / d ** 0.5).bfloat16(),
            (rnd(B, H, d) / d ** 0.5).bfloat16(), rnd(B, 1)) for _ in range(steps)]
    eager_state = fresh()
    eager = [spk.sparsek_decode_step(eager_state, *x).clone() for x in new]
    torch.cuda.synchronize()

    st = fresh()
    qs, ks, vs, us = (t.clone() for t in new[0])
    out = torch.empty_like(qs)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):  # warm-up on a throw-away state
        spk.sparsek_decode_step(fresh(), qs, ks, vs, us, out=out)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        spk.sparsek_decode_step(st, qs, ks, vs, us, out=out)
    # the capture itself ran nothing: the state is still the loaded one
    for i, x in enumerate(new):
        for dst, src in zip((qs, ks, vs, us), x):
            dst.copy_(src)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager[i]), i
    assert (spk.sparsek_decode_status(st) == spk.sparsek_decode_status(eager_state)).all()
