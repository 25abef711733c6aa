#!/usr/bin/env python3
"""Benchmark of the SparseK hot path on one MI355X.

A step is one pass of the whole prefill path over one batch of synthetic input:
sparsek_mask (thresholds + lifetimes) followed by sparsek_attn_fwd, at the
Llama-7B-shaped long-context configuration (B=1, H=32, n=32768, d=128, k=w=1024, bf16).
Inputs are resident in HBM before the timed region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-prefill-configs] [--no-bwd]
                    [--no-decode] [--no-scores] [--no-chunk] [--only LEG]

Besides the headline (config 4) the line carries one object per further leg: the prefill of configs 1-3, the
backward at config 3, the score pipeline, the chunk-wise recurrent prefill and the decode of config 5, each with
its roofline object and, where the oracle covers it, a cpu_baseline.
"""
import argparse
import json
import math
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2516.6  # 256 CUs x 2.4 GHz x 4096 flop/clk, dense
HBM_PEAK_GBS = 8000.0


FP32_VECTOR_PEAK_TFLOPS = 157.3  # 256 CUs x 4 SIMDs x 16 lanes x 2 (packed) x 2 flop x 2.4 GHz


def stats(samples):
    """mean / median / min of per-iteration times (ms)."""
    xs = sorted(samples)
    return {"mean": sum(xs) / len(xs), "median": xs[len(xs) // 2], "min": xs[0], "n": len(xs)}


def timed(fn, iters=20, warm=3):
    """Per-iteration device times (ms) of fn from HIP events on the launch stream."""
    import torch

    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in ev]


def graph_timed(fn, iters=20, warm=3):
    """fn captured once as a HIP graph (the entry points are plain launches on the caller's stream) and replayed:
    per-replay device times (ms).  For the launch-bound legs this is what a serving loop would see."""
    import torch

    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fn()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return timed(g.replay, iters, warm)


def attended_pairs(n, k, w):
    """Number of (query, key) pairs one head attends: window part + selected part."""
    win = n * w - w * (w - 1) // 2 if n >= w else n * (n + 1) // 2
    m = max(n - w, 0)  # queries with a selected part; query i sees min(k, i-w+1) selected keys
    sel = m * k - k * (k - 1) // 2 if m >= k else m * (m + 1) // 2
    return win + sel


def device_inputs(cfg, seed):
    """Config-4 recipe drawn on the device: q,k,v ~ N(0,1)/sqrt(d) in bf16, u ~ N(0,1) fp32."""
    import torch

    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    shape = (cfg["B"], cfg["H"], cfg["n"], cfg["d"])
    div = math.sqrt(cfg["d"])
    q, k, v = ((torch.randn(shape, device="cuda", generator=g) / div).bfloat16() for _ in range(3))
    u = torch.randn((cfg["B"], cfg["Gu"], cfg["n"]), device="cuda", generator=g)
    return q, k, v, u


def cpu_baseline(cfg, q, k, v, u, rows_per_head=16384):
    """The CPU oracle, untuned, on a bounded sample of the same workload: thresholds and
    lifetimes of the full score row, then `rows_per_head` query rows from the middle of the
    sequence for as many heads as there are host threads.  Attention time is scaled by the
    ratio of attended pairs; the result is whole-job tokens/s."""
    import numpy as np

    import oracle

    oracle.build()
    cores = min(os.cpu_count() or 1, 16, cfg["H"])
    n, kk, w, H = cfg["n"], cfg["k"], cfg["w"], cfg["H"]
    u0 = u[0, 0].cpu().numpy()
    t0 = time.perf_counter()
    tau = oracle.tau_prefixes(u0, kk)[0]
    death = oracle.death(u0, kk)
    t_mask = time.perf_counter() - t0
    a = n // 2
    e = a + rows_per_head
    heads = list(range(cores))
    qs = [q[0, h].float().cpu().numpy() for h in heads]
    ks = [k[0, h].float().cpu().numpy() for h in heads]
    vs = [v[0, h].float().cpu().numpy() for h in heads]

    def one(i):
        return oracle.attn_rows(qs[i], ks[i], vs[i], u0, tau, death, kk, w, 0, 1.0, a, e)

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        list(ex.map(one, range(len(heads))))
    t_attn = time.perf_counter() - t0
    sample_pairs = len(heads) * sum(min(i + 1, w) + min(kk, max(i - w + 1, 0)) for i in range(a, e))
    total_pairs = cfg["B"] * H * attended_pairs(n, kk, w)
    t_full = t_mask * cfg["B"] * cfg["Gu"] + t_attn * total_pairs / sample_pairs
    # one thread: a shorter span of one head
    e1 = a + max(rows_per_head // 8, 64)
    t0 = time.perf_counter()
    oracle.attn_rows(qs[0], ks[0], vs[0], u0, tau, death, kk, w, 0, 1.0, a, e1)
    t_one = time.perf_counter() - t0
    one_pairs = sum(min(i + 1, w) + min(kk, max(i - w + 1, 0)) for i in range(a, e1))
    t_full_one = t_mask * cfg["B"] * cfg["Gu"] + t_one * total_pairs / one_pairs
    return {
        "value": cfg["B"] * n / t_full,
        "unit": "tokens/s",
        "cores": cores,
        "kind": "oracle",
        "single_thread_value": cfg["B"] * n / t_full_one,
        "sample": "tau+lifetimes of the full score row (%.1f s, one thread) and query rows %d..%d of %d heads "
                  "(%.1f s), attention time scaled by attended pairs to all %d heads x %d rows; single thread: "
                  "rows %d..%d of one head (%.1f s), scaled the same way"
                  % (t_mask, a, e - 1, len(heads), t_attn, H, n, a, e1 - 1, t_one),
    }


def prefill_leg(config, iters=20, warm=3, with_cpu=True):
    """Configs 1-3 as the headline is measured: one step = sparsek_mask + sparsek_attn_fwd on the configuration's
    own recipe (drawn on the host: the CPU oracle gets the identical bytes).  Config 2 is bound by HBM (d = 64,
    small k + w), config 3 by the matrix cores, config 1 (fp32, one head) runs the vector-ALU kernel and is
    launch-bound.  The oracle is timed in full on all host threads, and on one thread on a slice of heads."""
    import numpy as np
    import torch

    import paper_2406_16747_amd as spk
    from paper_2406_16747_amd import synth

    inp = synth.make(config)
    B, H, n, d, k, w, Gu = (inp[x] for x in ("B", "H", "n", "d", "k", "w", "Gu"))
    bf16 = inp["dtype"] == "bf16"
    u = torch.from_numpy(inp["u"]).cuda()
    q, kk, v = (synth.to_device(inp[x], inp["dtype"]) for x in ("Q", "K", "V"))
    tau, death = spk.sparsek_mask(u, k)
    mask_ms = stats(timed(lambda: spk.sparsek_mask(u, k), iters, warm))
    attn_ms = stats(timed(lambda: spk.sparsek_attn_fwd(q, kk, v, u, tau, death, k, w, 0, 1.0), iters, warm))

    def step():
        t, dth = spk.sparsek_mask(u, k)
        spk.sparsek_attn_fwd(q, kk, v, u, t, dth, k, w, 0, 1.0)

    step_ms = stats(timed(step, iters, warm))
    graph_ms = stats(graph_timed(step, iters, warm))
    pairs = attended_pairs(n, k, w) * B * H
    flops = 4.0 * d * pairs
    nbytes = 4.0 * B * H * n * d * (2 if bf16 else 4) + B * H * n * 4 + 3.0 * B * Gu * n * 4
    t_attn = attn_ms["mean"] * 1e-3
    if config == 2:
        roof = {"bound": "hbm", "achieved": nbytes / t_attn / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "algorithmic_bytes": nbytes, "mfma_tflops": flops / t_attn / 1e12,
                "traffic": read_traffic("attn_fwd_mfma_config2_counters.txt")}
    elif config == 3:
        roof = {"bound": "mfma", "achieved": flops / t_attn / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "algorithmic_flops": flops, "traffic": read_traffic("attn_fwd_mfma_config3_counters.txt")}
    else:
        roof = {"bound": "alu", "achieved": flops / t_attn / 1e12, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                "algorithmic_flops": flops, "traffic": None,
                "note": "31 MFLOP in all: the two launches are latency-bound; microseconds are the figure to read"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["kernel"] = ("attn_fwd_mfma_kernel<%d> (+ block_lists_kernel, inside the timed call)" % d) if bf16 else \
        "attn_fwd_generic_kernel<float> (+ block_lists_kernel, inside the timed call)"
    roof["ms_per_launch"] = attn_ms["mean"]
    out = {
        "workload": "config %d: prefill fwd, B=%d H=%d n=%d d=%d k=%d w=%d %s, Gu=%d, gate_mode=0, mask+select+attention "
                    "per step" % (config, B, H, n, d, k, w, inp["dtype"], Gu),
        "ms_per_step": step_ms, "mask_ms": mask_ms, "attn_ms": attn_ms,
        "ms_per_step_as_hip_graph": graph_ms,
        "tokens_per_s": B * n / (step_ms["mean"] * 1e-3), "us_per_step": step_ms["mean"] * 1e3,
        "roofline": roof,
    }
    if with_cpu:
        import oracle

        oracle.build()
        cores = min(os.cpu_count() or 1, 16)
        t0 = time.perf_counter()
        tau_r, death_r = oracle.mask_all(inp["u"], k)
        t_mask = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.attn_fwd(inp["Q32"], inp["K32"], inp["V32"], inp["u"], tau_r, death_r, k, w, 0, 1.0, nthreads=cores)
        t_all = time.perf_counter() - t0
        hs = min(H, 2)  # one thread: the first heads of batch element 0, scaled by the head count
        t0 = time.perf_counter()
        oracle.attn_fwd(inp["Q32"][:1, :hs], inp["K32"][:1, :hs], inp["V32"][:1, :hs], inp["u"][:1, :1] if Gu == 1
                        else inp["u"][:1, :hs], tau_r[:1, :1] if Gu == 1 else tau_r[:1, :hs],
                        death_r[:1, :1] if Gu == 1 else death_r[:1, :hs], k, w, 0, 1.0, nthreads=1)
        t_one = (time.perf_counter() - t0) * (B * H / hs)
        out["cpu_baseline"] = {
            "value": B * n / (t_mask + t_all), "unit": "tokens/s", "cores": min(cores, B * H), "kind": "oracle",
            "single_thread_value": B * n / (t_mask + t_one),
            "sample": "the whole configuration: tau+lifetimes of all %d score rows (%.2f s, one thread), attention of "
                      "all %d heads on %d threads (%.2f s); single thread: %d head(s) (%.2f s scaled by %d/%d)"
                      % (B * Gu, t_mask, B * H, min(cores, B * H), t_all, hs, t_one, B * H, hs),
        }
    return out


def decode_cpu_baseline(hist, qs, ks, vs, us, n_ctx, k, w, B, H, steps):
    """The oracle beside the decode leg.  (a) decode by definition (every step recomputes thresholds and lifetimes
    of the whole history) on a slice of heads; (b) the incremental loop of Sec. 3.3 (two heaps; attention over k + w
    keys), steps only, the context already consumed -- what a CPU implementation of the method would run.  Both
    scaled linearly from the slice to all B*H heads (heads are independent)."""
    import numpy as np

    import oracle

    oracle.build()
    cores = min(os.cpu_count() or 1, 16)
    heads = sorted(hist)[:cores]

    def pack(bh):
        b, h = bh
        Kh, Vh, uh = hist[bh]
        return (qs[:, b, h].float().cpu().numpy(), np.concatenate([Kh, ks[:, b, h].float().cpu().numpy()]),
                np.concatenate([Vh, vs[:, b, h].float().cpu().numpy()]), np.concatenate([uh, us[:, b, 0].cpu().numpy()]))

    data = [pack(bh) for bh in heads]
    nd = min(len(data), 4)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=nd) as ex:
        list(ex.map(lambda a: oracle.decode_bydef(a[0], a[1], a[2], a[3], n_ctx, k, w, 0, 1.0), data[:nd]))
    t_def = time.perf_counter() - t0
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=len(data)) as ex:
        secs = [r[1] for r in ex.map(lambda a: oracle.decode_incremental(a[0], a[1], a[2], a[3], n_ctx, k, w, 0, 1.0),
                                     data)]
    t_inc_wall = time.perf_counter() - t0
    # per-head seconds of the steps alone, run len(data) at a time
    t_inc_steps = max(secs)
    one = oracle.decode_incremental(*data[0], n_ctx, k, w, 0, 1.0)[1]
    return {
        "value": B * steps / (t_def * (B * H / nd)), "unit": "tokens/s", "cores": nd, "kind": "oracle",
        "incremental": {"value": B * steps / (t_inc_steps * (B * H / len(data))), "unit": "tokens/s",
                        "cores": len(data), "single_thread_value": B * steps / (one * B * H),
                        "what": "orc_decode_incremental: two-heap threshold + heap of the k selected keys + attention "
                                "over k+w keys, time of the %d steps alone" % steps},
        "sample": "decode by definition of %d heads on %d threads (%.1f s, all %d steps incl. thresholds and lifetimes "
                  "of the 33 K history), scaled by %d/%d; incremental: %d heads on %d threads (%.2f s wall incl. "
                  "consuming the context, %.3f s for the steps), scaled by %d/%d"
                  % (nd, nd, t_def, steps, B * H, nd, len(data), len(data), t_inc_wall, t_inc_steps, B * H, len(data)),
    }


def decode_leg(steps=256, warm=8, with_cpu=True):
    """Config 5: B=64, H=32, d=128, k=w=1024, context 32768 already consumed, one token per
    sequence per step, `steps` consecutive steps.  Returns the extra JSON object."""
    import torch

    import paper_2406_16747_amd as spk

    B, H, Gu, d, k, w, n_ctx = 64, 32, 1, 128, 1024, 1024, 32768
    g = torch.Generator(device="cuda")
    g.manual_seed(1005)
    div = math.sqrt(d)
    K = torch.empty(B, H, n_ctx, d, device="cuda", dtype=torch.bfloat16)
    V = torch.empty_like(K)
    for b in range(B):  # per batch element, to keep the fp32 temporaries small
        K[b] = (torch.randn(H, n_ctx, d, device="cuda", generator=g) / div).bfloat16()
        V[b] = (torch.randn(H, n_ctx, d, device="cuda", generator=g) / div).bfloat16()
    u = torch.randn(B, Gu, n_ctx, device="cuda", generator=g)
    hist = {}
    if with_cpu:  # histories of a few heads for the CPU baselines, before K and V are dropped
        for i in range(16):
            b, h = (i * 4) % B, (i * 2 + 1) % H
            hist[(b, h)] = (K[b, h].float().cpu().numpy(), V[b, h].float().cpu().numpy(), u[b, 0].cpu().numpy())
    tau, death = spk.sparsek_mask(u, k)
    state = spk.DecodeState(B, H, Gu, d, k, w, torch.bfloat16)
    spk.sparsek_decode_load(state, K, V, u, tau, death)
    torch.cuda.synchronize()
    del K, V
    tot = steps + warm
    qs, ks, vs = ((torch.randn(tot, B, H, d, device="cuda", generator=g) / div).bfloat16() for _ in range(3))
    us = torch.randn(tot, B, Gu, device="cuda", generator=g)
    o = torch.empty(B, H, d, device="cuda", dtype=torch.bfloat16)
    for s in range(warm):
        spk.sparsek_decode_step(state, qs[s], ks[s], vs[s], us[s], out=o)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for s in range(warm, tot):
        ev[s - warm][0].record()
        spk.sparsek_decode_step(state, qs[s], ks[s], vs[s], us[s], out=o)
        ev[s - warm][1].record()
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) / steps * 1e6
    per_step = stats([a.elapsed_time(b) * 1e3 for a, b in ev])
    dev_us = ev[0][0].elapsed_time(ev[-1][1]) / steps * 1e3
    bytes_step = B * H * (k + w) * d * 2 * 2
    gbs = bytes_step / (dev_us * 1e-6) / 1e9
    overflow = bool(spk.sparsek_decode_status(state).any())
    out = {
        "workload": "config 5: decode, B=64 H=32 d=128 k=w=1024 bf16, context 32768, %d steps, Gu=1" % steps,
        "us_per_step": wall_us, "device_us_per_step": dev_us, "device_us_per_step_stats": per_step,
        "tokens_per_s": B / (wall_us * 1e-6), "candidate_overflow": overflow,
        "roofline": {"bound": "hbm", "kernel": "decode_update_kernel + decode_attn_kernel (the whole step)",
                     "achieved": gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "algorithmic_bytes": bytes_step,
                     "traffic": read_traffic("decode_config5_counters.txt")},
    }
    if with_cpu:
        out["cpu_baseline"] = decode_cpu_baseline(hist, qs[warm:], ks[warm:], vs[warm:], us[warm:], n_ctx, k, w, B, H,
                                                  steps)
    return out


def mask_bwd_leg(iters=20, warm=3):
    """Config 3: B=4, H=16, n=8192, d=128, k=w=512, bf16: forward, then the SPARSEK mask backward
    (du of L = sum(dO * O)) and the attention backward (dQ, dK, dV).  Returns the extra JSON object."""
    import torch

    import paper_2406_16747_amd as spk

    B, H, Gu, n, d, k, w = 4, 16, 1, 8192, 128, 512, 512
    g = torch.Generator(device="cuda")
    g.manual_seed(1003)
    div = math.sqrt(d)
    q, kk, v = ((torch.randn(B, H, n, d, device="cuda", generator=g) / div).bfloat16() for _ in range(3))
    dO = torch.randn(B, H, n, d, device="cuda", generator=g).bfloat16()
    pos = torch.arange(n, device="cuda", dtype=torch.float32)
    u = torch.randn(B, Gu, n, device="cuda", generator=g) + 0.5 * torch.sin(pos / 256.0)
    tau, death = spk.sparsek_mask(u, k)
    o, lse = spk.sparsek_attn_fwd(q, kk, v, u, tau, death, k, w, 0, 1.0)

    def timed(fn):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    fwd_ms = timed(lambda: spk.sparsek_attn_fwd(q, kk, v, u, tau, death, k, w, 0, 1.0))
    bwd_ms = timed(lambda: spk.sparsek_mask_bwd(q, kk, v, u, tau, death, o, lse, dO, k, w, 0, 1.0))
    abwd_ms = timed(lambda: spk.sparsek_attn_bwd(q, kk, v, u, tau, death, o, lse, dO, k, w, 0, 1.0))
    # five contractions per attended pair: S = Q.K^T, dO.V^T, dV += P^T.dO, dQ += dS.K, dK += dS^T.Q
    abwd_flops = 10.0 * d * attended_pairs(n, k, w) * B * H
    abwd_ach = abwd_flops / (abwd_ms * 1e-3) / 1e12
    # straight-through variant (gate_mode 3): forward without the gate multiplications, gradient at m = 1
    o_st, lse_st = spk.sparsek_attn_fwd(q, kk, v, u, tau, death, k, w, 3, 1.0)
    st_fwd_ms = timed(lambda: spk.sparsek_attn_fwd(q, kk, v, u, tau, death, k, w, 3, 1.0))
    st_bwd_ms = timed(lambda: spk.sparsek_mask_bwd(q, kk, v, u, tau, death, o_st, lse_st, dO, k, w, 3, 1.0))
    # pairs outside the window are the only ones with a soft gate: two contractions (Q.K^T and dO.V^T) over them
    sel_pairs = attended_pairs(n, k, w) - (n * w - w * (w - 1) // 2)
    flops = 4.0 * d * sel_pairs * B * H
    fwd_flops = 4.0 * d * attended_pairs(n, k, w) * B * H
    ach = flops / (bwd_ms * 1e-3) / 1e12
    return {
        "workload": "config 3: B=4 H=16 n=8192 d=128 k=w=512 bf16, Gu=1, gate_mode=0",
        "attn_fwd_ms": fwd_ms, "attn_fwd_tflops": fwd_flops / (fwd_ms * 1e-3) / 1e12,
        "mask_bwd_ms": bwd_ms,
        "attn_bwd": {"ms": abwd_ms, "fwd_plus_bwd_ms": fwd_ms + abwd_ms + bwd_ms,
                     "roofline": {"bound": "mfma", "kernel": "attn_bwd_dkv_kernel<128> + attn_bwd_dq_kernel<128> + merge",
                                  "achieved": abwd_ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                  "frac": abwd_ach / MFMA_BF16_PEAK_TFLOPS, "algorithmic_flops": abwd_flops,
                                  "traffic": read_traffic("attn_bwd_config3_counters.txt")}},
        "straight_through": {"gate_mode": 3, "attn_fwd_ms": st_fwd_ms, "mask_bwd_ms": st_bwd_ms,
                             "mask_bwd_tflops": flops / (st_bwd_ms * 1e-3) / 1e12},
        "roofline": {"bound": "mfma", "kernel": "mask_bwd_mfma_kernel<128> + epilogue", "achieved": ach,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                     "algorithmic_flops": flops, "traffic": read_traffic("mask_bwd_config3_counters.txt")},
    }


def scores_leg(iters=20, warm=3):
    """Importance scores from hidden states (projection + position slope + timestep normalisation):
    config 2's scorer shape and a Llama-7B-shaped hidden state at 32K.  HBM-bound: the hidden
    states are read once."""
    import torch

    import paper_2406_16747_amd as spk

    res = []
    for name, B, n, D in (("config 2 scorer: B=8 n=4096 D=768 bf16", 8, 4096, 768),
                          ("Llama-7B-shaped hidden state: B=1 n=32768 D=4096 bf16", 1, 32768, 4096)):
        g = torch.Generator(device="cuda")
        g.manual_seed(2000 + D)
        x = torch.randn(B, n, D, device="cuda", generator=g).bfloat16()
        w = torch.randn(D, device="cuda", generator=g) / math.sqrt(D)
        for _ in range(warm):
            spk.sparsek_scores(x, w, 2.0 ** -14, True, 1e-5)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            spk.sparsek_scores(x, w, 2.0 ** -14, True, 1e-5)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        nbytes = B * n * D * 2 + D * 4 + B * n * 4
        gbs = nbytes / (ms * 1e-3) / 1e9
        res.append({"workload": name + ", slope 2^-14, timestep norm", "ms": ms,
                    "roofline": {"bound": "hbm", "kernel": "scores_dot_kernel + partial + norm", "achieved": gbs,
                                 "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                                 "algorithmic_bytes": nbytes, "traffic": None}})
        del x
    return res


def chunk_leg(n=131072, c=8192):
    """Chunk-wise recurrent prefill (fixed-size scored cache): a 128K-token sequence of the config-4
    head shape (H=32, d=128, k=w=1024, bf16) consumed in chunks of 8192; the state never grows."""
    import torch

    import paper_2406_16747_amd as spk

    B, H, d, k, w = 1, 32, 128, 1024, 1024
    g = torch.Generator(device="cuda")
    g.manual_seed(1104)
    div = math.sqrt(d)
    chunks = []
    for _ in range(n // c):  # drawn chunk by chunk: the whole sequence never has to be resident
        q, kk, v = ((torch.randn(B, H, c, d, device="cuda", generator=g) / div).bfloat16() for _ in range(3))
        chunks.append((q, kk, v, torch.randn(B, 1, c, device="cuda", generator=g)))
    st = spk.ChunkState(B, H, 1, d, k, w, spk.BF16, c, 0, 1.0)
    for ch in chunks[:2]:
        spk.sparsek_chunk_prefill(st, *ch)
    st = spk.ChunkState(B, H, 1, d, k, w, spk.BF16, c, 0, 1.0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for ch in chunks:
        spk.sparsek_chunk_prefill(st, *ch)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    counts, flags = spk.sparsek_chunk_status(st)
    flops = 4.0 * d * attended_pairs(n, k, w) * B * H
    ach = flops / (ms * 1e-3) / 1e12
    # training with chunk-wise recurrence: every chunk's forward followed by its backward (cache gradient stopped)
    dOs = [torch.randn(B, H, c, d, device="cuda", generator=g).bfloat16() for _ in range(2)]
    st2 = spk.ChunkState(B, H, 1, d, k, w, spk.BF16, c, 0, 1.0)
    for i, ch in enumerate(chunks[:2]):
        spk.sparsek_chunk_bwd(st2, ch[0], spk.sparsek_chunk_prefill(st2, *ch), dOs[i % 2])
    st2 = spk.ChunkState(B, H, 1, d, k, w, spk.BF16, c, 0, 1.0)
    torch.cuda.synchronize()
    e0.record()
    for i, ch in enumerate(chunks):
        spk.sparsek_chunk_bwd(st2, ch[0], spk.sparsek_chunk_prefill(st2, *ch), dOs[i % 2])
    e1.record()
    torch.cuda.synchronize()
    train_ms = e0.elapsed_time(e1)
    return {"workload": "B=1 H=32 n=%d d=128 k=w=1024 bf16, Gu=1, gate_mode=0, chunks of %d" % (n, c),
            "training": {"ms_total": train_ms, "ms_per_chunk": train_ms / len(chunks),
                         "tokens_per_s": n / (train_ms * 1e-3), "what": "sparsek_chunk_prefill + sparsek_chunk_bwd per chunk",
                         "bwd_workspace_bytes": int(st2.bwd_ws.numel())},
            "ms_total": ms, "ms_per_chunk": ms / len(chunks), "tokens_per_s": n / (ms * 1e-3),
            "retained_entries": int(counts.max()), "overflow": bool(flags.any()),
            "state_bytes": int(st.buf.numel()), "workspace_bytes": int(st.ws.numel()),
            "roofline": {"bound": "mfma", "kernel": "whole chunk step (mask + attn_fwd_mfma_kernel<128> + state upkeep)",
                         "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": ach / MFMA_BF16_PEAK_TFLOPS, "algorithmic_flops": flops,
                         "traffic": read_traffic("chunked_prefill_counters.txt")}}


def source_digest(files):
    """sha256 (first 12 hex digits) over the kernel sources a counter summary was taken on."""
    import hashlib

    h = hashlib.sha256()
    for f in files:
        h.update(open(os.path.join(ROOT, "paper_2406_16747_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:12]


def read_traffic(name):
    """HBM bytes per launch of the dominant kernel (FETCH_SIZE / WRITE_SIZE counters, scaled by the copy-kernel
    calibration) from the committed counter summary -- counters cannot be read inside this process.  The summary
    names the kernel sources it was taken on and their digest; when the sources have changed since, the figure is
    stale and None is returned."""
    path = os.path.join(ROOT, "profiles", name)
    val, files, digest = None, None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                val = float(line.split(":")[1])
            elif line.startswith("kernel_sources:"):
                files = line.split(":")[1].split()
            elif line.startswith("kernel_sources_sha256:"):
                digest = line.split(":")[1].strip()
    except OSError:
        return None
    if val is None or not files or digest != source_digest(files):
        return None
    return val


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--gate-mode", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-bwd", action="store_true")
    ap.add_argument("--no-scores", action="store_true")
    ap.add_argument("--no-chunk", action="store_true")
    ap.add_argument("--no-prefill-configs", action="store_true", help="skip the config 1, 2, 3 prefill legs")
    ap.add_argument("--only", choices=["chunk", "scores", "bwd", "decode", "prefill_c1", "prefill_c2", "prefill_c3"],
                    help="run one of the side legs alone and print its object (for profiling that leg)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy (to calibrate FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch

    import paper_2406_16747_amd as spk

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    spk.lib()  # fail loudly if the HIP library is missing
    if args.only:
        cpu = not args.no_cpu_baseline
        leg = {"chunk": chunk_leg, "scores": scores_leg, "bwd": mask_bwd_leg,
               "decode": lambda: decode_leg(with_cpu=cpu),
               "prefill_c1": lambda: prefill_leg(1, with_cpu=cpu), "prefill_c2": lambda: prefill_leg(2, with_cpu=cpu),
               "prefill_c3": lambda: prefill_leg(3, with_cpu=cpu)}[args.only]
        print(json.dumps({"only": args.only, "result": leg()}))
        return
    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)  # reads 1 GiB, writes 1 GiB per launch
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": a.numel() * 4, "copy_bytes_written": a.numel() * 4, "launches": 3}))
        return

    cfg = dict(B=1, H=32, Gu=1, n=32768, d=128, k=1024, w=1024)
    q, k, v, u = device_inputs(cfg, seed=1004)
    scfg = spk.binding._attn_cfg(q, u, cfg["k"], cfg["w"], args.gate_mode, 1.0)
    import ctypes

    ws = torch.empty(spk.lib().sparsek_attn_fwd_workspace_bytes(ctypes.byref(scfg)), dtype=torch.uint8,
                     device="cuda")

    def step():
        tau, death = spk.sparsek_mask(u, cfg["k"])
        return spk.sparsek_attn_fwd(q, k, v, u, tau, death, cfg["k"], cfg["w"], args.gate_mode, 1.0,
                                    return_lse=True, ws=ws), tau, death

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # whole-step time: exactly K steps between synchronisations; the durations of the mask and of the dominant
    # kernel's launch from HIP events recorded on the launch stream around each call
    ev = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        tau, death = spk.sparsek_mask(u, cfg["k"])
        ev[i][1].record()
        spk.sparsek_attn_fwd(q, k, v, u, tau, death, cfg["k"], cfg["w"], args.gate_mode, 1.0, return_lse=True,
                             ws=ws)
        ev[i][2].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    attn_stats = stats([b.elapsed_time(c) for a, b, c in ev])
    mask_stats = stats([a.elapsed_time(b) for a, b, c in ev])
    step_stats = stats([a.elapsed_time(c) for a, b, c in ev])
    attn_ms = attn_stats["mean"]

    flops = 4.0 * cfg["d"] * attended_pairs(cfg["n"], cfg["k"], cfg["w"]) * cfg["B"] * cfg["H"]
    achieved = flops / (attn_ms * 1e-3) / 1e12
    out = {
        "metric": "SparseK attention fwd tokens/sec at n=32K,k=1024",
        "value": cfg["B"] * cfg["n"] / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "config 4: prefill fwd, B=1 H=32 n=32768 d=128 k=1024 w=1024, Gu=1, gate_mode=%d, "
                               "mask+select+attention per step" % args.gate_mode,
                   "global_batch": cfg["B"], "seq_len": cfg["n"], "parallelism": "single GPU"},
        "roofline": {"bound": "mfma", "kernel": "attn_fwd_mfma_kernel<128>", "achieved": achieved,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                     "ms_per_launch": attn_ms, "algorithmic_flops": flops,
                     "traffic": read_traffic("attn_fwd_mfma_config4_counters.txt")},
        "mask_ms": mask_stats["mean"],
        "device_ms": {"step": step_stats, "mask": mask_stats, "attn": attn_stats},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, q, k, v, u)
    # the same attention launch with the gate applied to the values only, and not at all
    gm = {}
    for mode in (0, 1, 2):
        tau, death = spk.sparsek_mask(u, cfg["k"])
        for _ in range(5):  # the host-side oracle run above leaves the GPU idle: warm up again
            spk.sparsek_attn_fwd(q, k, v, u, tau, death, cfg["k"], cfg["w"], mode, 1.0, return_lse=True, ws=ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            spk.sparsek_attn_fwd(q, k, v, u, tau, death, cfg["k"], cfg["w"], mode, 1.0, return_lse=True, ws=ws)
        e1.record()
        torch.cuda.synchronize()
        gm[str(mode)] = e0.elapsed_time(e1) / 10
    out["attn_ms_by_gate_mode"] = gm

    # variants at the same shape: one score row per head (Gu = H), and selection only (w = 0, k = 2048)
    def step_ms(uu, kk_sel, ww, iters=10):
        wsx = None
        for i in range(3 + iters):
            if i == 3:
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
            if i == 3 + iters - 1:
                m0.record()
            t2, d2 = spk.sparsek_mask(uu, kk_sel)
            if i == 3 + iters - 1:
                m1.record()
            spk.sparsek_attn_fwd(q, k, v, uu, t2, d2, kk_sel, ww, 0, 1.0, return_lse=True, ws=wsx)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters, m0.elapsed_time(m1)

    gq = torch.Generator(device="cuda")
    gq.manual_seed(1204)
    u_heads = torch.randn(cfg["B"], cfg["H"], cfg["n"], device="cuda", generator=gq)
    ms_h, mask_h = step_ms(u_heads, cfg["k"], cfg["w"])
    ms_w0, mask_w0 = step_ms(u, 2 * cfg["k"], 0)
    out["variants"] = {
        "per_head_selection": {"workload": "config 4 shape with Gu=H (32 score rows)", "ms_per_step": ms_h,
                               "mask_ms": mask_h, "tokens_per_s": cfg["B"] * cfg["n"] / (ms_h * 1e-3)},
        "selection_only": {"workload": "config 4 shape with w=0, k=2048", "ms_per_step": ms_w0, "mask_ms": mask_w0,
                           "tokens_per_s": cfg["B"] * cfg["n"] / (ms_w0 * 1e-3)},
    }
    del u_heads
    del q, k, v, ws
    torch.cuda.empty_cache()
    if not args.no_prefill_configs:
        for c in (1, 2, 3):
            out["prefill_c%d" % c] = prefill_leg(c, with_cpu=not args.no_cpu_baseline)
            torch.cuda.empty_cache()
    if not args.no_bwd:
        out["mask_bwd"] = mask_bwd_leg()
        torch.cuda.empty_cache()
    if not args.no_scores:
        out["scores"] = scores_leg()
        torch.cuda.empty_cache()
    if not args.no_chunk:
        out["chunked_prefill"] = chunk_leg()
        torch.cuda.empty_cache()
    if not args.no_decode:
        out["decode"] = decode_leg(with_cpu=not args.no_cpu_baseline)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
