#!/usr/bin/env python3
"""Benchmark of the SparseK hot path on one MI355X.

A step is one pass of the whole prefill path over one batch of synthetic input:
sparsek_mask (thresholds + lifetimes) followed by sparsek_attn_fwd, at the
Llama-7B-shaped long-context configuration (B=1, H=32, n=32768, d=128, k=w=1024, bf16).
Inputs are resident in HBM before the timed region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-bwd] [--no-decode] [--no-scores] [--no-chunk] [--only LEG]
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
    return {
        "value": cfg["B"] * n / t_full,
        "unit": "tokens/s",
        "cores": cores,
        "kind": "oracle",
        "sample": "tau+lifetimes of the full score row (%.1f s) and query rows %d..%d of %d heads "
                  "(%.1f s), attention time scaled by attended pairs to all %d heads x %d rows"
                  % (t_mask, a, e - 1, len(heads), t_attn, H, n),
    }


def decode_leg(steps=256, warm=8):
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
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for s in range(warm, tot):
        spk.sparsek_decode_step(state, qs[s], ks[s], vs[s], us[s], out=o)
    e1.record()
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) / steps * 1e6
    dev_us = e0.elapsed_time(e1) / steps * 1e3
    bytes_step = B * H * (k + w) * d * 2 * 2
    gbs = bytes_step / (dev_us * 1e-6) / 1e9
    overflow = bool(spk.sparsek_decode_status(state).any())
    return {
        "workload": "config 5: decode, B=64 H=32 d=128 k=w=1024 bf16, context 32768, %d steps, Gu=1" % steps,
        "us_per_step": wall_us, "device_us_per_step": dev_us, "tokens_per_s": B / (wall_us * 1e-6),
        "candidate_overflow": overflow,
        "roofline": {"bound": "hbm", "kernel": "decode_attn_kernel", "achieved": gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "algorithmic_bytes": bytes_step,
                     "traffic": read_traffic("decode_config5_counters.txt")},
    }


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
                                  "traffic": None}},
        "straight_through": {"gate_mode": 3, "attn_fwd_ms": st_fwd_ms, "mask_bwd_ms": st_bwd_ms,
                             "mask_bwd_tflops": flops / (st_bwd_ms * 1e-3) / 1e12},
        "roofline": {"bound": "mfma", "kernel": "mask_bwd_mfma_kernel<128> + epilogue", "achieved": ach,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                     "algorithmic_flops": flops, "traffic": None},
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
                         "frac": ach / MFMA_BF16_PEAK_TFLOPS, "algorithmic_flops": flops, "traffic": None}}


def read_traffic(name):
    """HBM bytes per launch of the dominant kernel, from the committed counter summary."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


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
    ap.add_argument("--only", choices=["chunk", "scores", "bwd", "decode"],
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
        leg = {"chunk": chunk_leg, "scores": scores_leg, "bwd": mask_bwd_leg, "decode": decode_leg}[args.only]
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

    # whole-step time: exactly K steps between synchronisations; the dominant kernel's own
    # duration from HIP events recorded on the launch stream around each attention call
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        tau, death = spk.sparsek_mask(u, cfg["k"])
        ev[i][0].record()
        spk.sparsek_attn_fwd(q, k, v, u, tau, death, cfg["k"], cfg["w"], args.gate_mode, 1.0, return_lse=True,
                             ws=ws)
        ev[i][1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    attn_ms = sum(a.elapsed_time(b) for a, b in ev) / args.steps

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
        "mask_ms": ms_per_step - attn_ms,
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
        out["decode"] = decode_leg()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
