"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and rounds them to the storage type; it holds
none of the method's arithmetic, so both the HIP path and the CPU oracle may be fed
from it.  The recipes stand in for activations of the models the paper trains
(GPT-2-small, Pythia, TinyLlama shapes; scores of about unit variance, as after the
paper's timestep normalisation, Sec. 3.5).

Draw order for a given seed: q, k, v, then the scores (x and w_s for config 2, u
otherwise), then dO when asked for.  bf16 tensors are produced as fp32 draws rounded to
nearest-even; the caller gets both the uint16 bit pattern (for the GPU) and the same
values widened to fp32 (for the oracle).
"""
import math

import numpy as np

# name -> shape parameters.  dtype: storage type of q,k,v,o.  qk_div: q,k,v ~ N(0,1)/qk_div.
CONFIGS = {
    1: dict(B=1, H=1, n=1024, d=64, k=64, w=64, dtype="fp32", qk_div=8.0, scores="normal",
            seed=1001),
    2: dict(B=8, H=12, n=4096, d=64, k=256, w=256, dtype="bf16", qk_div=8.0, scores="scorer",
            hidden=768, seed=1002),
    3: dict(B=4, H=16, n=8192, d=128, k=512, w=512, dtype="bf16", qk_div=math.sqrt(128.0),
            scores="drift", seed=1003),
    4: dict(B=1, H=32, n=32768, d=128, k=1024, w=1024, dtype="bf16", qk_div=math.sqrt(128.0),
            scores="normal", seed=1004),
    5: dict(B=64, H=32, n=32768, d=128, k=1024, w=1024, dtype="bf16", qk_div=math.sqrt(128.0),
            scores="normal", steps=256, seed=1005),
}


def bf16_bits(x):
    """fp32 array -> uint16 bf16 bit patterns, round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_widen(bits):
    """uint16 bf16 bit patterns -> the same values as fp32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x, dtype):
    """Returns (storage array for the GPU, fp32 values for the oracle)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp32":
        return x, x
    bits = bf16_bits(x)
    return bits, bf16_widen(bits)


def draw_scores(rng, kind, B, Gu, n, hidden=768):
    """The score tensor u [B,Gu,n] fp32 of a configuration."""
    if kind == "normal":
        return rng.standard_normal((B, Gu, n), dtype=np.float32)
    if kind == "drift":  # clustered important positions: slow sinusoidal drift
        base = rng.standard_normal((B, Gu, n), dtype=np.float32)
        pos = np.arange(n, dtype=np.float32)
        return (base + np.float32(0.5) * np.sin(pos / np.float32(256.0))).astype(np.float32)
    if kind == "scorer":  # a linear scorer on a hidden state; one group by construction
        assert Gu == 1
        x = rng.standard_normal((B, n, hidden), dtype=np.float32)
        ws = (rng.standard_normal(hidden, dtype=np.float32) / np.float32(math.sqrt(hidden)))
        return (x @ ws).astype(np.float32).reshape(B, 1, n)
    raise ValueError(kind)


def make(config, Gu=1, seed=None, with_dO=False, **override):
    """Host-side inputs of one configuration (optionally shrunk through ``override``).

    Returns a dict: shape parameters, ``scale`` (softmax scale, 1.0: the recipes already
    divide q,k by sqrt(d) or 8), storage arrays ``Q,K,V[,dO]`` (fp32 or uint16 bf16 bits)
    and their fp32 values ``Q32,K32,V32[,dO32]``, and ``u`` [B,Gu,n] fp32.
    """
    p = dict(CONFIGS[config])
    p.update(override)
    if seed is None:
        seed = p["seed"]
    B, H, n, d = p["B"], p["H"], p["n"], p["d"]
    rng = np.random.default_rng(seed)
    out = dict(p)
    out.update(Gu=Gu, seed=seed, scale=1.0)
    div = np.float32(p["qk_div"])
    for name in ("Q", "K", "V"):
        x = rng.standard_normal((B, H, n, d), dtype=np.float32) / div
        out[name], out[name + "32"] = _store(x, p["dtype"])
    out["u"] = draw_scores(rng, p["scores"], B, Gu, n, p.get("hidden", 768))
    if with_dO:
        x = rng.standard_normal((B, H, n, d), dtype=np.float32)
        out["dO"], out["dO32"] = _store(x, p["dtype"])
    return out


def decode_steps(config, B, H, Gu, d, steps, seed, dtype="bf16", qk_div=None):
    """Per-step decode inputs: Q,K,V [steps,B,H,d] (+ their fp32 values Q32,K32,V32) and u [steps,B,Gu]."""
    p = CONFIGS[config]
    div = np.float32(qk_div if qk_div is not None else p["qk_div"])
    rng = np.random.default_rng(seed)
    out = {}
    for name in ("Q", "K", "V"):
        x = rng.standard_normal((steps, B, H, d), dtype=np.float32) / div
        out[name], out[name + "32"] = _store(x, dtype)
    out["u"] = rng.standard_normal((steps, B, Gu), dtype=np.float32)
    return out


def to_device(arr, dtype, device="cuda"):
    """Storage array from ``make`` -> torch tensor on the device (bf16 bits reinterpreted)."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(arr))
    if dtype == "bf16" and arr.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.to(device)


def hidden_states(B, n, D, seed, dtype="bf16", offset=0.0):
    """Hidden states x [B,n,D] ~ N(offset,1) in the storage type and a scorer w [D] ~ N(0,1/D)
    fp32 (the recipe of config 2's scores).  Returns (storage array, fp32 values, w)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, n, D), dtype=np.float32) + np.float32(offset)
    w = rng.standard_normal(D, dtype=np.float32) / np.float32(math.sqrt(D))
    xs, x32 = _store(x, dtype)
    return xs, x32, w

