"""ctypes binding of libsparsek.so.  Function names mirror include/sparsek.h."""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsparsek.so")
_lib = None

F32, BF16 = 0, 1


class SparsekCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "H", "Gu", "n", "d", "k", "w", "dtype", "gate_mode")] + [
        ("softmax_scale", C.c_float)
    ]


class SparsekScoresCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "n", "D", "dtype", "norm")] + [("slope", C.c_float), ("norm_eps", C.c_float)]


class SparsekChunkCfg(C.Structure):
    _fields_ = [
        (n, C.c_int32) for n in ("B", "H", "Gu", "d", "k", "w", "cand_cap", "chunk_max", "dtype", "gate_mode")
    ] + [("softmax_scale", C.c_float)]


class SparsekDecodeCfg(C.Structure):
    _fields_ = [
        (n, C.c_int32) for n in ("B", "H", "Gu", "d", "k", "w", "cand_cap", "dtype", "gate_mode")
    ] + [("softmax_scale", C.c_float)]


def lib_path():
    return _LIB_PATH


def lib():
    """The loaded C-ABI library.  Raises if it has not been built (no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                "libsparsek.so is missing: build it with `python -m paper_2406_16747_amd.build` "
                "(there is no CPU fallback)"
            )
        L = C.CDLL(_LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        cfgp, dcfgp = C.POINTER(SparsekCfg), C.POINTER(SparsekDecodeCfg)
        L.sparsek_strerror.restype = C.c_char_p
        L.sparsek_strerror.argtypes = [C.c_int]
        for name in ("sparsek_mask_workspace_bytes", "sparsek_attn_fwd_workspace_bytes",
                     "sparsek_mask_bwd_workspace_bytes", "sparsek_attn_bwd_workspace_bytes"):
            getattr(L, name).restype = sz
            getattr(L, name).argtypes = [cfgp]
        L.sparsek_mask.argtypes = [cfgp, vp, vp, vp, vp, sz, vp]
        L.sparsek_mask_status.argtypes = [cfgp, vp, sz, vp, vp]
        L.sparsek_mask_status.restype = C.c_int
        L.sparsek_mask_static.argtypes = [cfgp, vp, vp, vp, vp]
        L.sparsek_mask_static.restype = C.c_int
        L.sparsek_materialize.argtypes = [cfgp, vp, vp, vp, i32, i32, vp, vp, vp]
        L.sparsek_attn_fwd.argtypes = [cfgp] + [vp] * 8 + [vp, sz, vp]
        L.sparsek_mask_bwd.argtypes = [cfgp] + [vp] * 10 + [vp, sz, vp]
        L.sparsek_attn_bwd.argtypes = [cfgp] + [vp] * 12 + [vp, sz, vp]
        L.sparsek_attn_bwd.restype = C.c_int
        L.sparsek_bwd.argtypes = [cfgp] + [vp] * 13 + [vp, sz, vp]
        L.sparsek_bwd.restype = C.c_int
        L.sparsek_bwd_workspace_bytes.restype = sz
        L.sparsek_bwd_workspace_bytes.argtypes = [cfgp]
        scfgp = C.POINTER(SparsekScoresCfg)
        L.sparsek_scores_workspace_bytes.restype = sz
        L.sparsek_scores_workspace_bytes.argtypes = [scfgp]
        L.sparsek_scores.argtypes = [scfgp, vp, vp, vp, vp, sz, vp]
        L.sparsek_scores.restype = C.c_int
        ccfgp = C.POINTER(SparsekChunkCfg)
        for name in ("sparsek_chunk_state_bytes", "sparsek_chunk_workspace_bytes", "sparsek_chunk_bwd_workspace_bytes"):
            getattr(L, name).restype = sz
            getattr(L, name).argtypes = [ccfgp]
        L.sparsek_chunk_init.argtypes = [ccfgp, vp, sz, vp]
        L.sparsek_chunk_prefill.argtypes = [ccfgp, vp, sz, i32] + [vp] * 5 + [vp, sz, vp]
        L.sparsek_chunk_status.argtypes = [ccfgp, vp, vp, vp, vp]
        L.sparsek_chunk_bwd.argtypes = [ccfgp, i32, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp, sz, vp]
        L.sparsek_chunk_bwd.restype = C.c_int
        L.sparsek_chunk_to_decode.argtypes = [ccfgp, vp, sz, C.c_int64, vp, sz, dcfgp, vp, sz, vp]
        for name in ("sparsek_chunk_init", "sparsek_chunk_prefill", "sparsek_chunk_status", "sparsek_chunk_to_decode"):
            getattr(L, name).restype = C.c_int
        L.sparsek_decode_state_bytes.restype = sz
        L.sparsek_decode_state_bytes.argtypes = [dcfgp]
        L.sparsek_decode_init.argtypes = [dcfgp, vp, sz, vp]
        L.sparsek_decode_load.argtypes = [dcfgp, vp, sz, i32] + [vp] * 5 + [vp]
        L.sparsek_decode_step.argtypes = [dcfgp, vp] + [vp] * 5 + [vp]
        L.sparsek_decode_status.argtypes = [dcfgp, vp, vp, vp]
        for name in ("sparsek_mask", "sparsek_materialize", "sparsek_attn_fwd", "sparsek_mask_bwd",
                     "sparsek_decode_init", "sparsek_decode_load", "sparsek_decode_step",
                     "sparsek_decode_status"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def check(rc):
    if rc != 0:
        raise RuntimeError("libsparsek: %s (%d)" % (lib().sparsek_strerror(rc).decode(), rc))


def _torch():
    import torch

    return torch


def _stream():
    return C.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _dtype_code(t):
    torch = _torch()
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("q,k,v must be float32 or bfloat16, got %s" % t.dtype)


def _need(t, dtype, name):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise ValueError("%s must be a contiguous %s tensor on the GPU" % (name, dtype))


def _ws(nbytes, device):
    return _torch().empty(max(int(nbytes), 256), dtype=_torch().uint8, device=device)


def _mask_cfg(u, k):
    B, Gu, n = u.shape
    return SparsekCfg(B=B, H=Gu, Gu=Gu, n=n, d=64, k=int(k), w=1, dtype=F32, gate_mode=0, softmax_scale=1.0)


def sparsek_mask(u, k, ws=None):
    """u [B,Gu,n] fp32 -> (tau [B,Gu,n] fp32, death [B,Gu,n] int32)."""
    torch = _torch()
    _need(u, torch.float32, "u")
    cfg = _mask_cfg(u, k)
    tau = torch.empty_like(u)
    death = torch.empty(u.shape, dtype=torch.int32, device=u.device)
    if ws is None:
        ws = _ws(lib().sparsek_mask_workspace_bytes(C.byref(cfg)), u.device)
    check(lib().sparsek_mask(C.byref(cfg), _ptr(u), _ptr(tau), _ptr(death), _ptr(ws), ws.numel(), _stream()))
    return tau, death


def sparsek_mask_static(u, k, tau=None, death=None):
    """sparsek_mask without a workspace (the library's built-in scratch array); tau, death may be preallocated."""
    torch = _torch()
    _need(u, torch.float32, "u")
    cfg = _mask_cfg(u, k)
    if tau is None:
        tau = torch.empty_like(u)
    if death is None:
        death = torch.empty(u.shape, dtype=torch.int32, device=u.device)
    _need(tau, torch.float32, "tau")
    _need(death, torch.int32, "death")
    check(lib().sparsek_mask_static(C.byref(cfg), _ptr(u), _ptr(tau), _ptr(death), _stream()))
    return tau, death


def sparsek_mask_workspace(u, k):
    """A workspace for sparsek_mask(u, k, ws=...), to be read back with sparsek_mask_status."""
    return _ws(lib().sparsek_mask_workspace_bytes(C.byref(_mask_cfg(u, k))), u.device)


def sparsek_mask_status(u, k, ws):
    """Status word of the last sparsek_mask(u, k, ws=ws) call (0 = every threshold solve converged).  Synchronises."""
    flag = C.c_int32(-1)
    check(lib().sparsek_mask_status(C.byref(_mask_cfg(u, k)), _ptr(ws), ws.numel(), C.byref(flag), _stream()))
    return int(flag.value)


def sparsek_materialize(u, tau, death, k, t_begin, t_end, with_gate=True):
    """Explicit top-k lists of prefixes [t_begin, t_end): idx, gate [B,Gu,nt,k]."""
    torch = _torch()
    B, Gu, n = u.shape
    cfg = SparsekCfg(B=B, H=Gu, Gu=Gu, n=n, d=64, k=int(k), w=1, dtype=F32, gate_mode=0, softmax_scale=1.0)
    nt = t_end - t_begin
    idx = torch.full((B, Gu, nt, max(int(k), 0)), -1, dtype=torch.int32, device=u.device)
    gate = torch.zeros((B, Gu, nt, max(int(k), 0)), dtype=torch.float32, device=u.device) if with_gate else None
    if idx.numel() == 0:
        return idx, gate
    check(lib().sparsek_materialize(C.byref(cfg), _ptr(u), _ptr(tau), _ptr(death), int(t_begin), int(t_end),
                                    _ptr(idx), _ptr(gate), _stream()))
    return idx, gate


def _attn_cfg(q, u, k, w, gate_mode, scale):
    B, H, n, d = q.shape
    Gu = u.shape[1]
    return SparsekCfg(B=B, H=H, Gu=Gu, n=n, d=d, k=int(k), w=int(w), dtype=_dtype_code(q),
                      gate_mode=int(gate_mode), softmax_scale=float(scale))


def sparsek_attn_fwd(q, k, v, u, tau, death, k_sel, w, gate_mode=0, scale=1.0, return_lse=True, ws=None):
    """q,k,v [B,H,n,d]; u,tau,death [B,Gu,n] -> o [B,H,n,d] (and lse [B,H,n] fp32)."""
    torch = _torch()
    cfg = _attn_cfg(q, u, k_sel, w, gate_mode, scale)
    for t, name in ((q, "q"), (k, "k"), (v, "v")):
        _need(t, q.dtype, name)
    _need(u, torch.float32, "u")
    _need(tau, torch.float32, "tau")
    _need(death, torch.int32, "death")
    o = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device) if return_lse else None
    if ws is None:
        ws = _ws(lib().sparsek_attn_fwd_workspace_bytes(C.byref(cfg)), q.device)
    check(lib().sparsek_attn_fwd(C.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(u), _ptr(tau), _ptr(death),
                                 _ptr(o), _ptr(lse), _ptr(ws), ws.numel(), _stream()))
    return (o, lse) if return_lse else o


def sparsek_mask_bwd(q, k, v, u, tau, death, o, lse, dO, k_sel, w, gate_mode=0, scale=1.0, ws=None):
    """du [B,Gu,n] fp32: gradient of sum(dO*O) w.r.t. the scores through the soft gates."""
    torch = _torch()
    cfg = _attn_cfg(q, u, k_sel, w, gate_mode, scale)
    du = torch.empty_like(u)
    if ws is None:
        ws = _ws(lib().sparsek_mask_bwd_workspace_bytes(C.byref(cfg)), q.device)
    check(lib().sparsek_mask_bwd(C.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(u), _ptr(tau), _ptr(death),
                                 _ptr(o), _ptr(lse), _ptr(dO), _ptr(du), _ptr(ws), ws.numel(), _stream()))
    return du


def sparsek_attn_bwd(q, k, v, u, tau, death, o, lse, dO, k_sel, w, gate_mode=0, scale=1.0, ws=None):
    """dq, dk, dv [B,H,n,d]: gradients of sum(dO*O) with respect to q, k, v (gates held fixed)."""
    torch = _torch()
    cfg = _attn_cfg(q, u, k_sel, w, gate_mode, scale)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    if ws is None:
        ws = _ws(lib().sparsek_attn_bwd_workspace_bytes(C.byref(cfg)), q.device)
    check(lib().sparsek_attn_bwd(C.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(u), _ptr(tau), _ptr(death), _ptr(o),
                                 _ptr(lse), _ptr(dO), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), ws.numel(), _stream()))
    return dq, dk, dv


def sparsek_bwd(q, k, v, u, tau, death, o, lse, dO, k_sel, w, gate_mode=0, scale=1.0, ws=None):
    """The whole backward in one call: (dq, dk, dv, du)."""
    torch = _torch()
    cfg = _attn_cfg(q, u, k_sel, w, gate_mode, scale)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    du = torch.empty_like(u)
    if ws is None:
        ws = _ws(lib().sparsek_bwd_workspace_bytes(C.byref(cfg)), q.device)
    check(lib().sparsek_bwd(C.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(u), _ptr(tau), _ptr(death), _ptr(o), _ptr(lse),
                            _ptr(dO), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(du), _ptr(ws), ws.numel(), _stream()))
    return dq, dk, dv, du


def sparsek_scores(x, w, slope=0.0, norm=False, norm_eps=1e-5, ws=None):
    """u [B,n] fp32 from hidden states x [B,n,D] (bf16 or fp32) and the scorer w [D] fp32:
    x.w + position slope, optionally timestep-normalised."""
    torch = _torch()
    B, n, D = x.shape
    assert x.is_contiguous() and w.is_contiguous() and w.dtype == torch.float32 and w.numel() == D
    dt = BF16 if x.dtype == torch.bfloat16 else F32
    assert dt == BF16 or x.dtype == torch.float32
    cfg = SparsekScoresCfg(B=B, n=n, D=D, dtype=dt, norm=int(bool(norm)), slope=float(slope), norm_eps=float(norm_eps))
    u = torch.empty(B, n, dtype=torch.float32, device=x.device)
    if ws is None:
        ws = _ws(lib().sparsek_scores_workspace_bytes(C.byref(cfg)), x.device)
    check(lib().sparsek_scores(C.byref(cfg), _ptr(x), _ptr(w), _ptr(u), _ptr(ws), ws.numel(), _stream()))
    return u


class ChunkState:
    """Caller-owned state of the chunk-wise recurrent prefill: a config, the state buffer and scratch."""

    def __init__(self, B, H, Gu, d, k, w, dtype, chunk_max, gate_mode=0, scale=1.0, cand_cap=0, device="cuda"):
        torch = _torch()
        self.cfg = SparsekChunkCfg(B=B, H=H, Gu=Gu, d=d, k=int(k), w=int(w), cand_cap=int(cand_cap),
                                   chunk_max=int(chunk_max), dtype=dtype, gate_mode=int(gate_mode),
                                   softmax_scale=float(scale))
        nbytes = lib().sparsek_chunk_state_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise ValueError("invalid chunk configuration")
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.ws = torch.empty(lib().sparsek_chunk_workspace_bytes(C.byref(self.cfg)), dtype=torch.uint8, device=device)
        check(lib().sparsek_chunk_init(C.byref(self.cfg), _ptr(self.buf), self.buf.numel(), _stream()))


def sparsek_chunk_prefill(state, q, k, v, u):
    """Attention output [B,H,c,d] of one chunk; the state moves on to the end of the chunk."""
    torch = _torch()
    c = q.shape[2]
    o = torch.empty_like(q)
    check(lib().sparsek_chunk_prefill(C.byref(state.cfg), _ptr(state.buf), state.buf.numel(), c, _ptr(q), _ptr(k),
                                      _ptr(v), _ptr(u), _ptr(o), _ptr(state.ws), state.ws.numel(), _stream()))
    return o


def sparsek_chunk_bwd(state, q, o, dO):
    """Gradients (dq, dk, dv [B,H,c,d], du [B,Gu,c]) of sum(dO * o) for the chunk that the last
    sparsek_chunk_prefill call on this state processed, the retained keys of earlier chunks held constant."""
    torch = _torch()
    c = q.shape[2]
    nbytes = lib().sparsek_chunk_bwd_workspace_bytes(C.byref(state.cfg))
    if nbytes == 0:
        raise ValueError("sparsek_chunk_bwd: unsupported configuration (bf16 with d = 64 or 128 only)")
    if getattr(state, "bwd_ws", None) is None or state.bwd_ws.numel() < nbytes:
        state.bwd_ws = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    du = torch.empty((state.cfg.B, state.cfg.Gu, c), dtype=torch.float32, device=q.device)
    check(lib().sparsek_chunk_bwd(C.byref(state.cfg), c, _ptr(q), _ptr(o), _ptr(dO), _ptr(state.ws), state.ws.numel(),
                                  _ptr(dq), _ptr(dk), _ptr(dv), _ptr(du), _ptr(state.bwd_ws), state.bwd_ws.numel(),
                                  _stream()))
    return dq, dk, dv, du


def sparsek_chunk_to_decode(state, n_consumed, decode_state):
    """Fills a DecodeState with the state after the n_consumed tokens the chunks have covered."""
    check(lib().sparsek_chunk_to_decode(C.byref(state.cfg), _ptr(state.buf), state.buf.numel(), int(n_consumed),
                                        _ptr(state.ws), state.ws.numel(), C.byref(decode_state.cfg),
                                        _ptr(decode_state.buf), decode_state.buf.numel(), _stream()))


def sparsek_chunk_status(state):
    """(retained entries, flag word) per score row, as two int32 numpy arrays; synchronises."""
    import numpy as np

    rows = state.cfg.B * state.cfg.Gu
    counts = np.zeros(rows, np.int32)
    flags = np.zeros(rows, np.int32)
    check(lib().sparsek_chunk_status(C.byref(state.cfg), _ptr(state.buf), counts.ctypes.data_as(C.c_void_p),
                                     flags.ctypes.data_as(C.c_void_p), _stream()))
    return counts, flags


class DecodeState:
    """Caller-owned decode state: a config plus one device buffer."""

    def __init__(self, B, H, Gu, d, k, w, dtype, gate_mode=0, scale=1.0, cand_cap=0, device="cuda"):
        torch = _torch()
        self.cfg = SparsekDecodeCfg(B=B, H=H, Gu=Gu, d=d, k=int(k), w=int(w), cand_cap=int(cand_cap),
                                    dtype=BF16 if dtype == torch.bfloat16 else F32,
                                    gate_mode=int(gate_mode), softmax_scale=float(scale))
        self.torch_dtype = dtype
        nbytes = lib().sparsek_decode_state_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise ValueError("unsupported decode configuration")
        self.buf = torch.empty(int(nbytes), dtype=torch.uint8, device=device)


def sparsek_decode_init(state):
    check(lib().sparsek_decode_init(C.byref(state.cfg), _ptr(state.buf), state.buf.numel(), _stream()))


def sparsek_decode_load(state, k, v, u, tau, death):
    n_ctx = k.shape[2]
    check(lib().sparsek_decode_load(C.byref(state.cfg), _ptr(state.buf), state.buf.numel(), int(n_ctx),
                                    _ptr(k), _ptr(v), _ptr(u), _ptr(tau), _ptr(death), _stream()))


def sparsek_decode_step(state, q_new, k_new, v_new, u_new, out=None):
    torch = _torch()
    o = out if out is not None else torch.empty_like(q_new)
    check(lib().sparsek_decode_step(C.byref(state.cfg), _ptr(state.buf), _ptr(q_new), _ptr(k_new),
                                    _ptr(v_new), _ptr(u_new), _ptr(o), _stream()))
    return o


def sparsek_decode_status(state):
    import numpy as np

    flags = np.zeros(state.cfg.B * state.cfg.Gu, np.int32)
    check(lib().sparsek_decode_status(C.byref(state.cfg), _ptr(state.buf),
                                      flags.ctypes.data_as(C.c_void_p), _stream()))
    return flags
