"""numpy/ctypes face of the plain-C oracle (test infrastructure, see sparsek_oracle.c).

Every function takes and returns numpy arrays; floating-point results are fp64.
Inputs that the GPU receives as bf16 are passed here as the same values widened to
fp32.  Section/equation references are to arXiv 2406.16747.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparsek_oracle.c")
_SO = os.path.join(_HERE, "libsparsek_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (about a second).  Rebuilds when the source is newer."""
    global _lib
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _SO)
        _lib = None
    return _SO


def _L():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def max_threads():
    return int(_L().orc_max_threads())


def sparsek(z, k):
    """SPARSEK(z, k) (Sec. 3.3): returns tau, mask p, u*, w*."""
    z = _f32(z)
    m = z.shape[0]
    tau = C.c_double()
    p = np.empty(m, np.float64)
    us, ws = C.c_int(), C.c_int()
    rc = _L().orc_sparsek(_p(z), m, int(k), C.byref(tau), _p(p), C.byref(us), C.byref(ws))
    assert rc == 0
    return tau.value, p, us.value, ws.value


def tau_prefixes(u_row, k):
    """tau_t, u*_t, w*_t of every causal prefix of one score row."""
    u_row = _f32(u_row)
    n = u_row.shape[0]
    tau = np.empty(n, np.float64)
    us = np.empty(n, np.int32)
    ws = np.empty(n, np.int32)
    rc = _L().orc_tau_prefixes(_p(u_row), n, int(k), _p(tau), _p(us), _p(ws))
    assert rc == 0
    return tau, us, ws


def select_prefix(u_row, t, k):
    """Hard top-k of prefix t (Sec. 3.2), ascending positions."""
    u_row = _f32(u_row)
    idx = np.empty(t + 1, np.int32)
    cnt = _L().orc_select_prefix(_p(u_row), int(t), int(k), _p(idx))
    return idx[:cnt].copy()


def death(u_row, k):
    """death[j] = first prefix t >= j whose top-k no longer holds j (n if none)."""
    u_row = _f32(u_row)
    n = u_row.shape[0]
    out = np.empty(n, np.int32)
    rc = _L().orc_death(_p(u_row), n, int(k), _p(out))
    assert rc == 0
    return out


def attn_query_bydef(q, K, V, u_row, k, w, gate_mode, scale, i):
    """One query of one head with tau and the top-k recomputed from scratch."""
    q, K, V, u_row = _f32(q), _f32(K), _f32(V), _f32(u_row)
    n, d = K.shape
    o = np.empty(d, np.float64)
    lse = C.c_double()
    rc = _L().orc_attn_query_bydef(
        _p(q), _p(K), _p(V), _p(u_row), n, d, int(k), int(w), int(gate_mode),
        C.c_double(scale), int(i), _p(o), C.byref(lse),
    )
    assert rc == 0
    return o, lse.value


def attn_rows(q, K, V, u_row, tau_row, death_row, k, w, gate_mode, scale, i_begin, i_end):
    """Rows [i_begin, i_end) of one head.  q,K,V [n,d]."""
    q, K, V, u_row = _f32(q), _f32(K), _f32(V), _f32(u_row)
    tau_row, death_row = _f64(tau_row), _i32(death_row)
    n, d = K.shape
    nr = i_end - i_begin
    o = np.empty((nr, d), np.float64)
    lse = np.empty(nr, np.float64)
    rc = _L().orc_attn_rows(
        _p(q), _p(K), _p(V), _p(u_row), _p(tau_row), _p(death_row), n, d, int(k), int(w),
        int(gate_mode), C.c_double(scale), int(i_begin), int(i_end), _p(o), _p(lse),
    )
    assert rc == 0
    return o, lse


def mask_all(u, k):
    """tau [B,Gu,n] fp64 and death [B,Gu,n] int32 for a whole score tensor."""
    u = _f32(u)
    B, Gu, n = u.shape
    tau = np.empty((B, Gu, n), np.float64)
    dth = np.empty((B, Gu, n), np.int32)
    for b in range(B):
        for g in range(Gu):
            tau[b, g] = tau_prefixes(u[b, g], k)[0]
            dth[b, g] = death(u[b, g], k)
    return tau, dth


def attn_fwd(q, K, V, u, tau, dth, k, w, gate_mode, scale, nthreads=0):
    """All heads.  q,K,V [B,H,n,d]; u,tau,death [B,Gu,n].  Returns o, lse, threads used."""
    q, K, V, u = _f32(q), _f32(K), _f32(V), _f32(u)
    tau, dth = _f64(tau), _i32(dth)
    B, H, n, d = q.shape
    Gu = u.shape[1]
    o = np.empty((B, H, n, d), np.float64)
    lse = np.empty((B, H, n), np.float64)
    used = _L().orc_attn_fwd(
        _p(q), _p(K), _p(V), _p(u), _p(tau), _p(dth), B, H, Gu, n, d, int(k), int(w),
        int(gate_mode), C.c_double(scale), _p(o), _p(lse), int(nthreads),
    )
    assert used > 0
    return o, lse, used


def mask_bwd(q, K, V, u, tau, dth, dO, k, w, gate_mode, scale, nthreads=0):
    """du [B,Gu,n] of L = sum(dO*O) through the soft gates (App. A.3)."""
    q, K, V, u, dO = _f32(q), _f32(K), _f32(V), _f32(u), _f32(dO)
    tau, dth = _f64(tau), _i32(dth)
    B, H, n, d = q.shape
    Gu = u.shape[1]
    du = np.empty((B, Gu, n), np.float64)
    used = _L().orc_mask_bwd(
        _p(q), _p(K), _p(V), _p(u), _p(tau), _p(dth), _p(dO), B, H, Gu, n, d, int(k), int(w),
        int(gate_mode), C.c_double(scale), _p(du), int(nthreads),
    )
    assert used > 0
    return du, used


def attn_bwd(q, K, V, u, tau, dth, dO, k, w, gate_mode, scale, nthreads=0):
    """dQ, dK, dV [B,H,n,d] fp64 of L = sum(dO*O), the gates held fixed (their gradient is mask_bwd)."""
    q, K, V, u, dO = _f32(q), _f32(K), _f32(V), _f32(u), _f32(dO)
    tau, dth = _f64(tau), _i32(dth)
    B, H, n, d = q.shape
    Gu = u.shape[1]
    dQ, dK, dV = (np.empty((B, H, n, d), np.float64) for _ in range(3))
    used = _L().orc_attn_bwd(
        _p(q), _p(K), _p(V), _p(u), _p(tau), _p(dth), _p(dO), B, H, Gu, n, d, int(k), int(w),
        int(gate_mode), C.c_double(scale), _p(dQ), _p(dK), _p(dV), int(nthreads),
    )
    assert used > 0
    return dQ, dK, dV


def decode_bydef(q_steps, K_hist, V_hist, u_hist, n_ctx, k, w, gate_mode, scale):
    """Decode by definition for one head: the output of the step that appends position t
    is row t of the prefill attention over the whole history (the chunk-recurrence
    equivalence of Sec. 3.4).  q_steps [steps,d] are the queries of positions
    n_ctx .. n_ctx+steps-1; K_hist, V_hist [n_ctx+steps, d]; u_hist [n_ctx+steps]."""
    q_steps = _f32(q_steps)
    steps, d = q_steps.shape
    n = n_ctx + steps
    assert K_hist.shape[0] == n and u_hist.shape[0] == n
    tau = tau_prefixes(u_hist, k)[0]
    dth = death(u_hist, k)
    q_full = np.zeros((n, d), np.float32)
    q_full[n_ctx:] = q_steps
    o, _ = attn_rows(q_full, K_hist, V_hist, u_hist, tau, dth, k, w, gate_mode, scale, n_ctx, n)
    return o


def tau_incremental(u_row, k):
    """tau_t of every causal prefix by the incremental two-heap evaluation of Sec. 3.3."""
    u_row = _f32(u_row)
    n = u_row.shape[0]
    tau = np.empty(n, np.float64)
    rc = _L().orc_tau_incremental(_p(u_row), n, int(k), _p(tau))
    assert rc == 0
    return tau


def decode_incremental(q_steps, K_hist, V_hist, u_hist, n_ctx, k, w, gate_mode, scale):
    """Decode of one head with constant work per token (incremental threshold, top-k as a heap of k keys,
    attention over k + w keys).  Same arguments and result as decode_bydef; also returns the seconds spent in
    the steps alone."""
    q_steps, K_hist, V_hist, u_hist = _f32(q_steps), _f32(K_hist), _f32(V_hist), _f32(u_hist)
    steps, d = q_steps.shape
    assert K_hist.shape[0] == n_ctx + steps and u_hist.shape[0] == n_ctx + steps
    o = np.empty((steps, d), np.float64)
    sec = C.c_double(0.0)
    rc = _L().orc_decode_incremental(_p(q_steps), _p(K_hist), _p(V_hist), _p(u_hist), int(n_ctx), int(steps), int(d),
                                     int(k), int(w), int(gate_mode), C.c_double(scale), _p(o), C.byref(sec))
    assert rc == 0
    return o, sec.value


def scores(X, w, slope=0.0, norm=False, norm_eps=1e-5):
    """Importance scores u [B,n] fp64 from hidden states X [B,n,D] and the scorer w [D]:
    X.w plus the position slope, optionally timestep-normalised (Sec. 3.2 / Sec. 3.5)."""
    X = _f32(X)
    w = _f32(w)
    B, n, D = X.shape
    u = np.zeros((B, n), np.float64)
    rc = _L().orc_scores(_p(X), _p(w), B, n, D, C.c_double(slope), int(bool(norm)), C.c_double(norm_eps), _p(u))
    if rc:
        raise ValueError("orc_scores: %d" % rc)
    return u

