"""Pins of the oracle's gated attention, decode-by-definition and score gradient.

Checks against a hand-worked query, library dense / banded attention (torch SDPA on
CPU) in the two limits the method reduces to, closed forms for degenerate inputs, the
from-scratch per-query routine, and finite differences of the forward for the gradient.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def sdpa(q, k, v, mask, scale):
    """Library attention on CPU in fp64 with an explicit boolean mask [n,n]."""
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double()[None], torch.from_numpy(k).double()[None],
        torch.from_numpy(v).double()[None], attn_mask=torch.from_numpy(mask)[None], scale=scale,
    )
    return out[0].numpy()


def rand_head(rng, n, d, spread=1.0):
    q = (rng.standard_normal((n, d)) * spread).astype(np.float32)
    k = (rng.standard_normal((n, d)) * spread).astype(np.float32)
    v = rng.standard_normal((n, d)).astype(np.float32)
    u = rng.standard_normal(n).astype(np.float32)
    return q, k, v, u


def full(oracle, q, k, v, u, kk, w, mode, scale):
    tau = oracle.tau_prefixes(u, kk)[0]
    dth = oracle.death(u, kk)
    return oracle.attn_rows(q, k, v, u, tau, dth, kk, w, mode, scale, 0, len(u))


def test_hand_worked_query(oracle):
    g = json.load(open(os.path.join(GOLD, "attention_worked_example.json")))
    env = {"log": math.log, "sqrt": math.sqrt}
    u = np.array(g["u"], np.float32)
    q = np.array(g["q"], np.float32)[:, None]
    k = np.array([eval(e, env) for e in g["keys_expr"]], np.float32)[:, None]
    v = np.array(g["v"], np.float32)[:, None]
    i = g["query"]
    # keys are rounded to fp32 when stored; tolerance covers that rounding only
    for mode in (0, 1, 2):
        o, lse = oracle.attn_query_bydef(q, k, v, u, g["k"], g["w"], mode, 1.0, i)
        assert o[0] == pytest.approx(eval(g["mode%d_o_expr" % mode], env), rel=2e-6)
        if "mode%d_lse_expr" % mode in g:
            assert lse == pytest.approx(eval(g["mode%d_lse_expr" % mode], env), rel=2e-6)
        o2, lse2 = full(oracle, q, k, v, u, g["k"], g["w"], mode, 1.0)
        assert o2[i, 0] == pytest.approx(o[0], rel=1e-12)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_k_ge_n_is_dense_causal(oracle, mode):
    rng = np.random.default_rng(1)
    n, d = 96, 16
    q, k, v, u = rand_head(rng, n, d)
    causal = np.tril(np.ones((n, n), bool))
    for kk, w in [(n, 8), (n + 5, 1), (n, 0)]:
        o, lse = full(oracle, q, k, v, u, kk, w, mode, 0.25)
        np.testing.assert_allclose(o, sdpa(q, k, v, causal, 0.25), atol=1e-12)
        s = 0.25 * q.astype(np.float64) @ k.astype(np.float64).T
        s[~causal] = -np.inf
        np.testing.assert_allclose(lse, np.log(np.exp(s).sum(1)), atol=1e-12)


def test_k0_is_sliding_window(oracle):
    rng = np.random.default_rng(2)
    n, d, w = 80, 8, 11
    q, k, v, u = rand_head(rng, n, d)
    i, j = np.indices((n, n))
    band = (j <= i) & (i - j < w)
    o, _ = full(oracle, q, k, v, u, 0, w, 0, 0.5)
    np.testing.assert_allclose(o, sdpa(q, k, v, band, 0.5), atol=1e-12)


def test_early_rows_are_dense_and_modes_agree_on_unit_gates(oracle):
    rng = np.random.default_rng(3)
    n, d, kk, w = 120, 8, 10, 7
    q, k, v, u = rand_head(rng, n, d)
    causal = np.tril(np.ones((n, n), bool))
    dense = sdpa(q, k, v, causal, 1.0)
    for mode in (0, 1):
        o, _ = full(oracle, q, k, v, u, kk, w, mode, 1.0)
        np.testing.assert_allclose(o[: kk + w], dense[: kk + w], atol=1e-12)
        assert np.abs(o[kk + w + 5:] - dense[kk + w + 5:]).max() > 1e-3
    # well separated scores: every selected gate is exactly 1, so all modes coincide
    u_sep = (rng.permutation(n) * 1.5).astype(np.float32)
    outs = [full(oracle, q, k, v, u_sep, kk, w, m, 1.0)[0] for m in (0, 1, 2)]
    np.testing.assert_allclose(outs[0], outs[1], atol=1e-12)
    np.testing.assert_allclose(outs[0], outs[2], atol=1e-12)
    # and they are the hard top-k + window attention
    i, j = np.indices((n, n))
    mask = (j <= i) & (i - j < w)
    for qi in range(w, n):
        mask[qi, oracle.select_prefix(u_sep, qi - w, kk)] = True
    np.testing.assert_allclose(outs[2], sdpa(q, k, v, mask, 1.0), atol=1e-12)


def test_closed_forms_for_zero_query_and_unit_values(oracle):
    rng = np.random.default_rng(4)
    n, d, kk, w = 70, 4, 6, 5
    q, k, v, u = rand_head(rng, n, d)
    tau = oracle.tau_prefixes(u, kk)[0]
    for qi in (w + kk + 3, n - 1):
        T = qi - w
        sel = oracle.select_prefix(u, T, kk)
        m = np.clip(u[sel].astype(np.float64) - tau[T], 0, 1)
        win = np.arange(qi - w + 1, qi + 1)
        # q = 0: uniform softmax over the k+w keys, values carry the gate (modes 0 and 1)
        o, lse = oracle.attn_query_bydef(np.zeros_like(q), k, v, u, kk, w, 0, 1.0, qi)
        want = ((m[:, None] * v[sel]).sum(0) + v[win].sum(0)) / (len(sel) + w)
        np.testing.assert_allclose(o, want, atol=1e-12)
        assert lse == pytest.approx(math.log(len(sel) + w))
        # v = 1, mode 1: o = sum_j p_ij m_ij with ungated logits
        s = np.concatenate([k[sel], k[win]]).astype(np.float64) @ q[qi].astype(np.float64)
        p = np.exp(s - s.max())
        p /= p.sum()
        o, _ = oracle.attn_query_bydef(q, k, np.ones_like(v), u, kk, w, 1, 1.0, qi)
        np.testing.assert_allclose(o, (p * np.concatenate([m, np.ones(w)])).sum(), atol=1e-12)
        # mode 0: the logits of the selected keys are scaled by their gates
        s0 = s * np.concatenate([m, np.ones(w)])
        p0 = np.exp(s0 - s0.max())
        p0 /= p0.sum()
        o, _ = oracle.attn_query_bydef(q, k, np.ones_like(v), u, kk, w, 0, 1.0, qi)
        np.testing.assert_allclose(o, (p0 * np.concatenate([m, np.ones(w)])).sum(), atol=1e-12)


@pytest.mark.parametrize("kk,w", [(5, 4), (7, 0), (3, 9), (0, 6)])
def test_whole_sequence_routine_equals_per_query_definition(oracle, kk, w):
    rng = np.random.default_rng(5)
    n, d = 64, 8
    q, k, v, u = rand_head(rng, n, d)
    u[20] = u[3]
    for mode in (0, 1, 2):
        o, lse = full(oracle, q, k, v, u, kk, w, mode, 0.7)
        for qi in range(n):
            o1, l1 = oracle.attn_query_bydef(q, k, v, u, kk, w, mode, 0.7, qi)
            np.testing.assert_allclose(o[qi], o1, atol=1e-13)
            assert lse[qi] == pytest.approx(l1, abs=1e-12)


def test_batched_entry_and_groups(oracle):
    rng = np.random.default_rng(6)
    B, H, n, d, kk, w = 2, 3, 40, 8, 4, 3
    q = rng.standard_normal((B, H, n, d)).astype(np.float32)
    k = rng.standard_normal((B, H, n, d)).astype(np.float32)
    v = rng.standard_normal((B, H, n, d)).astype(np.float32)
    for Gu in (1, H):
        u = rng.standard_normal((B, Gu, n)).astype(np.float32)
        tau, dth = oracle.mask_all(u, kk)
        o, lse, used = oracle.attn_fwd(q, k, v, u, tau, dth, kk, w, 0, 1.0, nthreads=2)
        assert used == 2
        for b in range(B):
            for h in range(H):
                g = 0 if Gu == 1 else h
                o1, l1 = full(oracle, q[b, h], k[b, h], v[b, h], u[b, g], kk, w, 0, 1.0)
                np.testing.assert_array_equal(o[b, h], o1)
                np.testing.assert_array_equal(lse[b, h], l1)


def test_decode_by_definition_is_the_prefill_row(oracle):
    rng = np.random.default_rng(7)
    n_ctx, steps, d, kk, w = 50, 9, 8, 6, 5
    n = n_ctx + steps
    q, k, v, u = rand_head(rng, n, d)
    o_full, _ = full(oracle, q, k, v, u, kk, w, 0, 1.0)
    o_dec = oracle.decode_bydef(q[n_ctx:], k, v, u, n_ctx, kk, w, 0, 1.0)
    np.testing.assert_array_equal(o_dec, o_full[n_ctx:])
    # the future does not leak: truncating the history after step s leaves step s unchanged
    s = 4
    o_trunc = oracle.decode_bydef(q[n_ctx:n_ctx + s + 1], k[: n_ctx + s + 1], v[: n_ctx + s + 1],
                                  u[: n_ctx + s + 1], n_ctx, kk, w, 0, 1.0)
    np.testing.assert_allclose(o_trunc[s], o_dec[s], atol=1e-14)


# ---------------------------------------------------------------- gradient w.r.t. u


def grid_scores(rng, n):
    """Distinct scores on a 1/16 grid, so that +-2^-10 steps are exact in fp32 and move
    no score across another score."""
    vals = rng.choice(np.arange(-40, 41), size=n, replace=False) / 16.0
    return vals.astype(np.float32)


@pytest.mark.parametrize("mode", [0, 1])
def test_du_matches_finite_differences(oracle, mode):
    rng = np.random.default_rng(12 + mode)
    B, H, n, d, kk, w = 1, 2, 28, 4, 5, 3
    h = 2.0 ** -10
    q = rng.standard_normal((B, H, n, d)).astype(np.float32)
    k = rng.standard_normal((B, H, n, d)).astype(np.float32)
    v = rng.standard_normal((B, H, n, d)).astype(np.float32)
    dO = rng.standard_normal((B, H, n, d)).astype(np.float32)
    u = grid_scores(rng, n).reshape(1, 1, n) + np.float32(1.0 / 64)
    tau, dth = oracle.mask_all(u, kk)
    du, _ = oracle.mask_bwd(q, k, v, u, tau, dth, dO, kk, w, mode, 0.6, nthreads=1)

    def loss(uu):
        t, dd = oracle.mask_all(uu, kk)
        np.testing.assert_array_equal(dd, dth)  # the hard set is held fixed
        o, _, _ = oracle.attn_fwd(q, k, v, uu, t, dd, kk, w, mode, 0.6, nthreads=1)
        return float((o * dO).sum())

    # coordinates whose +-h move crosses a kink of some prefix (u_j = tau_T or tau_T + 1) are skipped
    checked = 0
    for j in range(n):
        near = False
        for T in range(j, n):
            for edge in (tau[0, 0, T], tau[0, 0, T] + 1):
                if np.any(np.abs(u[0, 0, : T + 1].astype(np.float64) - edge) < 4 * h):
                    near = True
        if near:
            continue
        up, um = u.copy(), u.copy()
        up[0, 0, j] += np.float32(h)
        um[0, 0, j] -= np.float32(h)
        fd = (loss(up) - loss(um)) / (2 * h)
        assert du[0, 0, j] == pytest.approx(fd, abs=2e-5, rel=2e-4), j
        checked += 1
    assert checked >= 5
    assert abs(du.sum()) < 1e-10  # rows of the SPARSEK Jacobian sum to zero (App. A.3)


def _forward_with_gate_matrix(q, k, v, G, att, scale):
    """o_i = sum_j softmax_j(scale * G_ij q_i.k_j) G_ij v_j over the attended pairs att[i, j]
    (gates on keys and values), written out with numpy for one head."""
    n = q.shape[0]
    o = np.zeros((n, q.shape[1]))
    for i in range(n):
        js = np.nonzero(att[i])[0]
        s = scale * G[i, js] * (k[js].astype(np.float64) @ q[i].astype(np.float64))
        p = np.exp(s - s.max())
        p /= p.sum()
        o[i] = (p * G[i, js]) @ v[js].astype(np.float64)
    return o


def test_straight_through_du_matches_finite_differences(oracle):
    """Mode 3 (Sec. 3.4): the gates that enter the forward are m_soft(u) - m_soft(u0) + m_hard, so
    the forward value at u0 is the hard selection and the gradient is dL/dm at m = 1 pushed
    through the soft mask.  Checked against central differences of that forward, written out
    here with an explicit gate matrix (which is first checked against the oracle's own forward
    for soft gates, mode 0, and for unit gates, mode 2 = mode 3)."""
    rng = np.random.default_rng(15)
    n, d, kk, w = 28, 4, 5, 3
    h = 2.0 ** -10
    scale = 0.6
    q = rng.standard_normal((1, 1, n, d)).astype(np.float32)
    k = rng.standard_normal((1, 1, n, d)).astype(np.float32)
    v = rng.standard_normal((1, 1, n, d)).astype(np.float32)
    dO = rng.standard_normal((1, 1, n, d)).astype(np.float32)
    u0 = grid_scores(rng, n).reshape(1, 1, n) + np.float32(1.0 / 64)
    tau0, dth = oracle.mask_all(u0, kk)

    def attended_and_soft_gates(uu):
        t, dd = oracle.mask_all(uu, kk)
        np.testing.assert_array_equal(dd, dth)  # the hard set is held fixed
        att = np.zeros((n, n), bool)
        M = np.ones((n, n))
        for i in range(n):
            for j in range(i + 1):
                if i - j < w:
                    att[i, j] = True  # window, gate 1
                elif j <= i - w < dth[0, 0, j]:
                    att[i, j] = True
                    M[i, j] = min(max(float(uu[0, 0, j]) - t[0, 0, i - w], 0.0), 1.0)
        return att, M

    att, M0 = attended_and_soft_gates(u0)
    o_soft, _, _ = oracle.attn_fwd(q, k, v, u0, tau0, dth, kk, w, 0, scale, nthreads=1)
    np.testing.assert_allclose(_forward_with_gate_matrix(q[0, 0], k[0, 0], v[0, 0], M0, att, scale), o_soft[0, 0],
                               rtol=1e-12, atol=1e-12)
    for mode in (2, 3):
        o_hard, _, _ = oracle.attn_fwd(q, k, v, u0, tau0, dth, kk, w, mode, scale, nthreads=1)
        np.testing.assert_allclose(_forward_with_gate_matrix(q[0, 0], k[0, 0], v[0, 0], np.ones((n, n)), att, scale),
                                   o_hard[0, 0], rtol=1e-12, atol=1e-12)

    def loss(uu):
        _, M = attended_and_soft_gates(uu)
        o = _forward_with_gate_matrix(q[0, 0], k[0, 0], v[0, 0], M - M0 + 1.0, att, scale)
        return float((o * dO[0, 0]).sum())

    du, _ = oracle.mask_bwd(q, k, v, u0, tau0, dth, dO, kk, w, 3, scale, nthreads=1)
    du_soft, _ = oracle.mask_bwd(q, k, v, u0, tau0, dth, dO, kk, w, 0, scale, nthreads=1)
    assert np.abs(du - du_soft).max() > 1e-3  # not the soft-gate gradient
    checked = 0
    for j in range(n):
        near = False
        for T in range(j, n):
            for edge in (tau0[0, 0, T], tau0[0, 0, T] + 1):
                if np.any(np.abs(u0[0, 0, : T + 1].astype(np.float64) - edge) < 4 * h):
                    near = True
        if near:
            continue
        up, um = u0.copy(), u0.copy()
        up[0, 0, j] += np.float32(h)
        um[0, 0, j] -= np.float32(h)
        fd = (loss(up) - loss(um)) / (2 * h)
        assert du[0, 0, j] == pytest.approx(fd, abs=2e-5, rel=2e-4), j
        checked += 1
    assert checked >= 5
    assert abs(du.sum()) < 1e-10


def test_du_zero_without_fractional_gates_and_in_mode2(oracle):
    rng = np.random.default_rng(14)
    B, H, n, d, kk, w = 1, 1, 30, 4, 4, 2
    q = rng.standard_normal((B, H, n, d)).astype(np.float32)
    k = rng.standard_normal((B, H, n, d)).astype(np.float32)
    v = rng.standard_normal((B, H, n, d)).astype(np.float32)
    dO = rng.standard_normal((B, H, n, d)).astype(np.float32)
    u = (rng.permutation(n) * 1.5).astype(np.float32).reshape(1, 1, n)  # gaps >= 1: S* empty
    tau, dth = oracle.mask_all(u, kk)
    du, _ = oracle.mask_bwd(q, k, v, u, tau, dth, dO, kk, w, 0, 1.0)
    assert not du.any()
    u = rng.standard_normal((1, 1, n)).astype(np.float32)
    tau, dth = oracle.mask_all(u, kk)
    du, _ = oracle.mask_bwd(q, k, v, u, tau, dth, dO, kk, w, 2, 1.0)
    assert not du.any()
    du, _ = oracle.mask_bwd(q, k, v, u, tau, dth, dO, kk, w, 0, 1.0)
    assert du.any()
    # a key that is never strictly fractional in any prefix it belongs to gets no gradient
    for j in range(n):
        frac = any(tau[0, 0, T] < u[0, 0, j] < tau[0, 0, T] + 1 for T in range(j, n - w))
        if not frac:
            assert du[0, 0, j] == 0


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_qkv_gradients_match_finite_differences(oracle, mode):
    """dQ, dK, dV against central differences of the oracle's own forward (the scores, hence the
    gates, are held fixed)."""
    rng = np.random.default_rng(40 + mode)
    B, H, n, d, kk, w = 1, 2, 14, 3, 4, 3
    h = 2.0 ** -12
    q, k, v, dO = (rng.standard_normal((B, H, n, d)).astype(np.float32) for _ in range(4))
    u = rng.standard_normal((1, 1, n)).astype(np.float32)
    tau, dth = oracle.mask_all(u, kk)
    dQ, dK, dV = oracle.attn_bwd(q, k, v, u, tau, dth, dO, kk, w, mode, 0.7, nthreads=1)

    def loss(qq, kx, vx):
        o, _, _ = oracle.attn_fwd(qq, kx, vx, u, tau, dth, kk, w, mode, 0.7, nthreads=1)
        return float((o * dO).sum())

    for which, grad in (("q", dQ), ("k", dK), ("v", dV)):
        for idx in [(0, 0, 0, 0), (0, 1, 5, 2), (0, 0, 9, 1), (0, 1, 13, 0), (0, 0, 3, 2)]:
            args = {"q": q, "k": k, "v": v}
            xp, xm = args[which].copy(), args[which].copy()
            xp[idx] += np.float32(h)
            xm[idx] -= np.float32(h)
            ap, am = dict(args), dict(args)
            ap[which], am[which] = xp, xm
            fd = (loss(ap["q"], ap["k"], ap["v"]) - loss(am["q"], am["k"], am["v"])) / (2 * h)
            assert grad[idx] == pytest.approx(fd, abs=5e-6, rel=5e-5), (which, idx)


def test_qkv_gradients_dense_limit_against_autograd(oracle):
    """k >= n: plain causal attention, whose gradients torch's autograd gives (fp64, CPU)."""
    rng = np.random.default_rng(44)
    n, d = 24, 5
    q, k, v, dO = (rng.standard_normal((1, 1, n, d)).astype(np.float32) for _ in range(4))
    u = rng.standard_normal((1, 1, n)).astype(np.float32)
    tau, dth = oracle.mask_all(u, n + 3)
    dQ, dK, dV = oracle.attn_bwd(q, k, v, u, tau, dth, dO, n + 3, 4, 0, 0.5)
    tq, tk, tv = (torch.from_numpy(x[0, 0]).double().requires_grad_(True) for x in (q, k, v))
    mask = torch.tril(torch.ones(n, n, dtype=torch.bool))
    o = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None], attn_mask=mask[None], scale=0.5)
    (o[0] * torch.from_numpy(dO[0, 0]).double()).sum().backward()
    np.testing.assert_allclose(dQ[0, 0], tq.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dK[0, 0], tk.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dV[0, 0], tv.grad.numpy(), rtol=1e-9, atol=1e-11)



@pytest.mark.parametrize("k,w,mode", [(20, 10, 0), (5, 0, 1), (0, 8, 2), (600, 3, 0), (16, 16, 3), (1, 1, 0)])
def test_incremental_decode_equals_decode_by_definition(oracle, k, w, mode):
    """The constant-work decode loop (incremental threshold, heap of the k selected keys, attention over k + w
    keys) against the definition: row t of the attention over the whole history.  Scores on a coarse grid, so the
    tie rule of the selection (an equal newcomer does not evict) is exercised."""
    rng = np.random.default_rng(100 * k + w)
    n_ctx, steps, d = 500, 40, 16
    n = n_ctx + steps
    K, V = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(2))
    u = (np.round(rng.standard_normal(n) * 3) / 3).astype(np.float32)
    q = rng.standard_normal((steps, d)).astype(np.float32)
    want = oracle.decode_bydef(q, K, V, u, n_ctx, k, w, mode, 0.3)
    got, _ = oracle.decode_incremental(q, K, V, u, n_ctx, k, w, mode, 0.3)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-10)
    # from an empty context as well
    want = oracle.decode_bydef(q, K[:steps], V[:steps], u[:steps], 0, k, w, mode, 0.3)
    got, _ = oracle.decode_incremental(q, K[:steps], V[:steps], u[:steps], 0, k, w, mode, 0.3)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-10)
