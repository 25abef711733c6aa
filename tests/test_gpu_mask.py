"""GPU parity of stages 1+2 (sparsek_mask, sparsek_materialize) against the CPU oracle.

Bars: lifetimes and index sets bit-exact; thresholds and masks within 1e-5 (relative to
max(1,|ref|); masks live in [0,1]).
"""
import numpy as np
import pytest
import torch

import paper_2406_16747_amd as spk
from paper_2406_16747_amd import synth
from gpu_util import dev, host, require_gpu, say

pytestmark = pytest.mark.gpu


def scores(kind, rng, rows, n):
    if kind == "normal":
        return rng.standard_normal((rows, n), dtype=np.float32)
    if kind == "ties":  # coarse grid: many exact ties
        return (np.round(rng.standard_normal((rows, n)) * 4) / 4).astype(np.float32)
    if kind == "equal":
        return np.full((rows, n), 0.5, np.float32)
    if kind == "rising":  # every newcomer enters the top-k
        return (np.arange(n, dtype=np.float32)[None] * 0.01 + rng.standard_normal((rows, 1), dtype=np.float32))
    if kind == "falling":
        return (-np.arange(n, dtype=np.float32)[None] * 0.01).repeat(rows, 0)
    if kind == "wide":  # gaps mostly above 1: hard top-k, flat tau
        return (rng.standard_normal((rows, n)) * 50).astype(np.float32)
    if kind == "drift":
        pos = np.arange(n, dtype=np.float32)
        return (rng.standard_normal((rows, n), dtype=np.float32) + 0.5 * np.sin(pos / 256)).astype(np.float32)
    raise ValueError(kind)


def check_rows(oracle, u, k, sample_t=None):
    rows, n = u.shape
    ud = dev(u.reshape(rows, 1, n))
    ws = spk.sparsek_mask_workspace(ud, k)
    ws.fill_(0xFF)  # the call itself must clear its status word
    tau_g, death_g = spk.sparsek_mask(ud, k, ws=ws)
    assert spk.sparsek_mask_status(ud, k, ws) == 0  # every threshold solve converged
    tau_g, death_g = host(tau_g).reshape(rows, n), host(death_g).reshape(rows, n)
    for r in range(rows):
        tau_r, us, ws = oracle.tau_prefixes(u[r], k)
        death_r = oracle.death(u[r], k)
        np.testing.assert_array_equal(death_g[r], death_r)
        err = np.abs(tau_g[r].astype(np.float64) - tau_r) / np.maximum(1.0, np.abs(tau_r))
        assert err.max() <= 1e-5, (r, int(err.argmax()), err.max())
    # explicit lists + gates on sampled prefixes
    ts = sample_t if sample_t is not None else sorted(set([0, min(n - 1, max(k - 1, 0)), min(n - 1, k), n // 2, n - 1]))
    for t in ts:
        idx, gate = spk.sparsek_materialize(ud, dev(tau_g.reshape(rows, 1, n)), dev(death_g.reshape(rows, 1, n)),
                                            k, t, t + 1)
        idx, gate = host(idx).reshape(rows, -1), host(gate).reshape(rows, -1)
        for r in range(rows):
            want = oracle.select_prefix(u[r], t, k)
            got = idx[r][idx[r] >= 0]
            np.testing.assert_array_equal(got, want)
            assert np.all(idx[r][len(want):] == -1)
            tau_t, p, _, _ = oracle.sparsek(u[r, : t + 1], k)
            np.testing.assert_allclose(gate[r][: len(want)], p[want], atol=1e-5, rtol=0)
    return tau_g, death_g


@pytest.mark.parametrize("kind", ["normal", "ties", "equal", "rising", "falling", "wide", "drift"])
@pytest.mark.parametrize("n,k", [(1, 1), (5, 2), (130, 7), (1000, 64), (1024, 64), (2500, 300), (4500, 64)])
def test_mask_small(oracle, kind, n, k):
    require_gpu()
    say("mask", kind, n, k)
    rng = np.random.default_rng(n * 1000 + k)
    check_rows(oracle, scores(kind, rng, 3, n), k)


@pytest.mark.parametrize("n,k", [(300, 0), (300, 300), (300, 299), (300, 1000), (2049, 2048), (2300, 1)])
def test_mask_degenerate_k(oracle, n, k):
    require_gpu()
    say("mask degenerate", n, k)
    rng = np.random.default_rng(n + k)
    check_rows(oracle, scores("normal", rng, 2, n), k)


def test_mask_config1(oracle):
    require_gpu()
    inp = synth.make(1)
    say("mask config 1")
    check_rows(oracle, inp["u"].reshape(1, -1), inp["k"], sample_t=[63, 64, 100, 500, 1023])


def test_mask_candidate_overflow_fallback(oracle):
    """More scores above the threshold than the LDS list holds: the kernel must switch to
    its global-memory path and still be exact."""
    require_gpu()
    say("mask overflow")
    rng = np.random.default_rng(77)
    n, k = 12000, 5000
    u = (rng.standard_normal((1, n)) * 0.05).astype(np.float32)  # w* ~ n: everything is fractional
    check_rows(oracle, u, k, sample_t=[4999, 5000, 9000, n - 1])


def test_mask_is_deterministic(oracle):
    require_gpu()
    rng = np.random.default_rng(5)
    u = dev(rng.standard_normal((4, 1, 6000), dtype=np.float32))
    a = spk.sparsek_mask(u, 200)
    b = spk.sparsek_mask(u, 200)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_many_rows_take_the_two_stage_path_and_hand_on_what_does_not_fit(oracle):
    """With many score rows the chunks first go to the half-capacity kernel, which hands the chunks whose candidates
    do not fit its lists on to the full-capacity kernel: rows of unit-variance scores stay in the first stage, rows of
    narrow scores (nearly every score in the support of the threshold) are handed on.  Both kinds must match the
    oracle, and the call must clear the hand-on bits itself (the workspace starts as garbage)."""
    require_gpu()
    rng = np.random.default_rng(11)
    rows, n, k = 20, 16384, 300   # 20 x 128 chunks >= 2048
    u = rng.standard_normal((rows, n)).astype(np.float32)
    u[3] *= 0.02
    u[17] = (np.round(u[17] * 2) / 2).astype(np.float32) * 0.1   # narrow and full of ties
    ud = dev(u.reshape(1, rows, n))
    ws = spk.sparsek_mask_workspace(ud, k)
    for fill in (0xFF, 0x00):
        ws.fill_(fill)
        tau_g, death_g = spk.sparsek_mask(ud, k, ws=ws)
        assert spk.sparsek_mask_status(ud, k, ws) == 0
        tau_g, death_g = host(tau_g).reshape(rows, n), host(death_g).reshape(rows, n)
        for r in (0, 3, 17):
            say("  two-stage mask, row", r)
            tau_r = oracle.tau_incremental(u[r], k)   # pinned against the sort-based routine in the CPU tests
            np.testing.assert_array_equal(death_g[r], oracle.death(u[r], k))
            err = np.abs(tau_g[r].astype(np.float64) - tau_r) / np.maximum(1.0, np.abs(tau_r))
            assert err.max() <= 1e-5, (r, err.max())
