"""Pins of the oracle's score pipeline (scoring network + position slope + timestep normalisation).

Against library routines (numpy matmul in fp64; pandas' expanding mean / population variance),
a closed form for a constant hidden state, and the invariances the normalisation must have.
"""
import numpy as np
import pandas as pd
import pytest


def test_raw_scores_are_the_projection_plus_slope(oracle):
    rng = np.random.default_rng(5)
    B, n, D = 3, 37, 19
    X = rng.standard_normal((B, n, D)).astype(np.float32)
    w = rng.standard_normal(D).astype(np.float32)
    u = oracle.scores(X, w, slope=0.125)
    ref = X.astype(np.float64) @ w.astype(np.float64) + 0.125 * np.arange(n)
    np.testing.assert_allclose(u, ref, rtol=1e-13, atol=1e-13)
    # the slope is what separates two identical tokens at different positions
    X[:, 5] = X[:, 20]
    u = oracle.scores(X, w, slope=0.125)
    np.testing.assert_allclose(u[:, 20] - u[:, 5], 15 * 0.125, rtol=1e-12)


@pytest.mark.parametrize("eps", [0.0, 1e-5, 0.3])
def test_timestep_norm_against_expanding_statistics(oracle, eps):
    rng = np.random.default_rng(6)
    B, n, D = 2, 200, 8
    X = rng.standard_normal((B, n, D)).astype(np.float32)
    w = rng.standard_normal(D).astype(np.float32)
    raw = oracle.scores(X, w, slope=0.01)
    u = oracle.scores(X, w, slope=0.01, norm=True, norm_eps=eps)
    for b in range(B):
        s = pd.Series(raw[b])
        mean = s.expanding().mean().to_numpy()
        var = s.expanding().var(ddof=0).to_numpy()
        with np.errstate(invalid="ignore"):  # first timestep with eps = 0 is 0/0 on both sides
            ref = (raw[b] - mean) / np.sqrt(var + eps)
        np.testing.assert_allclose(u[b, 1:], ref[1:], rtol=1e-9, atol=1e-11)
        if eps > 0:
            assert u[b, 0] == 0.0  # first timestep: mean = itself, variance 0


def test_constant_hidden_state_closed_form(oracle):
    """X_t = x for all t: raw_t = a + t*slope, an arithmetic progression, whose running mean is
    a + slope*t/2 and running population variance slope^2 ((t+1)^2 - 1)/12."""
    D, n, slope = 6, 64, 0.25
    x = np.arange(1, D + 1, dtype=np.float32) / 8
    w = np.ones(D, np.float32) / 4
    X = np.broadcast_to(x, (1, n, D)).copy()
    u = oracle.scores(X, w, slope=slope, norm=True, norm_eps=0.0)
    t = np.arange(1, n)
    ref = (slope * t / 2) / np.sqrt(slope ** 2 * ((t + 1.0) ** 2 - 1) / 12)
    np.testing.assert_allclose(u[0, 1:], ref, rtol=1e-12)


def test_normalisation_invariances(oracle):
    rng = np.random.default_rng(7)
    n, D = 150, 5
    X = rng.standard_normal((1, n, D)).astype(np.float32)
    w = rng.standard_normal(D).astype(np.float32)
    base = oracle.scores(X, w, norm=True, norm_eps=0.0)
    # scaling the scorer by a power of two scales every raw score exactly: same normalised scores
    np.testing.assert_allclose(oracle.scores(X, 4 * w, norm=True, norm_eps=0.0)[0, 1:], base[0, 1:], rtol=1e-10)
    # a prefix is normalised on its own: truncating the sequence does not change earlier outputs
    np.testing.assert_array_equal(oracle.scores(X[:, :60], w, norm=True, norm_eps=0.0), base[:, :60])
    # at every timestep the normalised history has zero mean and unit variance *under that step's
    # statistics*: check the last one from the raw scores
    raw = oracle.scores(X, w)[0]
    z = (raw - raw.mean()) / raw.std()
    assert base[0, -1] == pytest.approx(z[-1], rel=1e-12)
    # sequences of a batch are independent
    X2 = np.concatenate([X, X[:, ::-1]], 0)
    np.testing.assert_array_equal(oracle.scores(X2, w, norm=True)[0], oracle.scores(X, w, norm=True)[0])
