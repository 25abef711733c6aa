"""Pins of the oracle's SPARSEK operator and hard top-k selection.

None of these re-type the oracle's algorithm: they check it against hand-worked closed
forms, the optimality (KKT) certificate of App. A.1 (sufficient and unique for this
convex problem), a bisection on the monotone constraint function, a generic constrained
solver applied to the definition, the textbook SparseMax formula (k=1), symmetries of
the projection, and numpy's stable sort for the selection.
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import optimize, stats

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def f_of(z, tau):
    return float(np.clip(z.astype(np.float64) - tau, 0.0, 1.0).sum())


def certify(z, k, tau, p, us, ws):
    """KKT certificate (App. A.1): p = clip(z - tau), box and sum constraints, and the
    order conditions z_(u*) >= tau+1 > z_(u*+1), z_(w*) > tau >= z_(w*+1)."""
    z64 = z.astype(np.float64)
    m = len(z)
    keff = min(k, m)
    assert np.all(p >= 0) and np.all(p <= 1)
    np.testing.assert_allclose(p, np.clip(z64 - tau, 0, 1), atol=1e-15)
    assert abs(p.sum() - keff) <= 1e-9 * max(1, keff)
    zs = np.sort(z64)[::-1]
    assert us == int((zs >= tau + 1).sum()) and ws == int((zs > tau).sum())
    if us > 0:
        assert zs[us - 1] >= tau + 1
    if us < m:
        assert zs[us] < tau + 1
    if ws > 0:
        assert zs[ws - 1] > tau
    if ws < m:
        assert zs[ws] <= tau


def test_worked_examples(oracle):
    cases = json.load(open(os.path.join(GOLD, "sparsek_worked_examples.json")))["cases"]
    for c in cases:
        z = np.array(c["z"], np.float32)
        tau, p, us, ws = oracle.sparsek(z, c["k"])
        assert tau == pytest.approx(float(Fraction(*c["tau"])), abs=1e-7), c["why"]
        want = [float(Fraction(*f)) for f in c["p"]]
        np.testing.assert_allclose(p, want, atol=1e-7, err_msg=c["why"])
        assert (us, ws) == (c["ustar"], c["wstar"]), c["why"]
        sel = oracle.select_prefix(z, len(z) - 1, c["k"])
        assert sel.tolist() == c["top_k"], c["why"]


@pytest.mark.parametrize("seed", range(6))
def test_kkt_certificate_and_bisection(oracle, seed):
    rng = np.random.default_rng(seed)
    for m, k in [(1, 1), (5, 2), (37, 7), (200, 64), (1000, 64), (513, 512), (64, 64), (50, 80)]:
        z = (rng.standard_normal(m) * rng.choice([0.3, 1.0, 4.0])).astype(np.float32)
        tau, p, us, ws = oracle.sparsek(z, k)
        certify(z, k, tau, p, us, ws)
        if ws > us and m > k:  # unique root: bisection on the monotone f must agree
            lo, hi = float(z.min()) - 1.0, float(z.max())
            for _ in range(200):
                mid = 0.5 * (lo + hi)
                if f_of(z, mid) >= k:
                    lo = mid
                else:
                    hi = mid
            assert abs(lo - tau) < 1e-10


def test_matches_generic_solver_on_the_definition(oracle):
    """argmin ||p - z||^2 over {0<=p<=1, sum p = k} (Sec. 3.3 definition) by SLSQP."""
    rng = np.random.default_rng(11)
    for m, k in [(4, 2), (6, 1), (7, 3), (9, 5)]:
        z = rng.standard_normal(m).astype(np.float32)
        _, p, _, _ = oracle.sparsek(z, k)
        z64 = z.astype(np.float64)
        res = optimize.minimize(
            lambda x: 0.5 * np.sum((x - z64) ** 2), np.full(m, k / m), jac=lambda x: x - z64,
            bounds=[(0, 1)] * m, constraints=[{"type": "eq", "fun": lambda x: x.sum() - k,
                                               "jac": lambda x: np.ones(m)}],
            method="SLSQP", options={"ftol": 1e-14, "maxiter": 500},
        )
        assert res.success
        np.testing.assert_allclose(p, res.x, atol=2e-6)


def test_k1_is_sparsemax(oracle):
    """k=1 reduces to SparseMax (Sec. 3.1): tau = (sum_{j<=rho} z_(j) - 1)/rho with
    rho = max{j : 1 + j z_(j) > sum_{i<=j} z_(i)} (Martins & Astudillo's sort formula)."""
    rng = np.random.default_rng(5)
    for m in (2, 3, 10, 100, 777):
        z = rng.standard_normal(m).astype(np.float32)
        zs = np.sort(z.astype(np.float64))[::-1]
        cs = np.cumsum(zs)
        j = np.arange(1, m + 1)
        rho = j[1 + j * zs > cs].max()
        tau_ref = (cs[rho - 1] - 1) / rho
        tau, p, _, ws = oracle.sparsek(z, 1)
        assert tau == pytest.approx(tau_ref, abs=1e-12)
        assert ws == rho
        np.testing.assert_allclose(p, np.maximum(z.astype(np.float64) - tau_ref, 0), atol=1e-12)


def test_all_equal_shift_and_complement(oracle):
    rng = np.random.default_rng(3)
    z = np.full(16, 0.75, np.float32)
    tau, p, _, _ = oracle.sparsek(z, 5)
    assert tau == pytest.approx(0.75 - 5 / 16, abs=1e-12)
    np.testing.assert_allclose(p, 5 / 16, atol=1e-12)
    # shift: values on a dyadic grid so that z + c is exact in fp32
    z = (np.round(rng.standard_normal(300) * 256) / 256).astype(np.float32)
    t0, p0, _, _ = oracle.sparsek(z, 40)
    t1, p1, _, _ = oracle.sparsek(z + np.float32(2.5), 40)
    assert t1 == pytest.approx(t0 + 2.5, abs=1e-12)
    np.testing.assert_allclose(p1, p0, atol=1e-12)
    # complement: projecting -z with budget m-k gives 1 - p
    _, pc, _, _ = oracle.sparsek(-z, 300 - 40)
    np.testing.assert_allclose(pc, 1 - p0, atol=1e-9)


def test_well_separated_scores_give_hard_topk(oracle):
    rng = np.random.default_rng(8)
    m, k = 60, 9
    z = (rng.permutation(m) * 1.25 - 20).astype(np.float32)  # all gaps >= 1
    tau, p, us, ws = oracle.sparsek(z, k)
    want = np.zeros(m)
    want[np.argsort(-z)[:k]] = 1
    np.testing.assert_array_equal(p, want)
    assert us == ws == k
    assert tau == pytest.approx(np.sort(z)[::-1][k - 1] - 1.0)  # sup rule: z_(k) - 1


def test_gaussian_statistics_match_population_threshold(oracle):
    """For n iid N(0,1) scores tau is close to the root of n E[clip(Z - tau,0,1)] = k,
    E[clip(Z-t,0,1)] = phi(t) - phi(t+1) - t (Phi(t+1)-Phi(t)) + (1 - Phi(t+1)) ... written
    with scipy's normal cdf/pdf; at n=32768, k=1024 that root is about 1.44."""
    n, k = 32768, 1024

    def g(t):
        a, b = t, t + 1
        part = (stats.norm.pdf(a) - stats.norm.pdf(b)) - t * (stats.norm.cdf(b) - stats.norm.cdf(a))
        return n * (part + stats.norm.sf(b)) - k

    root = optimize.brentq(g, 0, 4)
    assert abs(root - 1.44) < 0.02
    z = np.random.default_rng(0).standard_normal(n, dtype=np.float32)
    tau, p, us, ws = oracle.sparsek(z, k)
    assert abs(tau - root) < 0.03
    assert abs(ws - n * stats.norm.sf(root)) < 150 and abs(us - n * stats.norm.sf(root + 1)) < 60


def test_prefix_routine_equals_one_shot_and_is_monotone(oracle):
    rng = np.random.default_rng(21)
    n, k = 300, 17
    u = rng.standard_normal(n).astype(np.float32)
    u[50] = u[10]  # an exact tie
    tau, us, ws = oracle.tau_prefixes(u, k)
    for t in range(n):
        t1, _, u1, w1 = oracle.sparsek(u[: t + 1], k)
        assert tau[t] == t1 and us[t] == u1 and ws[t] == w1
        if t + 1 <= k:
            assert tau[t] == float(u[: t + 1].min()) - 1.0
    assert np.all(np.diff(tau[k - 1:]) >= 0)  # k-th largest of a growing set rises (Sec. 3.2)


def test_k0_reading(oracle):
    z = np.array([0.3, -1.0, 2.0], np.float32)
    tau, p, us, ws = oracle.sparsek(z, 0)
    assert tau == 2.0 and not p.any() and us == ws == 0


# ---------------------------------------------------------------- selection


def topk_numpy(u, t, k):
    order = np.argsort(-u[: t + 1], kind="stable")  # larger first, older first among equals
    return np.sort(order[:k])


@pytest.mark.parametrize("seed", range(3))
def test_selection_against_stable_sort(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    n, k = 160, 12
    u = rng.standard_normal(n).astype(np.float32)
    u[rng.integers(0, n, 20)] = u[rng.integers(0, n, 20)]  # plant exact ties
    dth = oracle.death(u, k)
    prev = set()
    for t in range(n):
        want = topk_numpy(u, t, k)
        got = oracle.select_prefix(u, t, k)
        assert got.tolist() == want.tolist()
        assert len(got) == min(k, t + 1)
        from_death = [j for j in range(t + 1) if dth[j] > t]
        assert from_death == want.tolist()
        assert set(want) - prev <= {t}  # irreversibility: only the newcomer may enter
        prev = set(want)


def test_selected_are_full_gates_plus_largest_fractional(oracle):
    rng = np.random.default_rng(9)
    u = rng.standard_normal(500).astype(np.float32)
    k = 30
    tau, p, us, ws = oracle.sparsek(u, k)
    assert us <= k <= ws
    sel = oracle.select_prefix(u, 499, k)
    assert np.all(p[sel] > 0)
    assert set(np.nonzero(p == 1)[0]) <= set(sel)


def test_death_edge_cases(oracle):
    u = np.array([1, 1, 1, 1, 1], np.float32)
    assert oracle.death(u, 2).tolist() == [5, 5, 2, 3, 4]  # older wins ties; later ones never enter
    assert oracle.death(u, 0).tolist() == [0, 1, 2, 3, 4]
    u = np.array([0, 1, 2, 3, 4], np.float32)
    assert oracle.death(u, 2).tolist() == [2, 3, 4, 5, 5]
    assert oracle.death(u, 9).tolist() == [5] * 5


def _score_rows(rng, n):
    yield "normal", rng.standard_normal(n).astype(np.float32)
    yield "ties", (np.round(rng.standard_normal(n) * 4) / 4).astype(np.float32)
    yield "equal", np.full(n, 0.5, np.float32)
    yield "rising", (np.arange(n) * 0.01).astype(np.float32)
    yield "falling", (-np.arange(n) * 0.3).astype(np.float32)
    yield "wide", (rng.standard_normal(n) * 50).astype(np.float32)
    yield "drift", (rng.standard_normal(n) + 0.5 * np.sin(np.arange(n) / 256)).astype(np.float32)


@pytest.mark.parametrize("n,k", [(300, 7), (1000, 64), (50, 60), (200, 0), (64, 1), (2000, 200)])
def test_incremental_two_heap_evaluation_equals_the_sort_based_one(oracle, n, k):
    """The step-by-step evaluation of Sec. 3.3 (two min-heaps with their sums, one breakpoint per step of the
    (u, w) walk) must give the threshold of the re-sorting routine on every prefix, including ties, flat
    segments (wide), prefixes of at most k scores and k = 0."""
    rng = np.random.default_rng(n + k)
    for name, u in _score_rows(rng, n):
        want = oracle.tau_prefixes(u, k)[0]
        got = oracle.tau_incremental(u, k)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-9 * max(1.0, np.abs(want).max()), err_msg=name)
