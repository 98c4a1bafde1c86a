"""Pins for the oracle's alpha-entmax (Eq. 2 and App. A of the paper).

Each test checks the oracle against something other than itself: a closed
form, an invariant the definition fixes, a library optimiser, or brute force.
"""
import itertools
import math

import numpy as np
import pytest
from scipy import optimize, special

from oracle import dash_oracle as orc

ALPHAS = [1.25, 1.5, 1.75, 2.0, 3.0]


def rng(seed):
    return np.random.default_rng(seed)


@pytest.mark.parametrize("alpha", ALPHAS)
def test_simplex_and_threshold_form(alpha):
    r = rng(1)
    for n in (1, 2, 5, 33, 257):
        s = r.normal(size=n) * 2.0
        p = orc.entmax(s, alpha)
        assert np.all(p >= 0.0)
        assert abs(p.sum() - 1.0) < 1e-12
        # zero exactly where (alpha-1) s_i <= tau  (text below Eq. 2)
        x = (alpha - 1) * s
        tau = orc.entmax_threshold(x, alpha)
        assert np.array_equal(p > 0, x > tau)


@pytest.mark.parametrize("alpha", ALPHAS)
def test_shift_invariance_and_permutation_equivariance(alpha):
    r = rng(2)
    s = r.normal(size=40)
    p = orc.entmax(s, alpha)
    assert np.allclose(orc.entmax(s + 3.7, alpha), p, atol=1e-12)
    perm = r.permutation(40)
    assert np.allclose(orc.entmax(s[perm], alpha), p[perm], atol=1e-13)


@pytest.mark.parametrize("alpha", ALPHAS)
def test_constant_input_is_uniform(alpha):
    n, c = 17, 0.8
    s = np.full(n, c)
    p = orc.entmax(s, alpha)
    assert np.allclose(p, 1.0 / n, atol=1e-13)
    tau = orc.entmax_threshold((alpha - 1) * s, alpha)
    assert abs(tau - ((alpha - 1) * c - n ** (-(alpha - 1)))) < 1e-12


def test_two_element_closed_forms():
    # sparsemax([a,b]) = ((1+a-b)/2, (1-a+b)/2) when |a-b| < 1, else one-hot
    for a, b in [(0.0, 0.0), (0.3, -0.2), (1.4, 1.0), (2.0, 0.5), (-1.0, 0.5)]:
        p = orc.entmax(np.array([a, b]), 2.0)
        if abs(a - b) < 1:
            want = np.array([(1 + a - b) / 2, (1 - a + b) / 2])
        else:
            want = np.array([1.0, 0.0]) if a > b else np.array([0.0, 1.0])
        assert np.allclose(p, want, atol=1e-14)
    # 1.5-entmax([a,b]): x = s/2, D = (a-b)/2; u1^2 + (u1-D)^2 = 1 gives
    # p1 = (D/2 + sqrt(1/2 - D^2/4))^2 while |D| < 1, else one-hot.
    for a, b in [(0.0, 0.0), (1.0, 0.0), (0.2, 1.9), (3.0, 0.5), (0.0, 2.0)]:
        p = orc.entmax(np.array([a, b]), 1.5)
        D = (a - b) / 2
        if abs(D) < 1:
            p1 = (D / 2 + math.sqrt(0.5 - D * D / 4)) ** 2
            want = np.array([p1, 1 - p1])
        else:
            want = np.array([1.0, 0.0]) if a > b else np.array([0.0, 1.0])
        assert np.allclose(p, want, atol=1e-14)
    # hand value: s = [1, 0], alpha = 1.5 -> p1 = (1/4 + sqrt(7)/4)^2
    p = orc.entmax(np.array([1.0, 0.0]), 1.5)
    assert abs(p[0] - ((1 + math.sqrt(7)) / 4) ** 2) < 1e-14


def test_alpha2_is_euclidean_projection_onto_simplex():
    r = rng(3)
    for n in (3, 6, 12):
        z = r.normal(size=n) * 1.5
        p = orc.entmax(z, 2.0)
        cons = ({"type": "eq", "fun": lambda q: q.sum() - 1.0},)
        res = optimize.minimize(lambda q: np.sum((q - z) ** 2), np.full(n, 1.0 / n),
                                jac=lambda q: 2 * (q - z), bounds=[(0, 1)] * n,
                                constraints=cons, method="SLSQP",
                                options={"ftol": 1e-14, "maxiter": 500})
        assert res.success
        assert np.allclose(p, res.x, atol=1e-6)


def _tsallis(p, alpha):
    return np.sum(p - p ** alpha) / (alpha * (alpha - 1))


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0])
def test_variational_definition(alpha):
    # App. A: entmax(z) = argmax_{p in simplex} p.z + H_alpha(p)
    r = rng(4)
    for n in (3, 5):
        z = r.normal(size=n) * 2
        p = orc.entmax(z, alpha)
        obj = lambda q: -(q @ z + _tsallis(np.maximum(q, 0), alpha))
        cons = ({"type": "eq", "fun": lambda q: q.sum() - 1.0},)
        best = None
        for start in (np.full(n, 1.0 / n), p * 0.5 + 0.5 / n):
            res = optimize.minimize(obj, start, bounds=[(0, 1)] * n, constraints=cons,
                                    method="SLSQP", options={"ftol": 1e-15, "maxiter": 1000})
            if best is None or res.fun < best.fun:
                best = res
        # the oracle's p must be at least as good as the optimiser's and close to it
        assert obj(p) <= best.fun + 1e-9
        assert np.allclose(p, best.x, atol=2e-4)


@pytest.mark.parametrize("alpha", [1.3, 1.5, 2.0, 2.5])
def test_brute_force_over_supports(alpha):
    # Enumerate every candidate support S; solve sum_{i in S}(x_i - t)^p = 1 on
    # it; the only self-consistent S (members > t >= non-members) is entmax's.
    r = rng(5)
    pw = 1.0 / (alpha - 1.0)
    for trial in range(12):
        n = int(r.integers(2, 8))
        s = r.normal(size=n) * (0.5 + trial % 3)
        x = (alpha - 1) * s
        found = []
        for k in range(1, n + 1):
            for S in itertools.combinations(range(n), k):
                xs = x[list(S)]
                f = lambda t: np.sum(np.maximum(xs - t, 0) ** pw) - 1.0
                lo, hi = xs.max() - 1.0 - 1e-9, xs.max()
                t = optimize.brentq(f, lo, hi, xtol=1e-15, rtol=1e-15)
                inside = np.zeros(n, bool); inside[list(S)] = True
                if np.all(x[inside] > t) and np.all(x[~inside] <= t):
                    found.append((S, t))
        assert len(found) == 1
        S, t = found[0]
        tau = orc.entmax_threshold(x, alpha)
        assert abs(tau - t) < 1e-11
        p = orc.entmax(s, alpha)
        assert set(np.nonzero(p)[0]) == set(S)


def test_exact_and_bisection_agree():
    r = rng(6)
    for alpha in (1.5, 2.0):
        for n in (1, 2, 9, 100, 700):
            x = (alpha - 1) * r.normal(size=n) * 3
            assert abs(orc.entmax_threshold_exact(x, alpha)
                       - orc.entmax_threshold_bisect(x, alpha)) < 1e-13


def test_alpha_to_one_recovers_softmax():
    r = rng(7)
    s = r.normal(size=12)
    sm = special.softmax(s)
    e1 = np.abs(orc.entmax(s, 1.01) - sm).max()
    e2 = np.abs(orc.entmax(s, 1.001) - sm).max()
    assert e1 < 2e-2 and e2 < 2e-3 and e2 < e1 / 5   # O(alpha - 1)


def test_sparsity_monotone_in_alpha():
    r = rng(8)
    for _ in range(10):
        s = r.normal(size=64) * 2
        zeros = [int(np.sum(orc.entmax(s, a) == 0)) for a in (1.1, 1.25, 1.5, 1.75, 2.0, 3.0)]
        assert zeros == sorted(zeros)


def test_entropy_bounded_by_log_support():
    # a sparse distribution has Shannon entropy <= log |support|
    r = rng(9)
    p = orc.entmax(r.normal(size=200) * 3, 1.5)
    nz = p[p > 0]
    assert -(nz * np.log(nz)).sum() <= math.log(nz.size) + 1e-12
    assert nz.size < 200
