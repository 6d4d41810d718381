"""Pins of the float64 oracle's threshold and probability map (CPU only).

Each test checks the oracle against something other than itself: closed forms, the
variational definition solved by a generic optimiser, textbook limits, invariants.
"""
import math

import numpy as np
import pytest
from scipy import optimize

from oracle import entmax_oracle as eo

RNG = np.random.default_rng(1234)
ALPHAS = [1.25, 1.5, 1.75, 2.0, 1.1, 2.5, 3.0]


def tsallis_objective(p, s, alpha):
    # App. A: entmax = argmax_p <p, s> + H_alpha(p), H_alpha(p) = sum(p - p^alpha) / (alpha (alpha-1))
    p = np.clip(p, 0.0, None)
    return -(p @ s + np.sum(p - p ** alpha) / (alpha * (alpha - 1.0)))


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0, 1.8, 2.5, 3.0])
def test_matches_variational_definition(alpha):
    # generic constrained optimiser on the simplex, tiny n
    for n in (3, 5, 7):
        s = RNG.normal(size=n) * 1.5
        p, _ = eo.entmax(s, alpha)
        cons = [{"type": "eq", "fun": lambda q: q.sum() - 1.0}]
        best = None
        for start in (np.full(n, 1.0 / n), p * 0.5 + 0.5 / n):
            res = optimize.minimize(tsallis_objective, start, args=(s, alpha), method="SLSQP",
                                    bounds=[(0.0, 1.0)] * n, constraints=cons,
                                    options={"ftol": 1e-15, "maxiter": 500})
            if best is None or res.fun < best.fun:
                best = res
        assert np.abs(best.x - p).max() < 2e-5, (alpha, n, best.x, p)
        # and the oracle's point is at least as good as the optimiser's
        assert tsallis_objective(p, s, alpha) <= best.fun + 1e-10


def test_sparsemax_two_element_closed_form():
    # alpha = 2: scores (a, b), a >= b: p = (1, 0), tau = a - 1 if a - b >= 1,
    # else p = ((1 + a - b)/2, (1 - a + b)/2)
    for a, b in [(0.3, -0.1), (2.0, 0.5), (1.0, 0.0), (0.2, 0.2), (5.0, 4.5)]:
        p, tau = eo.entmax(np.array([a, b]), 2.0)
        if a - b >= 1:
            assert np.allclose(p, [1.0, 0.0], atol=1e-15) and abs(tau - (a - 1.0)) < 1e-15
        else:
            assert np.allclose(p, [(1 + a - b) / 2, (1 - a + b) / 2], atol=1e-15)
            assert abs(tau - (a + b - 1) / 2) < 1e-15


def test_entmax15_two_element_closed_form():
    # alpha = 1.5, x = s/2: (x_a - tau)^2 + (x_b - tau)^2 = 1 when both active
    for a, b in [(0.3, -0.1), (1.0, 0.2), (4.0, 0.5), (0.0, 0.0)]:
        xa, xb = a / 2, b / 2
        p, tau = eo.entmax(np.array([a, b]), 1.5)
        if xa - xb >= 1:
            assert np.allclose(p, [1.0, 0.0], atol=1e-15) and abs(tau - (xa - 1)) < 1e-15
        else:
            t = (xa + xb) / 2 - math.sqrt(0.5 - (xa - xb) ** 2 / 4)
            assert abs(tau - t) < 1e-14
            assert np.allclose(p, [(xa - t) ** 2, (xb - t) ** 2], atol=1e-14)


def test_alpha3_two_element_closed_form():
    # alpha = 3, x = 2 s: sqrt(x_a - tau) + sqrt(x_b - tau) = 1 when both are active; with
    # u = sqrt(x_a - tau): x_a - x_b = u^2 - (1 - u)^2 = 2u - 1, so p = ((1 + D)/2, (1 - D)/2), D = x_a - x_b < 1
    for a, b in [(0.3, -0.1), (0.2, 0.2), (1.0, 0.6), (3.0, 0.5), (0.45, 0.0)]:
        xa, xb = 2 * a, 2 * b
        p, tau = eo.entmax(np.array([a, b]), 3.0)
        if xa - xb >= 1:
            assert np.allclose(p, [1.0, 0.0], atol=1e-12) and abs(tau - (xa - 1)) < 1e-12
        else:
            u = (1 + xa - xb) / 2
            assert np.allclose(p, [u, 1 - u], atol=1e-11)
            assert abs(tau - (xa - u * u)) < 1e-11


def sparsemax_textbook(s):
    # Euclidean projection onto the simplex, Held et al. / Duchi et al. formulation:
    # rho = max{k : s_(k) - (sum_{i<=k} s_(i) - 1)/k > 0}
    u = np.sort(s)[::-1]
    css = np.cumsum(u)
    k = np.arange(1, len(s) + 1)
    rho = k[u - (css - 1) / k > 0][-1]
    theta = (css[rho - 1] - 1) / rho
    return np.maximum(s - theta, 0), theta


def test_alpha2_is_simplex_projection():
    for n in (1, 2, 17, 300):
        s = RNG.normal(size=n) * 2
        p, tau = eo.entmax(s, 2.0)
        q, theta = sparsemax_textbook(s)
        assert np.abs(p - q).max() < 1e-14 and abs(tau - theta) < 1e-14
        # projection property: p minimises ||p - s||^2 on the simplex -> KKT residual
        support = p > 0
        assert np.allclose((s - p)[support], tau, atol=1e-13)
        assert np.all((s - p)[~support] <= tau + 1e-13)


@pytest.mark.parametrize("alpha", [1.5, 2.0])
def test_sort_solver_agrees_with_bisection(alpha):
    for n, scale in [(5, 1.0), (64, 0.3), (1000, 3.0), (4096, 1.0)]:
        x = (alpha - 1) * RNG.normal(size=n) * scale
        assert abs(eo.tau_sort(x, alpha) - eo.tau_bisect(x, alpha, 1e-13)) < 1e-10


@pytest.mark.parametrize("alpha", ALPHAS)
def test_candidate_restriction_changes_nothing(alpha):
    for n in (3, 50, 2000):
        x = (alpha - 1) * RNG.normal(size=n) * 2.0
        assert abs(eo.tau_row(x, alpha, full=False) - eo.tau_row(x, alpha, full=True)) < 2e-12


@pytest.mark.parametrize("alpha", ALPHAS)
def test_probability_vector_and_root(alpha):
    for n, scale in [(1, 1.0), (2, 1.0), (33, 0.1), (500, 1.0), (4096, 4.0)]:
        s = RNG.normal(size=n) * scale
        p, tau = eo.entmax(s, alpha)
        assert np.all(p >= 0)
        assert abs(p.sum() - 1.0) < 1e-10
        x = (alpha - 1) * s
        # Eq. 5 bracket
        m = x.max()
        assert m - 1 - 1e-12 <= tau <= m - n ** (1 - alpha) + 1e-12
        # f strictly decreasing around the root, root unique
        assert eo.f(x, alpha, tau - 1e-3) > 0 > eo.f(x, alpha, tau + 1e-3)
        # zero exactly where (alpha-1) s <= tau
        assert np.array_equal(p > 0, x > tau)


@pytest.mark.parametrize("alpha", ALPHAS)
def test_special_rows(alpha):
    # all-equal scores: p = 1/n, tau at the upper end of Eq. 5
    for n in (1, 4, 100):
        s = np.full(n, 0.7)
        p, tau = eo.entmax(s, alpha)
        assert np.allclose(p, 1.0 / n, atol=1e-11)
        assert abs(tau - ((alpha - 1) * 0.7 - n ** (1 - alpha))) < 1e-11
    # one score at least 1/(alpha-1) above the rest: one-hot, tau at the lower end
    s = np.array([0.0, -1.0 / (alpha - 1) - 0.01, -5.0 / (alpha - 1)])
    p, tau = eo.entmax(s, alpha)
    assert np.allclose(p, [1, 0, 0], atol=1e-12) and abs(tau - (-1.0)) < 1e-12


@pytest.mark.parametrize("alpha", ALPHAS)
def test_shift_invariance(alpha):
    s = RNG.normal(size=40)
    p0, t0 = eo.entmax(s, alpha)
    for c in (-3.0, 0.25, 100.0):
        p1, t1 = eo.entmax(s + c, alpha)
        assert np.abs(p1 - p0).max() < 1e-9
        assert abs(t1 - (t0 + (alpha - 1) * c)) < 1e-9


def test_alpha_to_one_is_softmax():
    s = RNG.normal(size=16)
    sm = np.exp(s - s.max()); sm /= sm.sum()
    prev = None
    for alpha in (1.1, 1.01, 1.001):
        p, _ = eo.entmax(s, alpha)
        err = np.abs(p - sm).max()
        assert err < (alpha - 1)
        assert prev is None or err < prev
        prev = err


def test_mask_word_packing():
    m = np.full((1, 1, 2, 40), -1.0)
    m[0, 0, 0, [0, 5, 31, 32, 39]] = 0.5
    w = eo.block_mask_words(m).view(np.uint32)
    assert w.shape == (1, 1, 2, 2)
    assert int(w[0, 0, 0, 0]) == (1 | (1 << 5) | (1 << 31)) and int(w[0, 0, 0, 1]) == (1 | (1 << 7))
    assert int(w[0, 0, 1, 0]) == 0
