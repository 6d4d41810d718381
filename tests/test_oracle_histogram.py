"""Pins of the histogram-initialisation oracle (CPU only)."""
import os

import numpy as np
import pytest

from oracle import entmax_oracle as eo
from oracle import histogram_oracle as ho

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(7)


def test_fig5_packed_word():
    lines = [l.split() for l in open(os.path.join(GOLDEN, "fig5_packed_word.txt")) if not l.startswith("#")]
    counts = [int(v) for v in lines[0][1:]]
    word = int(lines[1][1], 16)
    assert ho.pack_histogram_word(counts, 64) == word
    assert ho.unpack_histogram_word(word, 64, 8) == counts


def test_table5_capacity():
    for l in open(os.path.join(GOLDEN, "table5_capacity.txt")):
        if l.startswith("#"):
            continue
        w, B, b, mx, cap, h = l.split()
        w, B, b, mx, cap, h = int(w), int(B), int(b), int(mx), int(cap), float(h)
        assert w // B == b and (1 << b) - 1 == mx
        assert ho.histogram_capacity(w, B, 64) == cap
        assert 1.0 / B == h
    # Sec. 3.3: default configuration w=64, B=8, B_c=64 -> 16,320 keys
    assert ho.histogram_capacity(64, 8, 64) == 16320
    # App. C.5: flushes = ceil(T_c / (2^b - 1))
    assert ho.n_flush(256, 8) == 2 and ho.n_flush(255, 8) == 1 and ho.n_flush(1024, 8) == 5


def test_mask_row_packing():
    bits = [0] * 70
    for j in (0, 3, 31, 32, 69):
        bits[j] = 1
    assert ho.pack_mask_row(bits) == [1 | 8 | (1 << 31), 1, 1 << 5]


def test_binning_rules():
    B = 8
    z = np.array([-0.01, 0.0, 0.1249, 0.125, 0.99, 1.0])
    assert list(ho.bin_index(z, B)) == [-1, 0, 0, 1, 7, 7]   # z<0 dropped, z=1 clamped to B-1
    assert list(ho.histogram(z, B)) == [2, 1, 0, 0, 0, 0, 0, 2]


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0, 1.75])
@pytest.mark.parametrize("B", [4, 8, 16, 64])
def test_prop1_lower_bound_and_sandwich(alpha, B):
    h = 1.0 / B
    for n, scale in [(1, 1.0), (7, 1.0), (300, 0.5), (4096, 1.0), (4096, 6.0)]:
        x = (alpha - 1) * RNG.normal(size=n) * scale
        z, shift = ho.centre(x)
        assert abs(z.max() - 1.0) < 1e-15
        tau_star = eo.tau_row(x, alpha) - shift
        assert -1e-12 <= tau_star <= 1 - n ** (1 - alpha) + 1e-12     # App. A bracket in centred units
        H = ho.histogram(z, B)
        assert H.sum() == int((z >= 0).sum())
        tau_h = ho.solve_histogram(H, alpha)
        assert abs(ho.f_h(H, alpha, tau_h)) < 1e-9
        assert tau_star - h < tau_h + 1e-11 and tau_h <= tau_star + 1e-11      # Prop. 1
        for t in np.linspace(0.0, 1.0, 23):                                    # App. B.1 step 1
            assert ho.f_h(H, alpha, t) <= ho.f_true(z, alpha, t) + 1e-10
            if ho.f_true(z, alpha, t) > -1.0:                                  # some score above t
                assert ho.f_true(z, alpha, t) < ho.f_h(H, alpha, t - h) + 1e-10
        # support at max(tau_h, 0) contains the true support
        assert np.all((z > max(tau_h, 0)) | ~(z > tau_star))


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0, 3.0])
@pytest.mark.parametrize("B", [8, 63])
def test_right_edge_binning_bounds_the_threshold_from_above(alpha, B):
    # the mirror image of Prop. 1: tau* <= tau_h < tau* + h; every bin moves up by h against
    # left-edge binning, so the root does too; the support it leaves lies inside the true one
    h = 1.0 / B
    for n, scale in [(1, 1.0), (7, 1.0), (300, 0.5), (4096, 1.0), (4096, 6.0)]:
        x = (alpha - 1) * RNG.normal(size=n) * scale
        z, shift = ho.centre(x)
        tau_star = eo.tau_row(x, alpha) - shift
        HR = ho.histogram_right_edge(z, B)
        assert HR.sum() == int((z >= 0).sum()) and HR[B] >= 1          # the maximum sits on the last edge
        tau_r = ho.solve_histogram_right_edge(HR, alpha)
        assert abs(ho.f_h_right_edge(HR, alpha, tau_r)) < 1e-8
        assert tau_star - 1e-11 <= tau_r < tau_star + h + 1e-11
        for t in np.linspace(0.0, 1.0, 23):
            assert ho.f_h_right_edge(HR, alpha, t) >= ho.f_true(z, alpha, t) - 1e-10
        assert np.all(~(z > tau_r) | (z > tau_star - 1e-12))
        if alpha in (1.5, 2.0) or n > 1:
            tau_l = ho.solve_histogram(ho.histogram(z, B), alpha)
            assert abs(tau_r - (tau_l + h)) < 1e-9


def test_right_edge_binning_rule():
    B = 8
    z = np.array([-0.01, 0.0, 0.1249, 0.125, 0.1251, 0.99, 1.0])
    assert list(ho.histogram_right_edge(z, B)) == [1, 2, 1, 0, 0, 0, 0, 0, 2]


@pytest.mark.parametrize("alpha", [1.5, 2.0])
def test_closed_form_scan_agrees_with_generic_root(alpha):
    for B in (8, 32):
        for _ in range(20):
            H = RNG.integers(0, 6, size=B)
            H[B - 1] = max(H[B - 1], 1)            # the maximum always sits in the last bin
            t = ho.solve_histogram(H, alpha)
            lo, hi = -1.0 / B, (B - 1.0) / B
            while hi - lo > 1e-14:
                mid = 0.5 * (lo + hi)
                if ho.f_h(H, alpha, mid) >= 0: lo = mid
                else: hi = mid
            assert abs(t - lo) < 1e-10


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0, 2.5, 3.0])
def test_hybrid_solver_reaches_exact_threshold(alpha):
    for n, scale in [(1, 1.0), (50, 1.0), (4096, 1.0), (4096, 8.0)]:
        x = (alpha - 1) * RNG.normal(size=n) * scale
        exact = eo.tau_row(x, alpha)
        for B, tol in [(8, 1e-6), (64, 1e-4), (64, 1e-6)]:
            tau, it, tau0 = ho.tau_from_histogram(x, alpha, B, tol)
            assert abs(tau - exact) < 20 * tol
            # secant steps (alpha > 2) come down to bisection when a score sits on the root
            assert it <= (6 if alpha <= 2 else 30)


def test_secant_does_not_stop_on_a_short_step_far_from_the_root():
    # alpha = 3 and a score that sits almost on the root: f rises vertically just below it, and a
    # secant taken on the flat side proposes a step shorter than tol while still 5e-4 away.  A
    # solver that stops on that step misses the root by more than tol; the rule that lengthens
    # short steps while the bracket is wide does not.
    alpha, tol = 3.0, 1e-4
    x = np.array([15.42228769, 14.42482779, 14.41279519, 14.33566045, 14.29362637, 12.97043358, 12.05384912, 11.99181098])
    exact = eo.tau_row(x, alpha)
    tau, it, _ = ho.tau_from_histogram(x, alpha, 63, tol)
    assert abs(tau - exact) <= tol and it <= 30
    z, shift = ho.centre(x)
    tau_h = ho.solve_histogram(ho.histogram(z, 63), alpha)
    lo, hi, t, prev, naive = max(tau_h, 0.0), tau_h + 1 / 63, max(tau_h, 0.0), None, None
    for _ in range(30):                      # the same iteration without that rule
        f, delta = ho.hybrid_step(z, alpha, t, prev)
        prev = (t, f)
        if abs(f) <= tol:
            break
        lo, hi = (t, hi) if f > 0 else (lo, t)
        cand = t + delta if lo < t + delta < hi else 0.5 * (lo + hi)
        short = abs(cand - t) < tol
        t = cand
        if short:
            break
    assert abs(t + shift - exact) > 3 * tol


def test_solver_study_shape():
    """Sec. 4.1: Gaussian scores, n = 4096, alpha = 1.5: the histogram start puts the first
    refinement step orders of magnitude closer than the start itself, more bins help, and two
    steps reach the exact threshold to ~1e-6 or better."""
    alpha = 1.5
    err = {}
    for B in (4, 8, 16, 64):
        e0, e1, e2 = [], [], []
        for run in range(10):
            x = (alpha - 1) * np.random.default_rng(run).normal(size=4096)
            z, shift = ho.centre(x)
            exact = eo.tau_row(x, alpha) - shift
            tau_h = ho.solve_histogram(ho.histogram(z, B), alpha)
            t0 = max(tau_h, 0.0)
            tr = []
            ho.hybrid_solver(z, alpha, t0, t0, tau_h + 1.0 / B, 0.0, max_iter=2, trace=tr)
            e0.append(abs(tr[0] - exact)); e1.append(abs(tr[1] - exact)); e2.append(abs(tr[2] - exact))
        err[B] = (np.mean(e0), np.mean(e1), np.mean(e2))
        assert err[B][0] < 1.0 / B
        assert err[B][1] < err[B][0] / 10
        assert err[B][2] < 1e-5
    assert err[4][0] > err[8][0] > err[16][0] > err[64][0]
    assert err[4][1] > err[8][1] > err[16][1] > err[64][1]
