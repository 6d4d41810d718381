"""Float64 oracle of the threshold-initialisation stage of AdaSplash-2 (numpy).

TEST INFRASTRUCTURE ONLY; shares no code with the GPU path.

Follows the paper's steps in its own order and notation:
  centre        z = (alpha-1) s - (m - 1),  m = (alpha-1) max s            (Eq. 6)
  bin           b(z) = min(floor(B z), B-1) for z >= 0, z < 0 dropped       (Eq. 7, App. C.2)
  histogram     H_k = #{j : b(z_j) = k}                                     (Eq. 8)
  objective     f_h(tau) = -1 + sum_k H_k [k/B - tau]_+^{1/(alpha-1)}       (Eq. 9)
  solve         root tau_h of f_h (App. C.3), tau* - 1/B < tau_h <= tau*   (Prop. 1)
  refine        safeguarded hybrid solver on the true scores               (Sec. 3.2)
  right edge    b(z) = ceil(B z)/B: root >= tau*, the sparser approximation (Sec. 3.2, after Prop. 1)
and the packed encodings of App. C.2, C.4, C.5 (used as printed-value pins).
All thresholds in this module are in centred units (z), i.e. tau_z = tau_raw - (m - 1).
"""
import math

import numpy as np


def centre(x):
    """x = (alpha-1) s for the visible keys -> (z, shift) with z = x - shift, max z = 1 (Eq. 6)."""
    x = np.asarray(x, dtype=np.float64)
    shift = x.max() - 1.0
    return x - shift, shift


def bin_index(z, B):
    """Bin of every z >= 0 (Eq. 7 with the clamp of App. C.2); -1 for z < 0 (not counted)."""
    z = np.asarray(z, dtype=np.float64)
    k = np.minimum(np.maximum(np.floor(B * z), 0), B - 1).astype(np.int64)
    return np.where(z >= 0, k, -1)


def histogram(z, B):
    """H_k of Eq. 8."""
    k = bin_index(z, B)
    return np.bincount(k[k >= 0], minlength=B).astype(np.int64)


def histogram_right_edge(z, B):
    """Right-edge binning (Sec. 3.2, after Prop. 1): b(z) = ceil(B z) / B, so the counts sit on the
    B + 1 edges 0, 1/B, ..., 1; z < 0 dropped.  Returns H of length B + 1."""
    z = np.asarray(z, dtype=np.float64)
    k = np.ceil(B * z[z >= 0]).astype(np.int64)
    return np.bincount(np.minimum(k, B), minlength=B + 1).astype(np.int64)


def f_h_right_edge(H, alpha, tau):
    """Eq. 9 with the counts of histogram_right_edge: -1 + sum_k H_k [k/B - tau]_+^{1/(alpha-1)}, k = 0..B."""
    B = len(H) - 1
    y = np.arange(B + 1, dtype=np.float64) / B - tau
    act = y > 0
    return float(np.sum(np.asarray(H, dtype=np.float64)[act] * y[act] ** (1.0 / (alpha - 1.0))) - 1.0)


def solve_histogram_right_edge(H, alpha):
    """Root of f_h_right_edge by bisection on [-1/B, 1]; tau* <= root < tau* + 1/B."""
    B = len(H) - 1
    lo, hi = -1.0 / B, 1.0
    while hi - lo > 1e-13:
        mid = 0.5 * (lo + hi)
        if f_h_right_edge(H, alpha, mid) >= 0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def f_true(z, alpha, tau):
    """f(tau) of Eq. 4 on centred scores."""
    y = np.asarray(z, dtype=np.float64) - tau
    y = y[y > 0]
    return float(np.sum(y ** (1.0 / (alpha - 1.0))) - 1.0)


def f_h(H, alpha, tau):
    """f_h(tau) of Eq. 9."""
    B = len(H)
    edges = np.arange(B, dtype=np.float64) / B
    y = edges - tau
    act = y > 0
    return float(np.sum(np.asarray(H, dtype=np.float64)[act] * y[act] ** (1.0 / (alpha - 1.0))) - 1.0)


def solve_histogram(H, alpha):
    """Root tau_h of f_h.

    alpha in {1.5, 2}: descending scan over bins keeping S0, S1, S2 of the active set
    P = [B-1, ..., k]; the active set is the largest one whose closed-form root lies
    below the left edge of its lowest (non-empty) bin (App. C.3, read with the
    criterion of the sort-based solvers of App. A applied to the (edge, count) pairs).
    Other alpha: bisection of f_h on [-1/B, (B-1)/B] (App. C.3 "General alpha").
    The result can be negative (down to -1/B): the maximum itself is rounded down to
    (B-1)/B.  Callers clamp at 0 because tau* >= 0 in centred units (App. B preamble).
    """
    H = np.asarray(H, dtype=np.int64)
    B = len(H)
    if alpha == 2.0 or alpha == 1.5:
        S0 = S1 = S2 = 0.0
        best = None
        for k in range(B - 1, -1, -1):
            if H[k] == 0:
                continue
            e = k / B
            S0 += H[k]; S1 += H[k] * e; S2 += H[k] * e * e
            if alpha == 2.0:
                t = (S1 - 1.0) / S0
            else:
                mean = S1 / S0
                disc = max(mean * mean - (S2 - 1.0) / S0, 0.0)
                t = mean - math.sqrt(disc)
            if t < e:
                best = t
        return best
    lo, hi = -1.0 / B, (B - 1.0) / B
    while hi - lo > 1e-13:
        mid = 0.5 * (lo + hi)
        if f_h(H, alpha, mid) >= 0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def hybrid_step(z, alpha, tau, prev=None):
    """f, f', f'' of App. B part (i) on the true centred scores, and the raw update:
    Halley for alpha <= 1.5, Newton for 1.5 < alpha <= 2, and for alpha > 2, where f' is unbounded,
    the secant through this iterate and the one before, prev = (tau, f) (Sec. 3.2); no update
    (infinite) when there is no earlier iterate."""
    r = 1.0 / (alpha - 1.0)
    y = np.asarray(z, dtype=np.float64) - tau
    y = y[y > 0]
    f = float(np.sum(y ** r) - 1.0)
    if alpha > 2.0:
        if prev is None or prev[1] == f:
            return f, float("inf")
        return f, -f * (tau - prev[0]) / (f - prev[1])
    f1 = float(-r * np.sum(y ** (r - 1.0)))
    if alpha <= 1.5:
        f2 = float(r * (r - 1.0) * np.sum(y ** (r - 2.0)))
        den = 2.0 * f1 * f1 - f * f2
        delta = -2.0 * f * f1 / den if den != 0.0 else float("inf")
    else:
        delta = -f / f1 if f1 != 0.0 else float("inf")
    return f, delta


def hybrid_solver(z, alpha, tau0, lo, hi, tol, max_iter=64, trace=None):
    """Safeguarded hybrid refinement (Sec. 3.2): the proposed update is replaced by the
    bracket's midpoint when it leaves (lo, hi).

    One iteration = one evaluation of f (and derivatives) over the true scores followed
    by one update.  A row stops when |f| <= tol or when its update moves tau by less
    than tol.  For alpha > 2 a short secant step says nothing about the distance to the root
    (f rises vertically at every score): while the bracket is wider than tol such a step is
    lengthened to 2 tol, so the row stops on a short step only once the bracket is that narrow
    (or its midpoint that near).
    Returns (tau, iterations).
    """
    tau = float(tau0)
    it = 0
    prev = None
    while it < max_iter:
        f, delta = hybrid_step(z, alpha, tau, prev)
        prev = (tau, f)
        it += 1
        if trace is not None:
            trace.append(tau)
        if abs(f) <= tol:
            break
        if f > 0:
            lo = tau
        else:
            hi = tau
        if alpha > 2.0 and abs(delta) < tol and hi - lo >= tol:
            delta = 2 * tol if f > 0 else -2 * tol
        cand = tau + delta
        if not (lo < cand < hi):
            cand = 0.5 * (lo + hi)
        step = cand - tau
        tau = cand
        if abs(step) < tol:
            break
    if trace is not None:
        trace.append(tau)
    return tau, it


def tau_from_histogram(x, alpha, B, tol, max_iter=64):
    """Whole threshold pipeline for one row of pre-scaled scores x = (alpha-1) s:
    returns (tau_raw, iterations, tau0_centred)."""
    z, shift = centre(x)
    H = histogram(z, B)
    tau_h = solve_histogram(H, alpha)
    tau0 = max(tau_h, 0.0)
    tau, it = hybrid_solver(z, alpha, tau0, tau0, tau_h + 1.0 / B, tol, max_iter)
    return tau + shift, it, tau0


# ---- packed encodings (App. C.2, C.4, C.5): printed-value pins only -----------------

def pack_histogram_word(counts, w):
    """sum_k c_k 2^{k b}, b = w / B (App. C.2)."""
    B = len(counts)
    b = w // B
    word = 0
    for k, c in enumerate(counts):
        assert 0 <= c < (1 << b)
        word += int(c) << (k * b)
    return word


def unpack_histogram_word(word, w, B):
    b = w // B
    return [(word >> (k * b)) & ((1 << b) - 1) for k in range(B)]


def histogram_capacity(w, B, Bc):
    """C_max = B_c (2^{w/B} - 1) (Sec. 3.3 "Histogram capacity")."""
    return Bc * ((1 << (w // B)) - 1)


def n_flush(Tc, b):
    """ceil(T_c / (2^b - 1)) (App. C.5)."""
    return -(-Tc // ((1 << b) - 1))


def pack_mask_row(bits):
    """M^packed_{i,m} = sum_k M_{i,32m+k} 2^k (App. C.4), as unsigned 32-bit words."""
    bits = list(bits)
    W = (len(bits) + 31) // 32
    words = [0] * W
    for j, bit in enumerate(bits):
        if bit:
            words[j // 32] |= 1 << (j % 32)
    return words
