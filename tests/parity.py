"""Helpers shared by the GPU parity tests: run the HIP path and the oracle on the same seeded
inputs and compare element by element.

Tolerances (the benchmark spec): bf16 inputs with fp32 accumulation |dO| <= 1e-2 abs and
|dtau| <= 1e-3; fp32 path <= 1e-5; block mask bit-exact where the oracle's block margin is
clear of zero by more than 1e-3.  Gradients: the same absolute figures relative to
(1 + |oracle value|), since their scale follows that of dO, K and Q.
"""
import numpy as np
import torch

from oracle import entmax_oracle as eo

TOL = {
    torch.bfloat16: dict(O=1e-2, tau=1e-3, grad=1e-2),
    torch.float32: dict(O=1e-5, tau=1e-5, grad=1e-5),
}
MASK_BAND = 1e-3


def to_np64(t):
    return t.detach().to(torch.float64).cpu().numpy()


def unpack_mask(words, T):
    """int32 [..., T, W] -> bool [..., T, T]"""
    w = words.cpu().numpy().view(np.uint32)
    bits = ((w[..., :, :, None] >> np.arange(32, dtype=np.uint32)) & 1).astype(bool)
    return bits.reshape(*w.shape[:-1], -1)[..., :T]


def y_accuracy(X, dtype):
    """How well the kernels know y = (alpha-1) s - tau: the refinement stops within tol_solver (1e-4
    for bf16 inputs, 1e-6 for fp32) of the root, and an fp32 dot product of d terms carries a few
    units of 2^-24 of relative error."""
    tol_solver = 1e-4 if dtype == torch.bfloat16 else 1e-6
    return 2 * tol_solver + 2.0 ** -21 * (1 + np.abs(X))


def output_slack(Q, K, V, alpha, causal, tau_ref):
    """What a perturbation of y within y_accuracy can change in O, per element, worst case.  Needed
    for alpha > 2, where P = y_+^r with r = 1/(alpha-1) < 1 has an unbounded slope at the edge of
    the support (a score 1e-6 above the threshold already has P = 1e-3 at alpha = 3), and where fp32
    inputs are compared at a score scale whose own rounding exceeds the 1e-5 bar:
        bP = max |P(y +- eta) - P(y)|,   O moves by at most  bP |V|."""
    Qn, Kn, Vn = (to_np64(t) for t in (Q, K, V))
    B, H, N, d = Qn.shape
    r = 1.0 / (alpha - 1.0)
    out = np.zeros_like(Qn)
    vis = np.tril(np.ones((N, N), bool)) if causal else None
    for b in range(B):
        for h in range(H):
            X = (alpha - 1.0) * (Qn[b, h] @ Kn[b, h].T) / np.sqrt(d)
            y = X - tau_ref[b, h][:, None]
            if vis is not None:
                y = np.where(vis, y, -1e30)
            eta = y_accuracy(X, Q.dtype)
            p = np.maximum(y, 0) ** r
            bp = np.maximum(np.abs(np.maximum(y + eta, 0) ** r - p), np.abs(np.maximum(y - eta, 0) ** r - p))
            out[b, h] = bp @ np.abs(Vn[b, h])
    return out


def check_forward(Q, K, V, alpha, causal, O, tau, mask, ref=None, label="", rounding_slack=False):
    """Compare a GPU forward result with the oracle. Returns the oracle result for reuse.
    alpha > 2, or rounding_slack (fp32 inputs whose rows attend to dozens of keys: each P carries the
    rounding of its fp32 score, a few 1e-7 times the score, and O sums them over the support): the
    bound of output_slack is added to the tolerance of O, element by element."""
    tol = TOL[Q.dtype]
    if ref is None:
        ref = eo.attn_fwd(to_np64(Q), to_np64(K), to_np64(V), alpha, causal, tile=64)
    dtau = np.abs(to_np64(tau) - ref["tau"]).max()
    diffO = np.abs(to_np64(O) - ref["O"])
    dO = diffO.max()
    assert dtau <= tol["tau"], f"{label}: |dtau| = {dtau:.3e} > {tol['tau']}"
    if alpha > 2.0 or rounding_slack:
        allowed = tol["O"] + output_slack(Q, K, V, alpha, causal, ref["tau"])
        worst = (diffO / allowed).max()
        assert worst <= 1.0, f"{label}: O error is {worst:.3f} of what is allowed (|dO| = {dO:.3e})"
    else:
        assert dO <= tol["O"], f"{label}: |dO| = {dO:.3e} > {tol['O']}"
    T = Q.shape[2] // 64
    got = unpack_mask(mask, T)
    want = ref["margin"] > 0
    clear = np.abs(ref["margin"]) > MASK_BAND
    bad = (got != want) & clear
    assert not bad.any(), f"{label}: {bad.sum()} mask bits differ outside the {MASK_BAND} band"
    # padding bits and tiles above the diagonal must be zero
    w = mask.cpu().numpy().view(np.uint32)
    full = ((w[..., :, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(*w.shape[:-1], -1)
    assert not full[..., T:].any(), f"{label}: padding bits set"
    if causal:
        assert not (got & ~np.tril(np.ones((T, T), bool))).any(), f"{label}: bits above the diagonal"
    return ref, dict(dtau=float(dtau), dO=float(dO), band=int((~clear).sum()))


U_FLOOR = 1e-6      # alpha > 2: the kernels form U from max(y, 1e-6), so that it fits fp16 operands


def conditioning_slack(Q, K, V, dO, alpha, causal, tau_ref, tau_given=False):
    """What a perturbation of y = (alpha-1) s - tau within the arithmetic's own accuracy can change
    in dQ, dK, dV: a worst-case bound (sums of absolute values), per element.

    The kernels know y only up to eta = y_accuracy = 2 tol_solver + 2^-21 (1 + |x|); with tau_given
    (the backward was handed the oracle's thresholds, rounded to fp32) the solver's share drops out:
    eta = 2^-21 (1 + |x|).  At alpha = 2 the band of the block mask (1e-3) is used instead, as for
    the mask; for alpha > 2 eta is at least U_FLOOR.  The factors U = y_+^(r-1) and P = y_+^r
    (r = 1/(alpha-1)) can move by
        bU = sup |U(y') - U(y)| over |y' - y| <= eta,   bP likewise,   dn = U(y) - inf U(y')
    - for alpha <= 2 U is monotone, so the ends of the interval give them (alpha = 2: U jumps from 0
    to 1); for alpha > 2 U = y^(r-1) has a negative exponent, it grows without limit as y falls to
    zero, so bU is infinite when the interval reaches across zero, and the row, and through it every
    key of its support, is then not bound at all.  With g = dO V^T:
        delta = sum U g / sum U  moves by at most  D = sum bU |g - delta| / (sum U - sum dn)
        dS = U (g - delta)       by  bS = bU |g - delta| + (U + bU) D
        dQ by bS |K| / sqrt(d),  dK by bS^T |Q| / sqrt(d),  dV by bP^T |dO|.
    Used where the gradient is that sensitive by construction: alpha > 1.5, and fp32 inputs (whose
    1e-5 bar is of the order of the fp32 score rounding itself once a key is attended by hundreds of
    rows).  For bf16 inputs at alpha <= 1.5 the plain tolerance stands."""
    Qn, Kn, Vn, Gn = (to_np64(t) for t in (Q, K, V, dO))
    B, H, N, d = Qn.shape
    r = 1.0 / (alpha - 1.0)
    out = {k: np.zeros_like(Qn) for k in ("dQ", "dK", "dV")}
    vis = np.tril(np.ones((N, N), bool)) if causal else None

    def U(y):
        if alpha == 2.0:
            return (y > 0).astype(np.float64)
        with np.errstate(divide="ignore"):
            return np.where(y > 0, np.power(np.maximum(y, 0), r - 1.0), 0.0)

    def P(y):
        return np.power(np.maximum(y, 0), r)

    for b in range(B):
        for h in range(H):
            X = (alpha - 1.0) * (Qn[b, h] @ Kn[b, h].T) / np.sqrt(d)
            y = X - tau_ref[b, h][:, None]
            eta = 2.0 ** -21 * (1 + np.abs(X)) if tau_given else y_accuracy(X, Q.dtype)
            if alpha == 2.0:
                eta = np.maximum(eta, MASK_BAND)
            if alpha > 2.0:
                eta = np.maximum(eta, U_FLOOR)
            if vis is not None:
                y = np.where(vis, y, -1e30)
            u, p = U(y), P(y)
            up, um = U(y + eta), U(y - eta)
            bu = np.maximum(np.abs(up - u), np.abs(um - u))
            dn = np.maximum(u - np.minimum(up, um), 0.0)
            if alpha > 2.0:
                bu = np.where((y - eta <= 0) & (y + eta > 0), np.inf, bu)
            bp = np.maximum(np.abs(P(y + eta) - p), np.abs(P(y - eta) - p))
            g = Gn[b, h] @ Vn[b, h].T
            usum = u.sum(-1)
            delta = (u * g).sum(-1) / usum
            gd = np.abs(g - delta[:, None])
            touched = (u > 0) | (bu > 0)
            with np.errstate(invalid="ignore", divide="ignore"):
                num = np.where(touched, bu * gd, 0.0).sum(-1)
                den = usum - dn.sum(-1)
                D = np.where(den > 0, num / den, np.inf)
                D = np.where(num == 0, 0.0, D)
                bS = np.where(touched, bu * gd + (u + bu) * D[:, None], 0.0)
                bS = np.where(np.isnan(bS), np.inf, bS)
                sq = np.sqrt(d)
                # (0 * inf = nan in a matrix product: rows and keys that are not bound are put in afterwards)
                fin = np.where(np.isfinite(bS), bS, 0.0)
                out["dQ"][b, h] = fin @ np.abs(Kn[b, h]) / sq
                out["dK"][b, h] = fin.T @ np.abs(Qn[b, h]) / sq
                unbound = ~np.isfinite(bS)
                out["dQ"][b, h][unbound.any(1)] = np.inf
                out["dK"][b, h][unbound.any(0)] = np.inf
            out["dV"][b, h] = bp.T @ np.abs(Gn[b, h])
    return out


def check_backward(Q, K, V, dO, alpha, causal, dQ, dK, dV, ref=None, label="", tau_ref=None, tau_given=False):
    """|got - oracle| <= tol (1 + |oracle|) element-wise, tol = 1e-2 (bf16 inputs) or 1e-5 (fp32).
    For alpha > 1.5 and for fp32 inputs the bound of conditioning_slack is added (it needs the
    oracle's tau: pass tau_ref, or it is computed here).  tau_given: the gradients were computed
    from the oracle's thresholds (see conditioning_slack)."""
    tol = TOL[Q.dtype]["grad"]
    if ref is None:
        ref = eo.attn_bwd(to_np64(Q), to_np64(K), to_np64(V), to_np64(dO), alpha, causal)
    slack = None
    if alpha > 1.5 or Q.dtype == torch.float32:
        if tau_ref is None:
            tau_ref = eo.attn_fwd(to_np64(Q), to_np64(K), to_np64(V), alpha, causal, want_margin=False)["tau"]
        slack = conditioning_slack(Q, K, V, dO, alpha, causal, tau_ref, tau_given)
    out = {}
    for name, got in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        g = to_np64(got)
        allowed = tol * (1.0 + np.abs(ref[name])) + (slack[name] if slack is not None else 0.0)
        diff = np.abs(g - ref[name])
        out[name] = float((diff / (1.0 + np.abs(ref[name]))).max())
        worst = float((diff / allowed).max())
        if slack is not None:
            out[name + "_of_allowed"] = worst
            if alpha > 2.0:
                out[name + "_unbound"] = float(np.isinf(slack[name]).any(-1).mean())     # share of rows with no bound
        assert worst <= 1.0, f"{label}: {name} error is {worst:.3f} of what is allowed (scaled error {out[name]:.3e}, tol {tol})"
    return ref, out
