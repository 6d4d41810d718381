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


def check_forward(Q, K, V, alpha, causal, O, tau, mask, ref=None, label=""):
    """Compare a GPU forward result with the oracle. Returns the oracle result for reuse."""
    tol = TOL[Q.dtype]
    if ref is None:
        ref = eo.attn_fwd(to_np64(Q), to_np64(K), to_np64(V), alpha, causal, tile=64)
    dtau = np.abs(to_np64(tau) - ref["tau"]).max()
    dO = np.abs(to_np64(O) - ref["O"]).max()
    assert dtau <= tol["tau"], f"{label}: |dtau| = {dtau:.3e} > {tol['tau']}"
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


def check_backward(Q, K, V, dO, alpha, causal, dQ, dK, dV, ref=None, label="", exclude_rows=None):
    tol = TOL[Q.dtype]["grad"]
    if 1.5 < alpha < 2.0:
        # U = y^(r-1) with 0 < r-1 < 1 has an unbounded slope at the support edge:
        # dU = (r-1) y^(r-2) dy, so a score rounding dy is amplified for entries with small y.
        # No config of the workload uses such an alpha; the extra test allows 10x.
        tol *= 10
    if ref is None:
        ref = eo.attn_bwd(to_np64(Q), to_np64(K), to_np64(V), to_np64(dO), alpha, causal)
    out = {}
    for name, got in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        g = to_np64(got)
        err = np.abs(g - ref[name]) / (1.0 + np.abs(ref[name]))
        if exclude_rows is not None and name == "dQ":
            err = np.where(exclude_rows[..., None], 0.0, err)
        out[name] = float(err.max())
        assert err.max() <= tol, f"{label}: {name} scaled error {err.max():.3e} > {tol}"
    return ref, out


def near_threshold_rows(Q, K, alpha, causal, tau_ref, band=MASK_BAND):
    """Rows that have a score within `band` of their threshold: at alpha = 2 the factor U jumps
    from 0 to 1 there, so their gradient is not comparable at finite precision."""
    Qn, Kn = to_np64(Q), to_np64(K)
    d = Qn.shape[-1]
    X = (alpha - 1) * np.einsum("bhrc,bhjc->bhrj", Qn, Kn) / np.sqrt(d) - tau_ref[..., None]
    if causal:
        N = X.shape[-1]
        X = np.where(np.tril(np.ones((N, N), bool)), X, -np.inf)
    return (np.abs(X) < band).any(-1)
