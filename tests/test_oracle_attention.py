"""Pins of the oracle's attention forward and gradient (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import entmax_oracle as eo

RNG = np.random.default_rng(99)


def rand(*shape, scale=1.0):
    return RNG.normal(size=shape) * scale


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0, 2.5])
@pytest.mark.parametrize("causal", [False, True])
def test_forward_is_rowwise_entmax_times_v(alpha, causal):
    B, H, N, d = 2, 2, 24, 5
    Q, K, V = rand(B, H, N, d, scale=2), rand(B, H, N, d, scale=2), rand(B, H, N, d)
    out = eo.attn_fwd(Q, K, V, alpha, causal, tile=8, want_P=True)
    S = np.einsum("bhrc,bhjc->bhrj", Q, K) / np.sqrt(d)       # Eq. 2
    for b in range(B):
        for h in range(H):
            for r in range(N):
                nv = r + 1 if causal else N
                p, tau = eo.entmax(S[b, h, r, :nv], alpha)
                assert np.abs(out["P"][b, h, r, :nv] - p).max() < 1e-12
                assert np.all(out["P"][b, h, r, nv:] == 0)
                assert abs(out["tau"][b, h, r] - tau) < 1e-12
    assert np.abs(out["O"] - out["P"] @ V).max() < 1e-12
    assert np.abs(out["P"].sum(-1) - 1).max() < 1e-10
    # margins: definition, from P's own support and the raw scores
    X = (alpha - 1) * S - out["tau"][..., None]
    if causal:
        X = np.where(np.tril(np.ones((N, N), bool)), X, -np.inf)
    Mg = X.reshape(B, H, N // 8, 8, N // 8, 8).max(axis=(3, 5))
    assert np.array_equal(np.isinf(Mg), np.isinf(out["margin"]))
    fin = np.isfinite(Mg)
    assert np.abs(Mg[fin] - out["margin"][fin]).max() < 1e-12
    blk = out["P"].reshape(B, H, N // 8, 8, N // 8, 8).max(axis=(3, 5)) > 0
    assert np.array_equal(blk, out["margin"] > 0)


def test_forward_identity_values_and_first_causal_row():
    # V = I (d = N): O is P itself; causal row 0 sees one key: p = 1, tau = (alpha-1) s - 1
    N = 12
    Q, K = rand(1, 1, N, N), rand(1, 1, N, N)
    V = np.eye(N)[None, None]
    for alpha in (1.5, 2.0, 1.3):
        out = eo.attn_fwd(Q, K, V, alpha, True, tile=4, want_P=True)
        assert np.abs(out["O"] - out["P"]).max() < 1e-15
        s00 = Q[0, 0, 0] @ K[0, 0, 0] / np.sqrt(N)
        assert abs(out["tau"][0, 0, 0] - ((alpha - 1) * s00 - 1)) < 1e-12
        assert abs(out["O"][0, 0, 0, 0] - 1) < 1e-12


def test_forward_softmax_limit():
    B, H, N, d = 1, 1, 10, 4
    Q, K, V = rand(B, H, N, d), rand(B, H, N, d), rand(B, H, N, d)
    S = torch.from_numpy(np.einsum("bhrc,bhjc->bhrj", Q, K) / np.sqrt(d))
    ref = (torch.softmax(S, -1) @ torch.from_numpy(V)).numpy()
    errs = [np.abs(eo.attn_fwd(Q, K, V, a, False, want_margin=False)["O"] - ref).max() for a in (1.1, 1.01, 1.001)]
    assert errs[0] > errs[1] > errs[2] and errs[2] < 2e-3


def loss(Q, K, V, dO, alpha, causal):
    return float((eo.attn_fwd(Q, K, V, alpha, causal, want_margin=False)["O"] * dO).sum())


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0, 2.5, 3.0])
@pytest.mark.parametrize("causal", [False, True])
def test_gradient_matches_finite_differences(alpha, causal):
    B, H, N, d = 1, 2, 9, 4
    Q, K, V, dO = rand(B, H, N, d, scale=1.5), rand(B, H, N, d, scale=1.5), rand(B, H, N, d), rand(B, H, N, d)
    g = eo.attn_bwd(Q, K, V, dO, alpha, causal)
    # the sort-based thresholds are exact; the bisection leaves ~1e-12 of noise in tau, which a
    # difference quotient amplifies by 1/eps, so general alpha uses a wider stencil
    eps, tol = (1e-6, 5e-7) if alpha in (1.5, 2.0) else (1e-4, 2e-6)
    worst = 0.0
    for name, X in (("dQ", Q), ("dK", K), ("dV", V)):
        num = np.zeros_like(X)
        it = np.nditer(X, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = X[idx]
            X[idx] = old + eps; lp = loss(Q, K, V, dO, alpha, causal)
            X[idx] = old - eps; lm = loss(Q, K, V, dO, alpha, causal)
            X[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        err = np.abs(num - g[name]).max()
        worst = max(worst, err)
        # piecewise-smooth map: away from support changes central differences agree to O(eps^2)
        assert err < tol, (name, err)


def torch_entmax_attention(Q, K, V, alpha, causal):
    """Differentiable construction independent of the oracle's backward formula: tau from a
    sort (alpha in {1.5, 2}), autograd differentiates through the sort-based closed form."""
    d = Q.shape[-1]
    S = Q @ K.transpose(-1, -2) / d ** 0.5
    N = S.shape[-1]
    if causal:
        S = S.masked_fill(~torch.tril(torch.ones(N, N, dtype=torch.bool)), -1e30)
    X = (alpha - 1) * S
    Xs, _ = torch.sort(X, dim=-1, descending=True)
    k = torch.arange(1, N + 1, dtype=X.dtype)
    if alpha == 2.0:
        t = (Xs.cumsum(-1) - 1) / k
    else:
        mean = Xs.cumsum(-1) / k
        mean_sq = (Xs ** 2).cumsum(-1) / k
        disc = torch.clamp(mean ** 2 - (mean_sq - 1 / k), min=0)
        t = mean - torch.sqrt(disc)
    supp = (Xs > t).sum(-1, keepdim=True)
    tau = t.gather(-1, supp - 1)
    Y = torch.clamp(X - tau, min=0)
    P = Y if alpha == 2.0 else Y ** 2
    return P @ V, tau.squeeze(-1)


@pytest.mark.parametrize("alpha", [1.5, 2.0])
@pytest.mark.parametrize("causal", [False, True])
def test_gradient_matches_autograd_through_sort(alpha, causal):
    B, H, N, d = 2, 2, 33, 8
    Qn, Kn, Vn, dOn = rand(B, H, N, d, scale=1.5), rand(B, H, N, d, scale=1.5), rand(B, H, N, d), rand(B, H, N, d)
    Q, K, V = (torch.tensor(a, requires_grad=True) for a in (Qn, Kn, Vn))
    O, tau = torch_entmax_attention(Q, K, V, alpha, causal)
    (O * torch.from_numpy(dOn)).sum().backward()
    fw = eo.attn_fwd(Qn, Kn, Vn, alpha, causal, want_margin=False)
    assert np.abs(fw["O"] - O.detach().numpy()).max() < 1e-12
    assert np.abs(fw["tau"] - tau.detach().numpy()).max() < 1e-12
    g = eo.attn_bwd(Qn, Kn, Vn, dOn, alpha, causal)
    for name, t in (("dQ", Q), ("dK", K), ("dV", V)):
        assert np.abs(g[name] - t.grad.numpy()).max() < 1e-11, name


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0, 2.5, 3.0])
def test_gradient_invariants(alpha):
    B, H, N, d = 1, 1, 40, 6
    Q, K, V, dO = rand(B, H, N, d, scale=2), rand(B, H, N, d, scale=2), rand(B, H, N, d), rand(B, H, N, d)
    g = eo.attn_bwd(Q, K, V, dO, alpha, True)
    # rows of P sum to one -> sum_j dV_j = sum_r dO_r
    assert np.abs(g["dV"].sum(2) - dO.sum(2)).max() < 1e-10
    # shifting all scores of a row changes nothing: K -> K + 1 c^T gives the same loss, so
    # sum_j dK_j must vanish (dS rows sum to zero)
    assert np.abs(g["dK"].sum(2)).max() < 1e-10
    # gradients vanish off the support (Sec. 3.3): a key nobody attends to gets dK = dV = 0
    P = eo.attn_fwd(Q, K, V, alpha, True, want_margin=False, want_P=True)["P"]
    unused = P[0, 0].max(0) == 0
    assert unused.any()
    assert np.all(g["dK"][0, 0, unused] == 0) and np.all(g["dV"][0, 0, unused] == 0)


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0, 3.0])
def test_decode_is_the_last_causal_row(alpha):
    # the inference variant (one query against all cached keys) must equal what the attention
    # oracle, a separate C routine, gives for the last row of a causal problem, whose query sees
    # every key; and its probabilities must solve Eq. 3-4
    rng = np.random.default_rng(5)
    B, H, N, d = 1, 2, 96, 16
    Q, K, V = (1.5 * rng.standard_normal((B, H, N, d)) for _ in range(3))
    full = eo.attn_fwd(Q, K, V, alpha, True, tile=32, want_margin=False)
    dec = eo.attn_decode(Q[:, :, -1], K, V, alpha)
    assert np.abs(dec["O"] - full["O"][:, :, -1]).max() < 1e-12
    assert np.abs(dec["tau"] - full["tau"][:, :, -1]).max() < 1e-12
    assert np.abs(dec["P"].sum(-1) - 1).max() < 1e-10 and dec["P"].min() >= 0   # (bisection stops at a 1e-12 bracket in tau)
    x = (alpha - 1) * dec["z"] - dec["tau"][..., None]
    assert np.abs(dec["P"] - np.maximum(x, 0) ** (1 / (alpha - 1))).max() < 1e-12


def test_decode_one_dominant_key_and_equal_keys():
    # a key far ahead of the rest: one-hot, o = its value row, tau = (alpha-1) z_max - 1 (lower
    # end of Eq. 5); all keys equal: uniform, o = mean of V, tau = (alpha-1) z - n^(1-alpha)
    rng = np.random.default_rng(6)
    N, d, alpha = 40, 8, 1.5
    q = np.ones((1, 1, d)); K = np.zeros((1, 1, N, d)); K[0, 0, 7] = 10.0
    V = rng.standard_normal((1, 1, N, d))
    dec = eo.attn_decode(q, K, V, alpha)
    assert np.abs(dec["O"][0, 0] - V[0, 0, 7]).max() < 1e-12
    assert abs(dec["tau"][0, 0] - ((alpha - 1) * 10.0 * d / np.sqrt(d) - 1)) < 1e-12
    K[:] = 0.3
    dec = eo.attn_decode(q, K, V, alpha)
    assert np.abs(dec["O"][0, 0] - V[0, 0].mean(0)).max() < 1e-12
    assert abs(dec["tau"][0, 0] - ((alpha - 1) * 0.3 * d / np.sqrt(d) - N ** (1 - alpha))) < 1e-12


@pytest.mark.parametrize("alpha,dtype", [(1.75, torch.bfloat16), (2.0, torch.bfloat16), (1.5, torch.float32), (1.25, torch.float32),
                                         (2.5, torch.bfloat16), (3.0, torch.float32)])
def test_conditioning_slack_bounds_a_shift_of_the_thresholds(alpha, dtype):
    # the slack the GPU gradient comparison adds for alpha > 1.5 and for fp32 inputs is a bound of
    # what a perturbation of y = (alpha-1) s - tau within eta changes: shift every row's threshold by
    # +-eta_min (a perturbation inside that budget) in a plain numpy backward and compare
    from tests import parity
    B, H, N, d, causal = 1, 1, 96, 16, True
    g = torch.Generator().manual_seed(5)
    q, k, v, do = (torch.randn(B, H, N, d, generator=g).to(dtype) for _ in range(4))
    Q, K, V, G = (parity.to_np64(t)[0, 0] for t in (q, k, v, do))
    tau = eo.attn_fwd(Q[None, None], K[None, None], V[None, None], alpha, causal, want_margin=False)["tau"]
    slack = parity.conditioning_slack(q, k, v, do, alpha, causal, tau)
    r = 1.0 / (alpha - 1.0)
    X = (alpha - 1.0) * Q @ K.T / np.sqrt(d)
    vis = np.tril(np.ones((N, N), bool))

    def grads(shift):
        y = np.where(vis, X - tau[0, 0][:, None] - shift[:, None], -1.0)
        yp = np.maximum(y, 0)
        P = yp ** r
        with np.errstate(divide="ignore"):
            U = np.where(y > 0, yp ** (r - 1.0), 0.0) if alpha != 2.0 else (y > 0).astype(float)
        gg = G @ V.T
        delta = (U * gg).sum(-1) / U.sum(-1)
        dS = U * (gg - delta[:, None])
        return dS @ K / np.sqrt(d), dS.T @ Q / np.sqrt(d), P.T @ G

    base = grads(np.zeros(N))
    ref = eo.attn_bwd(Q[None, None], K[None, None], V[None, None], G[None, None], alpha, causal)
    for name, b in zip(("dQ", "dK", "dV"), base):
        assert np.abs(b - ref[name][0, 0]).max() < 1e-9          # the numpy backward is the oracle's
    tol_solver = 1e-4 if dtype == torch.bfloat16 else 1e-6
    eta_min = 1e-3 if alpha == 2.0 else 2 * tol_solver
    rng = np.random.default_rng(3)
    for trial in range(4):
        shift = eta_min * rng.uniform(-1, 1, N)
        for name, b, s_ in zip(("dQ", "dK", "dV"), base, grads(shift)):
            assert (np.abs(s_ - b) <= slack[name][0, 0] + 1e-12).all(), name
    assert all((slack[n_] >= 0).all() for n_ in slack)
    if alpha > 2.0:
        # rows with a score within eta of their threshold are not bound at all; most rows are
        unbound = np.isinf(slack["dQ"][0, 0]).any(-1)
        assert unbound.mean() < 0.5 and (unbound.any() or dtype == torch.float32)


@pytest.mark.parametrize("alpha,dtype", [(2.5, torch.float32), (3.0, torch.bfloat16)])
def test_output_slack_bounds_a_shift_of_the_thresholds(alpha, dtype):
    # the slack the GPU comparison adds to O's tolerance for alpha > 2: shift every row's threshold
    # by up to +-2 tol_solver (inside the budget) in a plain numpy forward and compare
    from tests import parity
    B, H, N, d, causal = 1, 1, 96, 16, True
    g = torch.Generator().manual_seed(8)
    q, k, v = (torch.randn(B, H, N, d, generator=g).to(dtype) for _ in range(3))
    Q, K, V = (parity.to_np64(t)[0, 0] for t in (q, k, v))
    out = eo.attn_fwd(Q[None, None], K[None, None], V[None, None], alpha, causal, want_margin=False)
    slack = parity.output_slack(q, k, v, alpha, causal, out["tau"])[0, 0]
    r = 1.0 / (alpha - 1.0)
    X = (alpha - 1.0) * Q @ K.T / np.sqrt(d)
    vis = np.tril(np.ones((N, N), bool))

    def fwd(shift):
        y = np.where(vis, X - out["tau"][0, 0][:, None] - shift[:, None], -1.0)
        return (np.maximum(y, 0) ** r) @ V

    base = fwd(np.zeros(N))
    assert np.abs(base - out["O"][0, 0]).max() < 1e-10
    eta_min = 2 * (1e-4 if dtype == torch.bfloat16 else 1e-6)
    rng = np.random.default_rng(4)
    for trial in range(4):
        moved = fwd(eta_min * rng.uniform(-1, 1, N))
        assert (np.abs(moved - base) <= slack + 1e-13).all()
    # and the slack is what makes the difference: the plain tolerance alone would not hold
    assert slack.max() > parity.TOL[dtype]["O"] * 0.1
