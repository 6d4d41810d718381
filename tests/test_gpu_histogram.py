"""GPU checks of the histogram stage by itself (Eq. 6-9, App. C.3, Prop. 1) - the threshold parity
tests alone would not see a wrong bin, window move or closed-form root, because the safeguarded
refinement repairs a bad start - and metamorphic checks of the whole path that need no oracle."""
import numpy as np
import pytest
import torch

import workloads
from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ea():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2604_15180_amd as ea
    ea.lib()
    return ea


def grid_histogram_root(x, alpha, nb):
    """Float64 root of f_h (Eq. 9) for one row of pre-scaled scores x = (alpha-1) s, with the bins the
    GPU uses: width h = 1/nb on an absolute grid (bin a holds nb x in [a, a+1)), of which the nb + 1
    bins up to the one holding the maximum are kept.  Returns (tau_h, max x)."""
    h, r = 1.0 / nb, 1.0 / (alpha - 1.0)
    m = x.max()
    top = int(np.floor(nb * m))
    a = np.floor(nb * x).astype(np.int64)
    keep = a >= top - nb
    edges, counts = np.unique(a[keep], return_counts=True)
    e = edges.astype(np.float64) * h

    def f(tau):
        y = np.maximum(e - tau, 0.0)
        return float((counts * y ** r).sum() - 1.0)

    lo, hi = e.max() - 1.0 - 2 * h, e.max()        # f(lo) >= 0: the top bin alone weighs (1 + 2h)^r there; f(hi) = -1
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if f(mid) >= 0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi), m


CASES = [("bf16", 64, 1.5, "gauss", 2.0, True), ("bf16", 128, 1.5, "gauss", 1.0, True), ("bf16", 128, 2.0, "gauss", 3.0, False),
         ("bf16", 64, 1.25, "gauss", 2.0, True), ("f32", 64, 1.5, "gauss", 1.0, False), ("bf16", 64, 1.5, "ramp", 0.25, True),
         ("bf16", 64, 1.5, "ramp", 2.5, False), ("bf16", 64, 1.5, "flat", 0.3, True), ("f32", 64, 2.0, "flat", 0.3, True)]


@pytest.mark.parametrize("dtype,d,alpha,kind,scale,causal", CASES)
def test_histogram_root_brackets_the_threshold(ea, dtype, d, alpha, kind, scale, causal):
    # Prop. 1 on what the kernels' histogram stage produced: tau_0 <= tau* <= upper, upper - tau_0 <= 1/B
    # (+ rounding slack), and tau_0 equal to the float64 root of the same histogram.  Flat inputs
    # overflow the candidate lists of the long rows, which the sweep-based kernel then redoes.
    from oracle import entmax_oracle as eo
    B, H, N = 1, 2, (2048 if kind == "flat" else 640)
    print(f"histogram case {dtype} d={d} alpha={alpha} {kind} {scale} causal={causal}", flush=True)
    if kind == "ramp":
        q, k, v, _ = workloads.ramp_qkv(B, H, N, d, dtype, scale, seed=41)
    else:
        q, k, v, _ = workloads.gaussian_qkv(B, H, N, d, dtype, scale, seed=43)
    ws = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, False), dtype=torch.uint8, device="cuda")
    O, tau, mask, iters = ea.entmax_attn_fwd(q.cuda(), k.cuda(), v.cuda(), alpha, causal, want_iters=True, workspace=ws)
    tau0, upper = ea.entmax_attn_fwd_histogram_bounds(ws, B, H, N, d, dtype)
    torch.cuda.synchronize()
    if kind == "flat" and alpha == 1.5:
        assert ea.read_stats(ws)["list_overflow_blocks"] > 0
    nb = ea.entmax_attn_histogram_bins()
    ref = eo.attn_fwd(parity.to_np64(q), parity.to_np64(k), parity.to_np64(v), alpha, causal, want_margin=False)
    t0, up, tg = (parity.to_np64(t) for t in (tau0, upper, tau))
    ts = ref["tau"]
    eps = 3e-5 * (1.0 + np.abs(ts))            # fp32 scores and sums against float64
    assert (t0 <= ts + eps).all(), f"tau_0 above the true threshold by {(t0 - ts).max():.3e}"
    assert (ts <= up + eps).all(), f"true threshold above the bracket by {(ts - up).max():.3e}"
    assert (up - t0 <= 1.0 / nb + 1e-4).all(), f"bracket wider than 1/B: {(up - t0).max():.3e}"
    assert (tg >= t0 - eps).all() and (tg <= up + eps).all()
    # the root itself, against float64 on the same bins
    Qn, Kn = parity.to_np64(q), parity.to_np64(k)
    want = np.empty_like(ts)
    for h_ in range(H):
        X = (alpha - 1.0) * (Qn[0, h_] @ Kn[0, h_].T) / np.sqrt(d)
        for r_ in range(N):
            x = X[r_, : r_ + 1] if causal else X[r_]
            th, m = grid_histogram_root(x, alpha, nb)
            want[0, h_, r_] = max(th, m - 1.0)
    diff = np.abs(t0 - want)
    close = (diff <= 1e-4 * (1.0 + np.abs(want))).mean()
    print(f"  tau_0 within 1e-4 of the float64 root of the same bins on {100 * close:.2f} % of the rows; max {diff.max():.3e};"
          f" tau* - tau_0 mean {np.mean(ts - t0):.4f}; mean iters {iters.float().mean().item():.2f}", flush=True)
    # a score that fp32 puts on the other side of a bin edge moves one count by one bin
    assert close >= 0.995 and diff.max() <= 1.0 / nb + 1e-4


def test_shifting_every_key_by_one_vector(ea):
    # K <- K + 1 c^T adds q_r . c / sqrt(d) to every score of row r: P, O and every gradient stay,
    # tau_r moves by (alpha - 1) q_r . c / sqrt(d)   (fp32 path; shift invariance of Eq. 3)
    B, H, N, d, alpha = 1, 2, 512, 64, 1.5
    for causal in (False, True):
        q, k, v, do = workloads.gaussian_qkv(B, H, N, d, "f32", 1.0, seed=51)
        g = torch.Generator().manual_seed(52)
        c = 0.5 * torch.randn(d, generator=g)
        Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
        K2 = (k + c).cuda()
        O, tau, mask = ea.entmax_attn_fwd(Q, K, V, alpha, causal)
        O2, tau2, mask2 = ea.entmax_attn_fwd(Q, K2, V, alpha, causal)
        g1 = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask)
        g2 = ea.entmax_attn_bwd(Q, K2, V, O2, dO, tau2, alpha, causal, block_mask=mask2)
        torch.cuda.synchronize()
        shift = (alpha - 1.0) * (q.double() @ c.double()) / d ** 0.5
        assert (tau2.double().cpu() - tau.double().cpu() - shift).abs().max().item() <= 2e-5
        assert (O2 - O).abs().max().item() <= 2e-5
        assert (mask2 != mask).sum().item() <= 2          # (a tile whose largest probability is about 1e-6 may flip)
        for name, a, b in zip(("dQ", "dK", "dV"), g1, g2):
            err = ((a - b).abs() / (1 + a.abs())).max().item()
            assert err <= 5e-5, f"{name} moved by {err:.3e} (causal={causal})"


def test_permuting_key_tiles(ea):
    # not causal: whole 64-key tiles of K and V in another order leave O, tau and dQ as they are and
    # move the rows of dK, dV and the bits of the mask the same way
    B, H, N, d, alpha = 1, 2, 768, 64, 1.5
    T = N // 64
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, "f32", 1.5, seed=61)
    perm = torch.randperm(T, generator=torch.Generator().manual_seed(62))
    idx = (perm[:, None] * 64 + torch.arange(64)[None, :]).reshape(-1)        # new position p holds old key idx[p]
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    K2, V2 = k[:, :, idx].contiguous().cuda(), v[:, :, idx].contiguous().cuda()
    O, tau, mask = ea.entmax_attn_fwd(Q, K, V, alpha, False)
    O2, tau2, mask2 = ea.entmax_attn_fwd(Q, K2, V2, alpha, False)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, False, block_mask=mask)
    dQ2, dK2, dV2 = ea.entmax_attn_bwd(Q, K2, V2, O2, dO, tau2, alpha, False, block_mask=mask2)
    torch.cuda.synchronize()
    assert (tau2 - tau).abs().max().item() <= 1e-5 and (O2 - O).abs().max().item() <= 2e-5
    assert ((dQ2 - dQ).abs() / (1 + dQ.abs())).max().item() <= 5e-5
    idx_c = idx.cuda()
    assert ((dK2 - dK[:, :, idx_c]).abs() / (1 + dK2.abs())).max().item() <= 5e-5
    assert ((dV2 - dV[:, :, idx_c]).abs() / (1 + dV2.abs())).max().item() <= 5e-5
    bits, bits2 = parity.unpack_mask(mask, T), parity.unpack_mask(mask2, T)
    assert (bits2 != bits[..., perm.numpy()]).sum() <= 2


@pytest.mark.parametrize("dtype,d,alpha,sigma,causal,N", [("bf16", 128, 1.5, 2.0, True, 1024), ("bf16", 64, 2.0, 2.0, False, 640),
                                                       ("f32", 64, 1.25, 1.0, True, 320), ("bf16", 64, 3.0, 2.0, True, 640),
                                                       ("bf16", 64, 1.5, 0.3, True, 2048), ("bf16", 128, 1.5, 4.0, True, 1024)])
def test_right_edge_binning_gives_a_sparser_approximation(ea, dtype, d, alpha, sigma, causal, N):
    # The approximate forward (Sec. 3.2, binning strategies): thresholds are the right-edge histogram
    # roots, unrefined.  Asserted: what defines the mode - tau* <= tau < tau* + h + slack against the
    # oracle's tau*, one evaluation per row, rows of P summing to at most 1, and O = P(tau) V for
    # the tau returned (float64, from the same inputs).  Its distance from the exact result is
    # printed, not asserted: the mode is not meant to reach it.  sigma = 0.3 overflows the candidate
    # lists (the sweep-based kernel), sigma = 4 takes the gather path.
    from oracle import entmax_oracle as eo
    B, H = 1, 2
    print(f"right-edge case N={N} d={d} {dtype} alpha={alpha} sigma={sigma} causal={causal}", flush=True)
    q, k, v, _ = workloads.gaussian_qkv(B, H, N, d, dtype, sigma, seed=77)
    Q, K, V = (t.cuda() for t in (q, k, v))
    ea.entmax_attn_right_edge_enable(True)
    try:
        O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True)
        torch.cuda.synchronize()
    finally:
        ea.entmax_attn_right_edge_enable(False)
    O2, tau2, mask2 = ea.entmax_attn_fwd(Q, K, V, alpha, causal)          # and the switch is off again
    torch.cuda.synchronize()
    ref = eo.attn_fwd(*(parity.to_np64(t) for t in (q, k, v)), alpha, causal, tile=64)
    parity.check_forward(q, k, v, alpha, causal, O2, tau2, mask2, ref=ref, label="exact mode after the approximate one")
    h = 1.0 / ea.entmax_attn_histogram_bins()
    t, ts = parity.to_np64(tau), ref["tau"]
    slack = 2e-6 * (1 + np.abs(ts))
    assert (t >= ts - slack).all() and (t <= ts + h + 2 * slack).all(), ((t - ts).min(), (t - ts).max())
    assert (iters.cpu().numpy() == 1).all()
    Qn, Kn, Vn = (parity.to_np64(x) for x in (q, k, v))
    r = 1.0 / (alpha - 1.0)
    worst_o, sums = 0.0, []
    for hh in range(H):
        X = (alpha - 1.0) * Qn[0, hh] @ Kn[0, hh].T / np.sqrt(d)
        if causal:
            X = np.where(np.tril(np.ones((N, N), bool)), X, -np.inf)
        P = np.maximum(X - t[0, hh][:, None], 0.0) ** r
        sums.append(P.sum(-1))
        worst_o = max(worst_o, np.abs(P @ Vn[0, hh] - parity.to_np64(O)[0, hh]).max())
    sums = np.concatenate(sums)
    assert sums.max() <= 1 + 1e-3
    assert worst_o <= parity.TOL[q.dtype]["O"], worst_o
    # block mask: every tile it marks is marked in the exact result (support inside the true one)
    T = N // 64
    got, exact = parity.unpack_mask(mask, T), parity.unpack_mask(mask2, T)
    assert not (got & ~exact).any()
    print("  right edge:", dict(tau_above=float((t - ts).mean()), row_sum_mean=float(sums.mean()), row_sum_min=float(sums.min()),
                               dO_vs_exact=float(np.abs(parity.to_np64(O) - ref["O"]).max()),
                               tiles=int(got.sum()), tiles_exact=int(exact.sum())), flush=True)
