"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle on the same
seeded inputs, element by element."""
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
    ea.lib()   # raises if the HIP library is not built: there is no fallback
    return ea


def run_case(ea, B, H, N, d, dtype, causal, alpha, sigma, seed, block_rho=0.0, backward=True, mask_arg=True):
    print(f"case B={B} H={H} N={N} d={d} {dtype} causal={causal} alpha={alpha} sigma={sigma} seed={seed}", flush=True)
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, dtype, sigma, seed, block_rho=block_rho)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True)
    torch.cuda.synchronize()
    label = f"N={N} d={d} {dtype} a={alpha} c={causal}"
    ref, info = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label=label)
    it = iters.cpu().numpy()
    # (alpha > 2: rows that end up bisecting, see test_alpha_above_two; twice the sweeps over the lists)
    assert it.min() >= 1 and it.max() <= (12 if alpha <= 2 else 36)
    print("  fwd", info, "mean iters", it.mean(), "max", it.max(), flush=True)
    if backward:
        dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask if mask_arg else None)
        torch.cuda.synchronize()
        gref, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, label=label, tau_ref=ref["tau"])
        print("  bwd", ginfo, flush=True)
        if alpha > 2:
            # the backward as an operation of its own: from the oracle's thresholds and output (rounded
            # to fp32), which takes the solver's tolerance out of what the comparison has to allow
            tau_o = torch.from_numpy(ref["tau"]).float().cuda()
            O_o = torch.from_numpy(ref["O"]).float().cuda()
            dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O_o, dO, tau_o, alpha, causal, block_mask=None)
            torch.cuda.synchronize()
            _, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, ref=gref, label=label + " tau given",
                                             tau_ref=ref["tau"], tau_given=True)
            print("  bwd from the oracle's tau", ginfo, flush=True)
    return info


def test_c1_fp32_exact_config(ea):
    # configs[0]: alpha=1.5, fp32, B=1, H=2, N=256, d=64, non-causal, N(0,1)
    run_case(ea, 1, 2, 256, 64, "f32", False, 1.5, 1.0, seed=1000)


@pytest.mark.parametrize("N,causal", [(64, True), (192, True), (320, False)])
def test_fp32_ragged_sizes(ea, N, causal):
    # N not a multiple of the 128-row work-group tile; N = 64 is a single tile
    run_case(ea, 1, 2, N, 64, "f32", causal, 1.5, 1.0, seed=7 + N)


@pytest.mark.parametrize("alpha", [1.25, 2.0, 1.75])
def test_fp32_alpha_sweep(ea, alpha):
    # sigma = 1 as in configs[0]: fp32 cannot hold 1e-5 absolute on O once |(alpha-1) s| grows
    # past a few units (alpha = 2 passes score rounding straight into P)
    run_case(ea, 1, 2, 256, 64, "f32", True, alpha, 1.0, seed=11)


@pytest.mark.parametrize("N,d,causal", [(2560, 128, False), (6144, 64, True)])
def test_fp32_rows_with_large_supports(ea, N, d, causal):
    # fp32 inputs at alpha = 2, sigma = 1, beyond the size of configs[0]: a row attends to dozens of
    # keys, P = y passes the rounding of every fp32 score (d products, a few 1e-7 times |s|) straight
    # into O, and the sum over the support reaches the 1e-5 bar by itself (a randomized sweep met
    # 1.0e-5 .. 1.3e-5 on such inputs, on both output paths).  O is held to 1e-5 plus the bound that
    # follows from that rounding and the solver's 1e-6 (parity.output_slack); tau, the mask and the
    # gradients to their usual bars.
    alpha = 2.0
    print(f"case fp32 large supports N={N} d={d} causal={causal}", flush=True)
    q, k, v, do = workloads.gaussian_qkv(1, 1, N, d, "f32", 1.0, seed=4400 + N)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask)
    torch.cuda.synchronize()
    ref, info = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label="fp32 large supports", rounding_slack=True)
    slack = parity.output_slack(q, k, v, alpha, causal, ref["tau"])
    support = ((alpha - 1.0) * (parity.to_np64(q)[0, 0] @ parity.to_np64(k)[0, 0].T) / np.sqrt(d) > ref["tau"][0, 0][:, None])
    if causal:
        support &= np.tril(np.ones((N, N), bool))
    print("  fwd", info, "largest slack", slack.max(), "mean support", support.sum(1).mean(), "max iters", iters.max().item(), flush=True)
    # the bound stays of the order of the bar it is added to
    assert slack.max() <= 1e-4 and info["dO"] <= 3e-5
    _, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, label="fp32 large supports", tau_ref=ref["tau"])
    print("  bwd", ginfo, flush=True)


def test_fp32_head_dim_128(ea):
    run_case(ea, 1, 1, 192, 128, "f32", True, 1.5, 1.0, seed=5)


@pytest.mark.parametrize("d,N,sigma", [(64, 512, 1.5), (128, 448, 2.0), (128, 1024, 1.0)])
def test_bf16_causal(ea, d, N, sigma):
    run_case(ea, 2, 2, N, d, "bf16", True, 1.5, sigma, seed=21)


@pytest.mark.parametrize("N,causal,alpha,d", [(64, True, 1.5, 128), (192, True, 2.0, 64), (320, False, 1.5, 64),
                                              (576, True, 2.0, 128)])
def test_bf16_ragged_sizes(ea, N, causal, alpha, d):
    # N not a multiple of the 256-row group of the threshold kernel for 16-bit inputs at alpha 1.5
    # and 2: its last group runs with some of its eight waves (and of the wave pairs that share
    # histogram words) idle; N = 64 is a single key tile
    run_case(ea, 1, 2, N, d, "bf16", causal, alpha, 2.0, seed=300 + N)


def test_bf16_noncausal(ea):
    run_case(ea, 1, 2, 384, 128, "bf16", False, 1.5, 1.5, seed=22)


@pytest.mark.parametrize("alpha", [1.25, 2.0])
def test_bf16_alpha_sweep(ea, alpha):
    # configs[4] shape at a size the oracle finishes quickly
    run_case(ea, 1, 2, 512, 64, "bf16", True, alpha, 2.0, seed=23)


@pytest.mark.parametrize("dtype,alpha,N,d,causal,sigma", [("f32", 2.5, 256, 64, True, 1.0), ("f32", 3.0, 320, 128, False, 1.0),
                                                          ("bf16", 2.5, 512, 64, True, 2.0), ("bf16", 3.0, 1024, 128, False, 1.5),
                                                          ("bf16", 3.0, 2048, 64, True, 0.3), ("bf16", 2.25, 1024, 128, True, 4.0)])
def test_alpha_above_two(ea, dtype, alpha, N, d, causal, sigma):
    # secant steps (Sec. 3.2) on the candidate lists; sigma = 0.3 overflows the lists, so the dense
    # kernel takes the first evaluation and the output kernel the rest; sigma = 4 leaves a handful
    # of keys per row (the gather kernels).  A row with a score within the tolerance of its root
    # bisects (f rises vertically at every score), up to 24 sweeps over the lists and 12 more in the
    # output kernel.  U = P^(2-alpha) is unbounded at the support's edge: the gradient bound of
    # parity.conditioning_slack applies, and does not bind rows with a score within its eta of the
    # threshold; the share of such rows is printed, and falls to a few per mille when the backward
    # is handed the oracle's thresholds
    run_case(ea, 1, 2, N, d, dtype, causal, alpha, sigma, seed=400 + N)


def test_bf16_block_sparse_inputs(ea):
    # block-correlated queries: many all-zero 64x64 tiles, exercises the skip paths
    info = run_case(ea, 1, 2, 1024, 64, "bf16", True, 1.5, 3.0, seed=24, block_rho=0.98)


def test_backward_rebuilds_mask_when_absent(ea):
    run_case(ea, 1, 2, 320, 64, "bf16", True, 1.5, 2.0, seed=25, mask_arg=False)


def test_degenerate_rows(ea):
    # all-equal scores (Q = 0): uniform attention over the visible keys, tau = -(n_vis)^(1-alpha)
    B, H, N, d = 1, 1, 128, 64
    g = torch.Generator().manual_seed(3)
    Q = torch.zeros(B, H, N, d).cuda()
    K = torch.randn(B, H, N, d, generator=g).cuda()
    V = torch.randn(B, H, N, d, generator=g).cuda()
    O, tau, mask = ea.entmax_attn_fwd(Q, K, V, 1.5, True)
    torch.cuda.synchronize()
    nvis = np.arange(1, N + 1, dtype=np.float64)
    assert np.abs(tau.cpu().numpy()[0, 0] - (-nvis ** -0.5)).max() < 1e-5
    ref = torch.cumsum(V.double().cpu(), 2) / torch.arange(1, N + 1).view(1, 1, N, 1)
    assert (O.double().cpu() - ref).abs().max() < 1e-5
    # one dominant key per row: one-hot rows, O_r = V_0
    Q = torch.ones(B, H, N, d).cuda()
    K = torch.zeros(B, H, N, d); K[:, :, 0] = 100.0; K = K.cuda()
    O, tau, mask = ea.entmax_attn_fwd(Q, K, V, 2.0, True)
    torch.cuda.synchronize()
    assert (O.cpu() - V.cpu()[:, :, :1]).abs().max() < 1e-5
    m = parity.unpack_mask(mask, N // 64)
    assert m[0, 0].tolist() == [[True, False], [True, False]]


@pytest.mark.parametrize("dtype,rise,causal", [("f32", 0.1, False), ("f32", 0.1, True), ("bf16", 0.25, True),
                                               ("bf16", 2.5, False), ("bf16", 2.5, True), ("bf16", -0.5, False)])
def test_drifting_row_maximum(ea, dtype, rise, causal):
    # the row maximum climbs by a fraction of the histogram window per key tile (0.1, 0.25), by
    # more than the whole window (2.5), or sits at the first keys (-0.5); the fp32 cases keep
    # |(alpha-1) s| near 1, where fp32 scores can hold the 1e-5 bar
    N, d = 640, 64
    print(f"case ramp {dtype} rise={rise} causal={causal}", flush=True)
    q, k, v, do = workloads.ramp_qkv(1, 2, N, d, dtype, rise, seed=31)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, 1.5, causal, want_iters=True)
    torch.cuda.synchronize()
    _, info = parity.check_forward(q, k, v, 1.5, causal, O, tau, mask, label="ramp")
    print("  ramp", info, "mean iters", iters.float().mean().item(), flush=True)
    # the backward in every case: all queries share one direction here and |K| reaches 50 along it,
    # so dQ is what is left after large terms cancel and dK sums hundreds of like-signed rows -
    # which second-stage operands of 11 significant bits did not hold to 1e-2 (they are cut in two
    # fp16 halves since)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, 1.5, causal, block_mask=mask)
    torch.cuda.synchronize()
    _, ginfo = parity.check_backward(q, k, v, do, 1.5, causal, dQ, dK, dV, label="ramp")
    print("  ramp bwd", ginfo, flush=True)
    assert iters.max().item() <= 12


@pytest.mark.parametrize("dtype,N", [("bf16", 2048), ("f32", 1024)])
def test_flat_attention_overflows_candidate_lists(ea, dtype, N):
    # tiny scores: every key lies within one unit of the row maximum, so rows with more visible
    # keys than their candidate lists hold are flagged and redone by the sweep-based threshold
    # kernel, while the short first rows of the same head stay on the list path
    B, H, d, alpha, causal = 1, 2, 64, 1.5, True
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, dtype, 0.3, seed=61)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    ws = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, False), dtype=torch.uint8, device="cuda")
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True, workspace=ws)
    torch.cuda.synchronize()
    st = ea.read_stats(ws)
    print("  flat attention:", {k_: st[k_] for k_ in ("list_overflow_blocks", "tau_subtiles")}, flush=True)
    assert 0 < st["list_overflow_blocks"] < B * H * (N // 64)
    _, info = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label="flat")
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask)
    torch.cuda.synchronize()
    _, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, label="flat")
    print("  flat", info, ginfo, "mean iters", iters.float().mean().item(), flush=True)


@pytest.mark.parametrize("dtype,d,alpha,sigma,want", [("bf16", 128, 1.5, 3.0, "all"), ("bf16", 64, 2.0, 3.0, "all"),
                                                        ("f32", 64, 1.5, 2.0, "any"), ("bf16", 64, 1.25, 2.5, "any"), ("bf16", 128, 1.5, 0.3, "none"),
                                                        ("bf16", 64, 1.5, 1.6, "any")])
def test_sparse_row_groups_gather_their_output(ea, dtype, d, alpha, sigma, want):
    # peaked attention: a handful of keys per row, whose rows of V the gather kernel sums instead
    # of the block-sparse matrix products; flat attention (tiny scores: every key in the support): no row group qualifies;
    # in between both output paths may serve parts of one head.  Checked against the oracle alike.
    B, H, N, causal = 1, 2, 1280, True
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, dtype, sigma, seed=83)
    Q, K, V = (t.cuda() for t in (q, k, v))
    ws = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, False), dtype=torch.uint8, device="cuda")
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True, workspace=ws)
    torch.cuda.synchronize()
    st = ea.read_stats(ws)
    print("  gather rows", st["gather_rows"], "of", B * H * N, "out sub-tiles", st["out_subtiles"], flush=True)
    if want == "all":
        assert st["gather_rows"] == B * H * N and st["out_subtiles"] == 0
    elif want == "none":
        assert st["gather_rows"] == 0
    _, info = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label=f"gather {dtype} {alpha} {sigma}")
    assert int(iters.min()) >= 1
    print("  ", info, "mean iters", iters.float().mean().item(), flush=True)


@pytest.mark.parametrize("dtype,d,alpha,sigma,mask_arg,fwd_lists", [("bf16", 128, 1.5, 3.0, True, False), ("bf16", 64, 2.0, 3.0, True, False),
                                                                     ("f32", 64, 1.5, 1.0, True, False), ("bf16", 128, 1.25, 4.0, True, False),
                                                                     ("bf16", 128, 1.5, 3.0, False, False), ("bf16", 128, 1.5, 3.0, True, True),
                                                                     ("bf16", 64, 2.0, 2.0, True, True), ("bf16", 128, 1.25, 4.0, True, True)])
def test_sparse_row_groups_gather_their_gradients(ea, dtype, d, alpha, sigma, mask_arg, fwd_lists):
    # peaked attention: the backward lists each row's support and forms dQ row by row and dK, dV
    # key by key instead of through the matrix kernels; with and without the caller's mask.
    # (Not causal, 48 key tiles: the gather path is only taken when the mask marks enough tiles
    # per 64-row block for the matrix kernels to cost more than a few passes over dK, dV.)
    B, H, N, causal = 1, 2, 3072, False
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, dtype, sigma, seed=91)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    # fwd_lists: the backward is handed the forward's workspace and takes the supports from the
    # forward's lists instead of finding them again (no list sweep)
    wf = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, False), dtype=torch.uint8, device="cuda")
    O, tau, mask, _ = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True, workspace=wf)
    ws = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, True), dtype=torch.uint8, device="cuda")
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask if mask_arg else None, workspace=ws,
                                    fwd_workspace=wf if fwd_lists else None)
    torch.cuda.synchronize()
    st = ea.read_stats(ws)
    print("  backward gather rows", st["bwd_gather_rows"], "of", B * H * N, "dq sub-tiles", st["dq_subtiles"],
          "list sweep sub-tiles", st["bwd_list_subtiles"], flush=True)
    if fwd_lists:
        assert st["bwd_list_subtiles"] == 0 and st["bwd_gather_rows"] > 0
        # the lists are left as they were found: a second backward from them gives the same dQ
        dQ2, _, _ = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=ws, fwd_workspace=wf)
        torch.cuda.synchronize()
        assert torch.equal(dQ, dQ2)
    # (fp32 inputs: at the score scale where fp32 scores allow the 1e-5 bar no row group is sparse
    # enough; the fp32 gather path at a larger scale is checked against the matrix path in
    # test_gather_and_matrix_paths_agree)
    assert st["bwd_gather_rows"] > 0 or dtype == "f32"
    ref, _ = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label=f"fwd {dtype} {alpha}")
    _, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, label=f"bwd gather {dtype} {alpha}", tau_ref=ref["tau"])
    print("  ", ginfo, flush=True)


@pytest.mark.parametrize("dtype,d,sigma", [("bf16", 128, 3.0), ("f32", 128, 2.5)])
def test_gather_and_matrix_paths_agree(ea, dtype, d, sigma):
    # the same call with the gather paths switched off: every row group on the matrix kernels.
    # Each path is within `allowed` of the oracle - the tolerance plus what the accuracy of
    # y = (alpha-1) s - tau itself leaves open (parity.output_slack, parity.conditioning_slack; for
    # fp32 inputs at this score scale that is about 1e-4, ten times the plain bar) - so the two may
    # differ by twice that, element by element, and no more
    from oracle import entmax_oracle as eo
    B, H, N, alpha, causal = 1, 2, 3072, 1.5, False
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, dtype, sigma, seed=93)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    res = {}
    try:
        for on in (True, False):
            ea.entmax_attn_gather_enable(on)
            wf = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, False), dtype=torch.uint8, device="cuda")
            wb = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, True), dtype=torch.uint8, device="cuda")
            O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True, workspace=wf)
            dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=wb)
            torch.cuda.synchronize()
            sf, sb = ea.read_stats(wf), ea.read_stats(wb)
            res[on] = (O, tau, mask, iters, dQ, dK, dV, sf["gather_rows"], sb["bwd_gather_rows"])
    finally:
        ea.entmax_attn_gather_enable(True)
    # and the gather paths with the supports taken from the forward's lists instead of found again
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True, workspace=wf)
    g3 = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=wb, fwd_workspace=wf)
    torch.cuda.synchronize()
    sb3 = ea.read_stats(wb)
    # (only the row groups whose output the forward gathered have their supports in its lists; the
    # others stay on the matrix kernels, so the third run may mix both routes; it is compared with
    # the oracle below like the other two)
    assert sb3["bwd_list_subtiles"] == 0 and sb3["bwd_gather_rows"] <= min(res[True][7], res[True][8])
    assert sb3["bwd_gather_rows"] > 0 or res[True][7] == 0
    print("  rows by gather: forward", res[True][7], "backward", res[True][8], "of", B * H * N, flush=True)
    assert res[True][8] > B * H * N // 2 and (res[True][7] > B * H * N // 2 or dtype == "f32")
    assert res[False][7] == 0 and res[False][8] == 0
    # tau, mask and iteration counts come from the list kernel either way
    assert torch.equal(res[True][1], res[False][1]) and torch.equal(res[True][2], res[False][2]) and torch.equal(res[True][3], res[False][3])
    qn, kn, vn, gn = (parity.to_np64(t) for t in (q, k, v, do))
    ref = eo.attn_fwd(qn, kn, vn, alpha, causal, want_margin=False)
    gref = eo.attn_bwd(qn, kn, vn, gn, alpha, causal)
    tol = parity.TOL[q.dtype]
    slack = parity.conditioning_slack(q, k, v, do, alpha, causal, ref["tau"])
    allowed = {"O": tol["O"] + parity.output_slack(q, k, v, alpha, causal, ref["tau"])}
    for name in ("dQ", "dK", "dV"):
        allowed[name] = tol["grad"] * (1 + np.abs(gref[name])) + slack[name]
    for i, name in ((0, "O"), (4, "dQ"), (5, "dK"), (6, "dV")):
        a, b = parity.to_np64(res[True][i]), parity.to_np64(res[False][i])
        oracle = ref["O"] if name == "O" else gref[name]
        worst = (np.abs(a - b) / (2 * allowed[name])).max()
        print(f"  {name}: gather vs matrix {np.abs(a - b).max():.3e}, {worst:.3f} of what is allowed; against the oracle "
              f"{(np.abs(a - oracle) / allowed[name]).max():.3f} / {(np.abs(b - oracle) / allowed[name]).max():.3f}", flush=True)
        assert worst <= 1.0 and (np.abs(a - oracle) <= allowed[name]).all() and (np.abs(b - oracle) <= allowed[name]).all()
        if name != "O":
            c = parity.to_np64(g3[("dQ", "dK", "dV").index(name)])
            print(f"  {name}: supports from the forward's lists ({sb3['bwd_gather_rows']} rows by gather): "
                  f"{(np.abs(c - oracle) / allowed[name]).max():.3f} of what is allowed", flush=True)
            assert (np.abs(c - oracle) <= allowed[name]).all() and (np.abs(c - a) <= 2 * allowed[name]).all()


@pytest.mark.parametrize("dtype,d,N,sigma,causal,hubs", [("bf16", 128, 3072, 3.0, False, (5, 1777)),
                                                         ("bf16", 64, 6144, 2.5, True, (7, 300, 900)),
                                                         ("f32", 64, 3072, 1.0, False, (5, 1777))])
def test_keys_that_many_rows_attend_to(ea, dtype, d, N, sigma, causal, hubs):
    # hub keys that most queries attend to (a common direction added to all queries and to those
    # keys) on top of peaked Gaussian attention.  On the gather path a hub collects far more entries
    # than a key's list holds, and the rest arrive as atomic additions; on the matrix kernels dK, dV of
    # a hub sum thousands of rows (the d = 64 case missed 1e-2 with 11-bit second-stage operands).
    B, H, alpha = 1, 2, 1.5
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, dtype, sigma, seed=95)
    g = torch.Generator().manual_seed(96)
    dirn = torch.randn(d, generator=g)
    dirn = dirn / dirn.norm()
    amp = (sigma * sigma * 3.5 * d ** 0.5) ** 0.5          # amp^2 / sqrt(d) = 3.5 sigma^2: near the row maximum, so a hub is in the support of many rows, not all
    q = (q.float() + amp * dirn).to(q.dtype)
    k = k.clone()
    for hub in hubs:
        k[:, :, hub] = (k[:, :, hub].float() + amp * dirn).to(k.dtype)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    wf = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, False), dtype=torch.uint8, device="cuda")
    O, tau, mask, _ = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True, workspace=wf)
    ws = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, True), dtype=torch.uint8, device="cuda")
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=ws)
    torch.cuda.synchronize()
    st = ea.read_stats(ws)
    print("  backward gather rows", st["bwd_gather_rows"], "of", B * H * N, flush=True)
    if dtype == "bf16" and d == 128:
        assert st["bwd_gather_rows"] > 0
        # once more from the forward's lists (the marks of overfull keys go into them and come off again)
        g2 = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=ws, fwd_workspace=wf)
        torch.cuda.synchronize()
        assert ea.read_stats(ws)["bwd_gather_rows"] > 0
        for name, a, b in zip(("dQ", "dK", "dV"), (dQ, dK, dV), g2):
            assert ((a - b).abs() / (1 + a.abs())).max().item() <= 1e-4, name
    ref, _ = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label="hubs")
    _, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, label="hubs", tau_ref=ref["tau"])
    print("  ", ginfo, flush=True)


def test_sparsemax_with_near_uniform_attention(ea):
    # alpha = 2 with small scores: thousands of keys per row, many of them within the band around
    # the threshold where U jumps between 0 and 1; what those entries may change in dQ, dK, dV is
    # the slack the comparison derives, everything else must meet the plain bar
    run_case(ea, 1, 2, 2048, 64, "bf16", True, 2.0, 0.5, seed=12)


@pytest.mark.parametrize("alphas", [[1.25, 1.5, 2.0], [2.5, 1.75, 3.0]])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_alpha_per_head(ea, dtype, alphas):
    # one alpha per head (general-alpha code for all heads, constants from the per-head table),
    # each head against the oracle run with that head's alpha
    B, H, N, d, causal = 2, 3, 320, 64, True
    sigma = 1.0 if dtype == "f32" else 2.0
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, dtype, sigma, seed=71)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alphas, causal, want_iters=True)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alphas, causal, block_mask=mask)
    torch.cuda.synchronize()
    for hh, a in enumerate(alphas):
        sl = slice(hh, hh + 1)
        ref, info = parity.check_forward(q[:, sl], k[:, sl], v[:, sl], a, causal, O[:, sl], tau[:, sl], mask[:, sl],
                                         label=f"head {hh} alpha {a}")
        _, ginfo = parity.check_backward(q[:, sl], k[:, sl], v[:, sl], do[:, sl], a, causal, dQ[:, sl], dK[:, sl],
                                         dV[:, sl], label=f"head {hh} alpha {a}", tau_ref=ref["tau"])
        print(f"  head {hh} alpha {a}:", info, ginfo, flush=True)
    # equal values take the single-alpha path and must give its result bit for bit
    O1, tau1, mask1 = ea.entmax_attn_fwd(Q, K, V, [1.5] * H, causal)
    O2, tau2, mask2 = ea.entmax_attn_fwd(Q, K, V, 1.5, causal)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(tau1, tau2) and torch.equal(mask1, mask2)
    with pytest.raises(ea.EntmaxAttnError):
        ea.entmax_attn_fwd(Q, K, V, [1.5, 3.5, 1.5], causal)


def test_mfma_probe_runs(ea):
    # measurement aid: every lane sums its accumulators into `sink`; with operands of +-1 the sums
    # are integers, and the argument checks of the binding hold
    data = torch.ones(8192, dtype=torch.float16, device="cuda")
    sink = torch.full((256 * 4,), float("nan"), device="cuda")
    flops = ea.entmax_attn_mfma_probe(data, sink, 4, 3)
    torch.cuda.synchronize()
    assert flops == 4 * 4 * 3 * 32 * 32768.0
    # each accumulator entry: 3 rounds x 8 MFMAs x 16 products of 1 x 1; 64 entries per lane
    assert torch.all(sink == 3 * 8 * 16 * 64).item()
    with pytest.raises(ValueError):
        ea.entmax_attn_mfma_probe(data[:100], sink, 4, 3)
    # the co-issue probe: each lane ends with x0 + x2 = tid + 2 + 2 n (n = rounds x additions / 2)
    # plus its 32 accumulator entries; without MFMAs those are zero
    sink2 = torch.full((512 * 512,), float("nan"), device="cuda")
    ea.entmax_attn_coissue_probe(sink2, 3, 64, False)
    torch.cuda.synchronize()
    tid = torch.arange(512, device="cuda", dtype=torch.float32).repeat(512)
    assert torch.equal(sink2, tid + 2 + 3 * 32 * (1 + 3))
    ea.entmax_attn_coissue_probe(sink2, 2, 0, True)
    torch.cuda.synchronize()
    assert torch.isfinite(sink2).all().item()
    with pytest.raises(ea.EntmaxAttnError):
        ea.entmax_attn_coissue_probe(sink2, 2, 100, True)


def test_c2_exact_config(ea):
    # configs[1] in full: alpha=1.5 bf16 B=4 H=16 N=4096 d=64 causal sigma=1.5, all 64 heads against the oracle
    run_case(ea, 4, 16, 4096, 64, "bf16", True, 1.5, 1.5, seed=2000)


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0])
def test_c5_shape_one_head(ea, alpha):
    # configs[4]: alpha sweep, bf16, N=8192, d=64, causal, Q,K ~ N(0,4); one head
    run_case(ea, 1, 1, 8192, 64, "bf16", True, alpha, 2.0, seed=5000)


def test_c4_shape_planted_keys(ea):
    # configs[3] recipe (planted high-similarity keys, sigma=3) at N=4096, d=128: near-empty masks
    q, k, v, do = workloads.planted_qkv(1, 2, 4096, 128, "bf16", 3.0, seed=4000)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, 1.5, True, want_iters=True)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, 1.5, True, block_mask=mask)
    torch.cuda.synchronize()
    ref, info = parity.check_forward(q, k, v, 1.5, True, O, tau, mask, label="planted")
    _, ginfo = parity.check_backward(q, k, v, do, 1.5, True, dQ, dK, dV, label="planted")
    sparsity = 1.0 - (ref["margin"] > 0).sum() / (2 * 64 * 65 / 2)
    print("  planted: block sparsity", sparsity, info, ginfo, flush=True)
    assert sparsity > 0.5


@pytest.mark.parametrize("hub", [False, True])
def test_backward_twice_gives_the_same_gradients(ea, hub):
    # run-to-run stability.  The matrix kernels accumulate in a fixed order: bit-identical.  On the
    # gather path a key's entries are filed in the order an integer atomic hands out slots, but
    # summed in the order of their query rows: bit-identical too - except for a key that more rows
    # attend to than its list holds (the hub), whose remaining entries arrive as fp32 atomic
    # additions: its dK, dV may differ in the last bits between runs.  dQ is formed row by row in
    # list order and must not.
    B, H, N, d, alpha, causal, sigma = 1, 2, 3072, 128, 1.5, False, 3.0
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, "bf16", sigma, seed=97)
    if hub:
        g = torch.Generator().manual_seed(98)
        dirn = torch.randn(d, generator=g)
        dirn = dirn / dirn.norm()
        amp = (sigma * sigma * 3.5 * d ** 0.5) ** 0.5
        q = (q.float() + amp * dirn).to(q.dtype)
        k = k.clone()
        k[:, :, 11] = (k[:, :, 11].float() + amp * dirn).to(k.dtype)        # one hub key: more entries than its list holds
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    O, tau, mask = ea.entmax_attn_fwd(Q, K, V, alpha, causal)
    try:
        for on in (True, False):
            ea.entmax_attn_gather_enable(on)
            ws = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", causal, True), dtype=torch.uint8, device="cuda")
            runs = []
            for rep in range(2):
                runs.append(ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=ws))
                torch.cuda.synchronize()
            rows = ea.read_stats(ws)["bwd_gather_rows"]
            spread = {n_: ((a - b).abs() / (1 + a.abs())).max().item() for n_, a, b in zip(("dQ", "dK", "dV"), runs[0], runs[1])}
            print(f"  gather paths {'on' if on else 'off'}: rows by gather {rows}, spread between two runs {spread}", flush=True)
            assert (rows > 0) == on
            assert spread["dQ"] == 0.0
            if on and hub:
                assert spread["dK"] <= 1e-4 and spread["dV"] <= 1e-4          # fp32 atomics in another order: far inside the 1e-2 bar
                # the hub, and the few keys whose own component along the hub's direction makes hundreds
                # of rows attend to them too; every other key repeats exactly
                moved = ((runs[0][1] != runs[1][1]).any(-1) | (runs[0][2] != runs[1][2]).any(-1))
                print("  keys that differ between the runs:", int(moved.sum().item()), "of", moved.numel(), flush=True)
                assert moved[:, :, 11].all().item() and moved.float().mean().item() < 0.02
            else:
                assert spread["dK"] == 0.0 and spread["dV"] == 0.0
    finally:
        ea.entmax_attn_gather_enable(True)


def test_values_beyond_fp16_range_are_clamped_and_counted(ea):
    # bf16 inputs above 65504 do not fit the fp16 operands of the matrix kernels: they are copied as
    # +-65504 and counted, so that the caller can tell; in-range inputs count nothing
    B, H, N, d, alpha, causal = 1, 1, 256, 64, 1.5, True
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, "bf16", 1.0, seed=99)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    try:
        ea.entmax_attn_gather_enable(False)            # the matrix kernels, which need the copies, serve every row
        for big in (False, True):
            V2 = V.clone()
            if big:
                V2[0, 0, 3, 5] = 1.0e5
                V2[0, 0, 9, 7] = -2.0e5
            O, tau, mask = ea.entmax_attn_fwd(Q, K, V2, alpha, causal)
            wf = ea.entmax_attn_fwd.last_workspace
            ws = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", causal, True), dtype=torch.uint8, device="cuda")
            ea.entmax_attn_bwd(Q, K, V2, O, dO, tau, alpha, causal, block_mask=mask, workspace=ws)
            torch.cuda.synchronize()
            got = (ea.read_stats(wf)["f16_clamped"], ea.read_stats(ws)["f16_clamped"])
            print("  clamped values counted (forward, backward):", got, flush=True)
            assert got == ((2, 2) if big else (0, 0))
    finally:
        ea.entmax_attn_gather_enable(True)
