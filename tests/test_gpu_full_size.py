"""GPU parity at the benchmark's full size (configs[2]: B=2, H=16, N=16384, d=128, bf16, causal),
in the launch configuration bench.py times.  The oracle cannot run all 32 heads in test time, so
it runs whole heads sampled from the batch (dK/dV of a head need every query row of that head),
and the remaining heads are covered by properties that hold at any size."""
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


@pytest.mark.parametrize("sigma,heads", [(1.0, [(0, 3), (1, 12)]), (2.0, [(0, 7)]), (3.0, [(1, 2)]), (4.0, [(0, 3), (1, 12)])])
def test_c3_full_size_sampled_heads(ea, sigma, heads):
    from oracle import entmax_oracle as eo
    cfg = workloads.CONFIGS["c3_bf16_n16k"]
    B, H, N, d, alpha, causal = cfg["B"], cfg["H"], cfg["N"], cfg["d"], cfg["alpha"], cfg["causal"]
    print(f"case c3 full size sigma={sigma}", flush=True)
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, "bf16", sigma, seed=3000 + int(sigma))
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    wf = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", causal, False), dtype=torch.uint8, device="cuda")
    wb = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", causal, True), dtype=torch.uint8, device="cuda")
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True, workspace=wf)
    # (as bench.py calls it: the backward is handed the forward's workspace)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=wb, fwd_workspace=wf)
    torch.cuda.synchronize()
    # which path served the rows, as in the launch configuration bench.py times: at sigma = 4 every
    # row group goes by gather in both passes, at sigma = 1 the backward is split between the gather
    # and the matrix kernels
    sf, sb = ea.read_stats(wf), ea.read_stats(wb)
    print("  rows by gather: forward", sf["gather_rows"], "backward", sb["bwd_gather_rows"], "of", B * H * N, flush=True)
    if sigma >= 2.0:
        assert sf["gather_rows"] == B * H * N and sb["bwd_gather_rows"] == B * H * N
    else:
        assert 0 < sb["bwd_gather_rows"] < B * H * N and sb["dq_subtiles"] > 0
    del wf, wb
    # properties over all heads
    assert torch.isfinite(O).all() and torch.isfinite(dQ).all() and torch.isfinite(dK).all() and torch.isfinite(dV).all()
    # rows of P sum to one  ->  sum_j dV_j = sum_r dO_r   (per head and channel)
    lhs = dV.double().sum(2)
    rhs = do.double().sum(2).cuda()
    assert (lhs - rhs).abs().max().item() < 0.5, (lhs - rhs).abs().max().item()
    it = iters.float()
    assert it.min().item() >= 1 and it.mean().item() <= 2.0 + 1e-6
    # sampled heads against the oracle, whole heads (every sigma of the benchmark's sweep is covered)
    for (b, h) in heads:
        sl = (slice(b, b + 1), slice(h, h + 1))
        qs, ks, vs, dos = (t[sl] for t in (q, k, v, do))
        label = f"c3 sigma={sigma} head=({b},{h})"
        print("  oracle on", label, flush=True)
        ref, info = parity.check_forward(qs, ks, vs, alpha, causal, O[sl], tau[sl], mask[sl], label=label)
        _, ginfo = parity.check_backward(qs, ks, vs, dos, alpha, causal, dQ[sl], dK[sl], dV[sl], label=label)
        print("  ", info, ginfo, flush=True)


def test_c4_full_size_one_head(ea):
    # configs[3]: B=1, H=8, N=65536, d=128, bf16, causal, sigma=3 plus planted keys.  N is past
    # the range in which a 16-bit histogram counter cannot overflow, so this runs the kernel
    # variant with one row per lane and 32-bit counters.
    cfg = workloads.CONFIGS["c4_bf16_n64k"]
    B, H, N, d, alpha, causal = cfg["B"], cfg["H"], cfg["N"], cfg["d"], cfg["alpha"], cfg["causal"]
    print("case c4 full size", flush=True)
    q, k, v, do = workloads.planted_qkv(B, H, N, d, "bf16", cfg["sigma"], seed=4001)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask)
    torch.cuda.synchronize()
    assert torch.isfinite(O).all() and torch.isfinite(dQ).all() and torch.isfinite(dK).all() and torch.isfinite(dV).all()
    lhs = dV.double().sum(2)
    rhs = do.double().sum(2).cuda()
    assert (lhs - rhs).abs().max().item() < 1.0, (lhs - rhs).abs().max().item()
    T = N // 64
    bits = parity.unpack_mask(mask, T)
    sparsity = 1.0 - bits.sum() / (B * H * T * (T + 1) / 2)
    print("  block sparsity", sparsity, "mean iters", iters.float().mean().item(), flush=True)
    assert sparsity > 0.9
    assert iters.max().item() <= 12
    sl = (slice(0, 1), slice(5, 6))
    qs, ks, vs, dos = (t[sl] for t in (q, k, v, do))
    print("  oracle on head (0,5)", flush=True)
    ref, info = parity.check_forward(qs, ks, vs, alpha, causal, O[sl], tau[sl], mask[sl], label="c4 head=(0,5)")
    _, ginfo = parity.check_backward(qs, ks, vs, dos, alpha, causal, dQ[sl], dK[sl], dV[sl], label="c4 head=(0,5)")
    print("  ", info, ginfo, flush=True)


@pytest.mark.parametrize("N", [4096, 32768, 65536])
def test_context_scaling_recipe(ea, N):
    # the second workload's inputs (planted keys, d = 64, sigma = 3; `bench.py --workload context`
    # and the `context` rows of the default line), one head per length against the oracle; the
    # longest length is the planted case of test_maximum_sequence_length (32768 and 65536 tokens:
    # the two part lengths of the dK, dV kernel's long mask columns)
    B, H, d, alpha, causal = 1, 1, 64, 1.5, True
    print(f"case context scaling N={N}", flush=True)
    q, k, v, do = workloads.planted_qkv(B, H, N, d, "bf16", 3.0, seed=7000 + N // 4096)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask)
    torch.cuda.synchronize()
    print("  oracle", flush=True)
    ref, info = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label=f"context N={N}")
    _, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, label=f"context N={N}")
    T = N // 64
    sparsity = 1.0 - (ref["margin"] > 0).sum() / (T * (T + 1) / 2)
    print("  block sparsity", sparsity, info, ginfo, "mean iters", iters.float().mean().item(), flush=True)
    assert sparsity > 0.6 and iters.float().mean().item() <= 2.0


@pytest.mark.parametrize("recipe", ["gaussian", "planted"])
def test_maximum_sequence_length(ea, recipe):
    # N = 131072 is the largest size the library accepts (2048 key tiles, 64 mask words per row);
    # one head, d = 64: i.i.d. Gaussian Q, K with sigma = 3, and the planted-key recipe of the
    # context-scaling workload (every support key of a query tile carries the same planted
    # direction, so dQ and dK are what is left after those terms cancel)
    B, H, N, d, alpha, causal = 1, 1, 131072, 64, 1.5, True
    print(f"case N=131072 {recipe}", flush=True)
    if recipe == "planted":
        q, k, v, do = workloads.planted_qkv(B, H, N, d, "bf16", 3.0, seed=7032)
    else:
        q, k, v, do = workloads.gaussian_qkv(B, H, N, d, "bf16", 3.0, seed=4002)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask)
    torch.cuda.synchronize()
    assert iters.max().item() <= 12
    print("  oracle", flush=True)
    ref, info = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label=f"N=131072 {recipe}")
    _, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, label=f"N=131072 {recipe}")
    T = N // 64
    sparsity = 1.0 - (ref["margin"] > 0).sum() / (T * (T + 1) / 2)
    print("  block sparsity", sparsity, info, ginfo, "mean iters", iters.float().mean().item(), flush=True)


def test_flat_attention_at_65536_tokens(ea):
    # From 65536 keys on a histogram bin can hold more keys than a 16-bit counter, so the sweep-based
    # threshold kernel switches to its variant with 32-bit counters; the list kernel's shared 16-bit
    # counters only ever count listed candidates (at most 512 per row).  Tiny scores put every
    # visible key within one unit of the row's maximum: all but the first rows overflow their
    # lists, are redone by the sweep-based kernel, and have thousands of keys in the support.
    B, H, N, d, alpha, causal = 1, 1, 65536, 64, 1.5, True
    print("case flat attention N=65536", flush=True)
    q, k, v, _ = workloads.gaussian_qkv(B, H, N, d, "bf16", 0.3, seed=4100)
    Q, K, V = (t.cuda() for t in (q, k, v))
    ws = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", causal, False), dtype=torch.uint8, device="cuda")
    O, tau, mask, iters = ea.entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=True, workspace=ws)
    torch.cuda.synchronize()
    st = ea.read_stats(ws)
    print("  stats", {k_: st[k_] for k_ in ("list_overflow_blocks", "tau_subtiles")}, "oracle", flush=True)
    assert st["list_overflow_blocks"] > 0.9 * (N // 64)
    assert iters.max().item() <= 12
    ref, info = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label="flat N=65536")
    support = ((alpha - 1) * 0 + (ref["margin"] > 0)).sum()
    print("  flat N=65536", info, "marked tiles", int(support), "mean iters", iters.float().mean().item(), flush=True)


def test_long_mask_columns_without_a_causal_mask(ea):
    # Past 16384 tokens the dK, dV kernel works a key block's mask column off in parts that add their
    # results with atomics (the causal cases above have a few such columns: planted keys).  Here
    # there is no causal mask and the gather paths are off, so every key block's column holds most
    # of the 272 query tiles and every dK, dV row is the sum of five parts; also run twice, which
    # must agree to rounding (the parts add in any order).
    B, H, N, d, alpha, causal = 1, 1, 17408, 64, 1.5, False
    print("case long columns, no causal mask, N=17408", flush=True)
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, "bf16", 2.0, seed=515)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    try:
        ea.entmax_attn_gather_enable(False)
        O, tau, mask = ea.entmax_attn_fwd(Q, K, V, alpha, causal)
        ws = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", causal, True), dtype=torch.uint8, device="cuda")
        dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=ws)
        again = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=ws)
        torch.cuda.synchronize()
        assert ea.read_stats(ws)["bwd_gather_rows"] == 0
    finally:
        ea.entmax_attn_gather_enable(True)
    T = N // 64
    bits = torch.tensor([bin(int(w) & 0xffffffff).count("1") for w in mask[0].reshape(-1).tolist()]).sum().item()
    print(f"  marked tiles {bits} of {T * T}", flush=True)
    assert bits > T * T // 2
    spread = {n_: ((a - b).abs() / (1 + a.abs())).max().item() for n_, a, b in zip(("dQ", "dK", "dV"), (dQ, dK, dV), again)}
    print("  spread between two runs", spread, flush=True)
    assert spread["dQ"] == 0.0 and spread["dK"] <= 1e-4 and spread["dV"] <= 1e-4
    print("  oracle", flush=True)
    ref, info = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label="long columns")
    _, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, label="long columns")
    print("  ", info, ginfo, flush=True)


@pytest.mark.parametrize("d,hub", [(64, False), (128, True)])
def test_gather_and_matrix_rows_together_at_32768_tokens(ea, d, hub):
    # i.i.d. inputs at sigma = 1, one head of 32768 tokens: about half (d = 64) or most (d = 128) of
    # the row groups go by the gather kernels, the early ones stay on the matrix kernels, whose key
    # blocks then see mask columns long enough to be worked off in parts; the backward takes the
    # supports from the forward's lists.  With hub keys three keys are attended by most later rows.
    B, H, N, alpha, causal, sigma = 1, 1, 32768, 1.5, True, 1.0
    print(f"case both routes N={N} d={d} hub={hub}", flush=True)
    q, k, v, do = workloads.gaussian_qkv(B, H, N, d, "bf16", sigma, seed=777 + d)
    if hub:
        g = torch.Generator().manual_seed(5)
        dirn = torch.randn(d, generator=g)
        dirn = dirn / dirn.norm()
        amp = (sigma * sigma * 3.5 * d ** 0.5) ** 0.5
        q = (q.float() + amp * dirn).to(q.dtype)
        k = k.clone()
        for j in (100, 5000, 20000):
            k[:, :, j] = (k[:, :, j].float() + amp * dirn).to(k.dtype)
    Q, K, V, dO = (t.cuda() for t in (q, k, v, do))
    wf = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", causal, False), dtype=torch.uint8, device="cuda")
    wb = torch.empty(ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", causal, True), dtype=torch.uint8, device="cuda")
    O, tau, mask = ea.entmax_attn_fwd(Q, K, V, alpha, causal, workspace=wf)
    dQ, dK, dV = ea.entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=mask, workspace=wb, fwd_workspace=wf)
    torch.cuda.synchronize()
    rows = ea.read_stats(wb)["bwd_gather_rows"]
    print(f"  rows by gather {rows} of {N}", flush=True)
    assert N // 4 < rows < N
    ref, info = parity.check_forward(q, k, v, alpha, causal, O, tau, mask, label="both routes")
    _, ginfo = parity.check_backward(q, k, v, do, alpha, causal, dQ, dK, dV, label="both routes", tau_ref=ref["tau"])
    print("  ", info, ginfo, flush=True)
