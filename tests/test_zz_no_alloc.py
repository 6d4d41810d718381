"""The allocation-free decode entry point (scratch in the library's own static device array)
against the entry point that takes a caller's workspace (same kernels), on two
calls in a row, the second with a smaller input (the array then still holds the first call's data)."""
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ea():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2604_15180_amd as ea
    ea.lib()
    return ea


def test_static_scratch_decode_matches_workspace_decode(ea):
    from oracle import entmax_oracle as eo
    import numpy as np
    for (B, H, N, d, dtype, alpha, sigma, seed) in [(2, 4, 12288, 128, "bf16", 1.5, 2.5, 501), (1, 3, 1000, 64, "bf16", 1.5, 2.0, 502)]:
        print(f"static decode case B={B} H={H} N={N} d={d} {dtype}", flush=True)
        q4, k, v, _ = workloads.gaussian_qkv(B, H, N, d, dtype, sigma, seed=seed)
        q = q4[:, :, -1].contiguous()
        Q, K, V = q.cuda(), k.cuda(), v.cuda()
        want = ea.entmax_attn_decode(Q, K, V, alpha)
        outs = tuple(torch.full_like(t, -7) for t in want)
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]      # allocations made so far
        got = ea.entmax_attn_decode_static(Q, K, V, alpha, out=outs)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before     # torch made none either
        # same kernels; the order in which a work-group's lanes file the logits they keep (an LDS
        # counter) differs from run to run, and with it the order of the fp32 sums: not the same
        # bits, but far inside the bar the library is held to against the oracle
        assert (got[0] - want[0]).abs().max().item() <= 1e-5 and (got[1] - want[1]).abs().max().item() <= 1e-6
        assert torch.equal(got[2], want[2])
        assert (got[3] > 0).all()
        ref = eo.attn_decode(q.double().numpy(), k.double().numpy(), v.double().numpy(), alpha)
        assert np.abs(got[0].double().cpu().numpy() - ref["O"]).max() <= 1e-2
        assert np.abs(got[1].double().cpu().numpy() - ref["tau"]).max() <= 1e-3


def test_static_scratch_decode_rejects_what_does_not_fit(ea):
    cap = ea.entmax_attn_decode_static_max_bytes()
    B, H, N, d = 1, 64, 131072, 64
    assert ea.entmax_attn_decode_workspace_bytes(B, H, N, d, "bf16") > cap
    # only the shapes are looked at before the size check: small stand-in tensors would be wrong
    # for a real call, so ask through the raw ABI with non-null dummy pointers
    import ctypes
    x = torch.zeros(64, device="cuda")
    p = ctypes.c_void_p(x.data_ptr())
    rc = ea.lib().entmax_attn_decode_static(p, p, p, p, p, None, None, B, H, N, d, 1, 1.5, None)
    assert rc == -7 and "scratch" in ea.entmax_attn_strerror(rc)
    torch.cuda.synchronize()
