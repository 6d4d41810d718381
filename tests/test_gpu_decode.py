"""GPU parity of the inference variant (one query per head against all cached keys) against the
float64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu

TOL = {"bf16": dict(O=1e-2, tau=1e-3), "f32": dict(O=1e-5, tau=1e-5)}


@pytest.fixture(scope="module")
def ea():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2604_15180_amd as ea
    ea.lib()
    return ea


def run(ea, B, H, N, d, dtype, alpha, sigma, seed, planted=False):
    from oracle import entmax_oracle as eo
    print(f"decode case B={B} H={H} N={N} d={d} {dtype} alpha={alpha} sigma={sigma}", flush=True)
    gen = workloads.planted_qkv if planted else workloads.gaussian_qkv
    q4, k, v, _ = gen(B, H, N, d, dtype, sigma, seed=seed)
    q = q4[:, :, -1].contiguous()                      # the newest token's query
    O, tau, support, iters = ea.entmax_attn_decode(q.cuda(), k.cuda(), v.cuda(), alpha)
    torch.cuda.synchronize()
    ref = eo.attn_decode(q.double().numpy(), k.double().numpy(), v.double().numpy(), alpha)
    dO = np.abs(O.double().cpu().numpy() - ref["O"]).max()
    dtau = np.abs(tau.double().cpu().numpy() - ref["tau"]).max()
    assert dO <= TOL[dtype]["O"], f"|dO| = {dO:.3e}"
    assert dtau <= TOL[dtype]["tau"], f"|dtau| = {dtau:.3e}"
    # support size: exact except for keys whose score lies within the tolerance band of tau
    x = (alpha - 1) * ref["z"] - ref["tau"][..., None]
    lo, hi = (x > 1e-3).sum(-1), (x > -1e-3).sum(-1)
    got = support.cpu().numpy()
    assert ((got >= lo) & (got <= hi)).all(), (got, lo, hi)
    assert 1 <= iters.min().item() and iters.max().item() <= (16 if alpha <= 2 else 32)
    print("  decode", dict(dO=float(dO), dtau=float(dtau), support=got.mean(), iters=iters.float().mean().item()), flush=True)


@pytest.mark.parametrize("N", [1, 37, 256, 4099])
def test_decode_fp32_sizes(ea, N):
    # any N: one key, a ragged row, several work-groups with a ragged tail
    run(ea, 1, 2, N, 64, "f32", 1.5, 1.0, seed=80 + N)


@pytest.mark.parametrize("d,alpha", [(64, 1.5), (128, 1.5), (128, 2.0), (64, 1.25), (64, 2.5), (128, 3.0)])
def test_decode_bf16(ea, d, alpha):
    run(ea, 2, 3, 8192, d, "bf16", alpha, 2.0, seed=91)


def test_decode_fp32_head_dim_128(ea):
    run(ea, 1, 2, 1000, 128, "f32", 2.0, 1.0, seed=92)


@pytest.mark.parametrize("alpha,N,sigma", [(2.5, 1000, 1.0), (3.0, 4099, 1.0), (3.0, 16384, 0.3)])
def test_decode_alpha_above_two(ea, alpha, N, sigma):
    # secant steps (Sec. 3.2); the last case overflows the candidate buffer, so each evaluation
    # streams the logits
    run(ea, 1, 2, N, 64, "f32" if N < 16384 else "bf16", alpha, sigma, seed=95)


def test_decode_flat_logits_overflow_the_candidate_buffer(ea):
    # tiny scores: every key is within one unit of the maximum, more than the LDS buffer holds, so
    # every evaluation streams the logits instead
    run(ea, 1, 2, 16384, 64, "bf16", 1.5, 0.3, seed=93)


def test_decode_long_cache_planted_keys(ea):
    # the 64k-token recipe (planted high-similarity keys): a handful of keys in the support
    run(ea, 1, 2, 65536, 128, "bf16", 1.5, 3.0, seed=94, planted=True)


def test_decode_errors(ea):
    q = torch.zeros(1, 1, 64, device="cuda")
    k = torch.zeros(1, 1, 8, 64, device="cuda")
    with pytest.raises(ea.EntmaxAttnError):
        ea.entmax_attn_decode(q, k, k, 3.5)
    with pytest.raises(ValueError):
        ea.entmax_attn_decode(q.cpu(), k, k, 1.5)
    assert ea.entmax_attn_decode_workspace_bytes(1, 1, 8, 96, "f32") == 0
