"""Seeded synthetic inputs shaped like the workloads of the AdaSplash-2 efficiency study.

This module holds no arithmetic of the method: it only draws tensors.  Both the GPU
tests/benchmark and the CPU oracle receive exactly the values produced here (bf16
workloads are rounded to bf16 once, on the host, and the same bits go to both sides).

Sec. 4.2 of the paper draws Q, K, V from zero-mean Gaussians and steers block sparsity
through the query/key variance; the recipes below follow that, plus the variants this
build adds (documented with each function).
"""
import math

import torch

CONFIGS = {
    # name: (B, H, N, d, dtype, causal, alpha, sigma)
    "c1_fp32_n256": dict(B=1, H=2, N=256, d=64, dtype="f32", causal=False, alpha=1.5, sigma=1.0),
    "c2_bf16_n4k": dict(B=4, H=16, N=4096, d=64, dtype="bf16", causal=True, alpha=1.5, sigma=1.5),
    "c3_bf16_n16k": dict(B=2, H=16, N=16384, d=128, dtype="bf16", causal=True, alpha=1.5, sigma=2.0),
    "c4_bf16_n64k": dict(B=1, H=8, N=65536, d=128, dtype="bf16", causal=True, alpha=1.5, sigma=3.0),
    "c5_bf16_n8k": dict(B=2, H=16, N=8192, d=64, dtype="bf16", causal=True, alpha=1.5, sigma=2.0),
}


def _gen(seed):
    return torch.Generator(device="cpu").manual_seed(int(seed))


def _finish(t, dtype):
    if dtype == "bf16":
        return t.to(torch.bfloat16)
    return t.to(torch.float32)


def gaussian_qkv(B, H, N, d, dtype, sigma, seed, block_rho=0.0, block=64):
    """Q, K ~ N(0, sigma^2), V, dO ~ N(0, 1), i.i.d. (Sec. 4.2 "Sparsity-speed tradeoff").

    block_rho > 0 adds this build's block-correlated variant: the 64 query rows of one
    query tile share a common direction, Q_r = sigma (sqrt(rho) g_tile + sqrt(1-rho) eps_r),
    so that whole 64x64 blocks become empty as sigma grows (i.i.d. rows keep at least one key
    at a random position each, which caps block sparsity).
    """
    g = _gen(seed)
    q = torch.randn(B, H, N, d, generator=g)
    k = torch.randn(B, H, N, d, generator=g)
    v = torch.randn(B, H, N, d, generator=g)
    do = torch.randn(B, H, N, d, generator=g)
    if block_rho > 0.0:
        shared = torch.randn(B, H, N // block, 1, d, generator=g)
        q = q.view(B, H, N // block, block, d)
        q = math.sqrt(block_rho) * shared + math.sqrt(1.0 - block_rho) * q
        q = q.reshape(B, H, N, d)
    q = q * sigma
    k = k * sigma
    return tuple(_finish(t, dtype) for t in (q, k, v, do))


def ramp_qkv(B, H, N, d, dtype, rise_per_tile, seed, noise=0.3, block=64):
    """Keys whose similarity to every query drifts with the key index: all queries share a
    direction u (plus noise), key j carries t_j u (plus noise) with t_j linear in j, so that
    (alpha-1) s at alpha = 1.5 moves by `rise_per_tile` per 64 keys.  Positive: each row's
    running maximum keeps climbing as keys stream by; negative: it is met at the first keys.
    Not a workload of the paper; it drives a single-sweep maximum through many updates."""
    g = _gen(seed)
    u = torch.randn(B, H, 1, d, generator=g)
    u = u / u.norm(dim=-1, keepdim=True)
    q = math.sqrt(d) * u + noise * torch.randn(B, H, N, d, generator=g)
    slope = 2.0 * rise_per_tile / block
    t = slope * torch.arange(N, dtype=torch.float32).view(1, 1, N, 1)
    if rise_per_tile < 0:
        t = t - t.min()
    k = t * u + noise * torch.randn(B, H, N, d, generator=g)
    v = torch.randn(B, H, N, d, generator=g)
    do = torch.randn(B, H, N, d, generator=g)
    return tuple(_finish(x, dtype) for x in (q, k, v, do))


def planted_qkv(B, H, N, d, dtype, sigma, seed, n_planted=32, strength=None, block=64):
    """Long-context recipe: Gaussian Q, K plus, for every 64-row query tile I > 0, a unit
    direction g_I added (scaled by `a`) to all 64 query rows and to `n_planted` key rows
    drawn among the keys visible to the whole tile (index < 64 I).  a^2/sqrt(d) defaults to
    60, clear of the i.i.d. score maximum, so each query tile attends to its planted keys."""
    g = _gen(seed)
    q = torch.randn(B, H, N, d, generator=g) * sigma
    k = torch.randn(B, H, N, d, generator=g) * sigma
    v = torch.randn(B, H, N, d, generator=g)
    do = torch.randn(B, H, N, d, generator=g)
    a = math.sqrt((strength if strength is not None else 60.0) * math.sqrt(d))
    T = N // block
    dirs = torch.randn(B, H, T, d, generator=g)
    dirs = dirs / dirs.norm(dim=-1, keepdim=True)
    q = q.view(B, H, T, block, d) + a * dirs.unsqueeze(3)
    q[:, :, 0] -= a * dirs[:, :, 0].unsqueeze(2)  # tile 0 has no earlier keys
    q = q.reshape(B, H, N, d)
    for I in range(1, T):
        pos = torch.randint(0, block * I, (B, H, n_planted), generator=g)
        add = a * dirs[:, :, I]  # [B,H,d]
        k.scatter_add_(2, pos.unsqueeze(-1).expand(B, H, n_planted, d),
                       add.unsqueeze(2).expand(B, H, n_planted, d).contiguous())
    return tuple(_finish(t, dtype) for t in (q, k, v, do))


def make(name, seed=0, **override):
    """Inputs of a named configuration: returns (cfg dict, Q, K, V, dO) on the CPU."""
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    kind = cfg.pop("kind", "planted" if name.startswith("c4") else "gaussian")
    args = (cfg["B"], cfg["H"], cfg["N"], cfg["d"], cfg["dtype"], cfg["sigma"], seed)
    if kind == "planted":
        q, k, v, do = planted_qkv(*args)
    else:
        q, k, v, do = gaussian_qkv(*args, block_rho=cfg.get("block_rho", 0.0))
    return cfg, q, k, v, do
