"""ctypes front end of the float64 C oracle (oracle/entmax_oracle.c).

TEST INFRASTRUCTURE ONLY: the slow, plain definition of alpha-entmax attention
(Eq. 2-4 of the AdaSplash-2 paper) and of its gradient (Sec. 3.3 "Backward
pass", Alg. 2-3), against which the GPU library is compared.  It shares no code
with the GPU path.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        L.oracle_f.restype = ctypes.c_double
        L.oracle_f.argtypes = [dp, ctypes.c_long, ctypes.c_double, ctypes.c_double]
        L.oracle_tau_bisect.restype = ctypes.c_double
        L.oracle_tau_bisect.argtypes = [dp, ctypes.c_long, ctypes.c_double, ctypes.c_double]
        L.oracle_tau_sort.restype = ctypes.c_double
        L.oracle_tau_sort.argtypes = [dp, ctypes.c_long, ctypes.c_double, dp]
        L.oracle_tau_row.restype = ctypes.c_double
        L.oracle_tau_row.argtypes = [dp, ctypes.c_long, ctypes.c_double, ctypes.c_int, dp]
        L.oracle_entmax.restype = ctypes.c_int
        L.oracle_entmax.argtypes = [dp, ctypes.c_long, ctypes.c_double, ctypes.c_int, dp, dp]
        L.oracle_entmax_attn_fwd.restype = ctypes.c_int
        L.oracle_entmax_attn_fwd.argtypes = [dp, dp, dp] + [ctypes.c_int] * 4 + [
            ctypes.c_double, ctypes.c_int, ctypes.c_int, dp, dp, dp, dp]
        L.oracle_entmax_attn_bwd.restype = ctypes.c_int
        L.oracle_entmax_attn_bwd.argtypes = [dp, dp, dp, dp] + [ctypes.c_int] * 4 + [
            ctypes.c_double, ctypes.c_int, dp, dp, dp, dp]
        L.oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _c(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def f(x, alpha, tau):
    """f(tau) of Eq. 4 for pre-scaled scores x = (alpha-1) s."""
    x = _c(x)
    return float(lib().oracle_f(_dp(x), x.size, alpha, tau))


def tau_bisect(x, alpha, tol=1e-12):
    """Bisection on the Eq. 5 bracket; x = (alpha-1) s."""
    x = _c(x)
    return float(lib().oracle_tau_bisect(_dp(x), x.size, alpha, tol))


def tau_sort(x, alpha):
    """Sort-based exact threshold (alpha in {1.5, 2} only); x = (alpha-1) s."""
    x = _c(x)
    work = np.empty(x.size, dtype=np.float64)
    return float(lib().oracle_tau_sort(_dp(x), x.size, alpha, _dp(work)))


def tau_row(x, alpha, full=False):
    x = _c(x)
    work = np.empty(3 * x.size, dtype=np.float64)
    return float(lib().oracle_tau_row(_dp(x), x.size, alpha, int(full), _dp(work)))


def entmax(s, alpha, full=False):
    """alpha-entmax of one raw score vector s (Eq. 3). Returns (p, tau)."""
    s = _c(s)
    p = np.empty_like(s)
    t = ctypes.c_double(0.0)
    rc = lib().oracle_entmax(_dp(s), s.size, alpha, int(full), _dp(p), ctypes.byref(t))
    if rc != 0:
        raise ValueError(f"oracle_entmax failed: {rc}")
    return p, t.value


def attn_fwd(Q, K, V, alpha, causal, tile=64, want_margin=True, want_P=False):
    """Q,K,V: [B,H,N,d] arrays (any float dtype; converted exactly to float64).

    Returns dict(O [B,H,N,d], tau [B,H,N], margin [B,H,T,T] or None, P [B,H,N,N] or None).
    The block-mask bit of tile (I,J) is margin[I,J] > 0.
    """
    Q, K, V = _c(Q), _c(K), _c(V)
    B, H, N, d = Q.shape
    O = np.empty((B, H, N, d), dtype=np.float64)
    tau = np.empty((B, H, N), dtype=np.float64)
    margin = None
    if want_margin:
        T = N // tile
        margin = np.empty((B, H, T, T), dtype=np.float64)
    P = np.empty((B, H, N, N), dtype=np.float64) if want_P else None
    rc = lib().oracle_entmax_attn_fwd(_dp(Q), _dp(K), _dp(V), B, H, N, d, float(alpha), int(bool(causal)),
                                      int(tile), _dp(O), _dp(tau), _dp(margin), _dp(P))
    if rc != 0:
        raise ValueError(f"oracle_entmax_attn_fwd failed: {rc}")
    return {"O": O, "tau": tau, "margin": margin, "P": P}


def attn_bwd(Q, K, V, dO, alpha, causal):
    """Gradient of sum(O*dO) w.r.t. Q,K,V. Returns dict(dQ,dK,dV [B,H,N,d], delta [B,H,N])."""
    Q, K, V, dO = _c(Q), _c(K), _c(V), _c(dO)
    B, H, N, d = Q.shape
    dQ = np.empty_like(Q); dK = np.empty_like(Q); dV = np.empty_like(Q)
    delta = np.empty((B, H, N), dtype=np.float64)
    rc = lib().oracle_entmax_attn_bwd(_dp(Q), _dp(K), _dp(V), _dp(dO), B, H, N, d, float(alpha),
                                      int(bool(causal)), _dp(dQ), _dp(dK), _dp(dV), _dp(delta))
    if rc != 0:
        raise ValueError(f"oracle_entmax_attn_bwd failed: {rc}")
    return {"dQ": dQ, "dK": dK, "dV": dV, "delta": delta}


def attn_decode(q, K, V, alpha):
    """Inference variant on materialised logits (the paper's appendix on language modelling runs
    inference on the whole logit vector of one query): one query row per head against all N
    cached keys.  z = K q / sqrt(d), p = alpha-entmax(z) (Eq. 3), o = p V.

    q: [B,H,d], K, V: [B,H,N,d].  Returns dict(O [B,H,d], tau [B,H] (raw convention:
    p = [(alpha-1) z - tau]_+^(1/(alpha-1))), P [B,H,N], z [B,H,N])."""
    q, K, V = _c(q), _c(K), _c(V)
    B, H, N, d = K.shape
    O = np.empty((B, H, d)); tau = np.empty((B, H)); P = np.empty((B, H, N)); Z = np.empty((B, H, N))
    for b in range(B):
        for h in range(H):
            z = K[b, h] @ q[b, h] / np.sqrt(d)
            pr, t = entmax(z, alpha)
            Z[b, h] = z; P[b, h] = pr; tau[b, h] = t
            O[b, h] = pr @ V[b, h]
    return {"O": O, "tau": tau, "P": P, "z": Z}


def block_mask_words(margin):
    """Pack margin > 0 into int32 words, bit k of word m <-> key tile 32m+k (App. C.4)."""
    bits = (margin > 0)
    *lead, T, Tc = bits.shape
    W = (Tc + 31) // 32
    padded = np.zeros((*lead, T, W * 32), dtype=np.uint64)
    padded[..., :Tc] = bits
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    words = (padded.reshape(*lead, T, W, 32) * weights).sum(axis=-1).astype(np.uint32)
    return words.view(np.int32)
