"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and turns bad arguments into error codes without touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2604_15180_amd as ea

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "entmax_attn.h"), os.path.join(ROOT, "include", "entmax_attn_aids.h")]


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(ea.lib_path()):
        from paper_2604_15180_amd import build
        build.build()
    return ea.lib()


def declared_symbols():
    names = set()
    for header in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(entmax_attn_\w+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert {"entmax_attn_fwd", "entmax_attn_bwd", "entmax_attn_workspace_bytes", "entmax_attn_mask_tile",
            "entmax_attn_strerror", "entmax_attn_last_hip_error", "entmax_attn_histogram_bins"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_introspection(L):
    assert ea.entmax_attn_mask_tile() == 64
    assert ea.entmax_attn_histogram_bins() >= 8
    assert ea.entmax_attn_strerror(0) == "ok"
    for code in range(-7, 0):
        assert ea.entmax_attn_strerror(code) not in ("ok", "unknown error code")
    assert ea.entmax_attn_strerror(-99) == "unknown error code"


def test_workspace_query(L):
    f = ea.entmax_attn_workspace_bytes
    assert f(2, 16, 16384, 128, "bf16", True, False) > 2 * 16 * 16384 * 128 * 2
    assert f(2, 16, 16384, 128, "bf16", True, True) > 3 * 2 * 16 * 16384 * 128 * 2
    assert f(1, 2, 256, 64, "f32", False, False) % 256 == 0
    for bad in [(0, 1, 256, 64), (1, 1, 100, 64), (1, 1, 256, 96), (1, 1, 262144, 64), (1, 1, -64, 64)]:
        assert f(*bad, "bf16", True, False) == 0
    assert f(1, 1, 256, 64, "int8", True, False) == 0


def test_gather_switch_and_its_workspace(L):
    # the switch is a host-side flag (no GPU call); the backward's workspace holds the support
    # lists, two per row, and the lists by key, whichever way the switch stands
    assert L.entmax_attn_gather_enable(0) == 0
    assert L.entmax_attn_gather_enable(1) == 0
    B, H, N, d = 1, 2, 4096, 128
    rows = B * H * N
    bwd = ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", True, True)
    assert bwd > 4 * rows * d * 2 + rows * 2 * 64 * 8 + rows * 64 * 16      # fp16 copies + both kinds of lists
    fwd = ea.entmax_attn_workspace_bytes(B, H, N, d, "bf16", True, False)
    assert fwd > rows * 2 * 256 * 8                                         # candidate lists


def call_fwd(L, ptrs, B=1, H=1, N=64, d=64, dtype=1, alpha=1.5, ws=0x1000, ws_bytes=1 << 30):
    vp = ctypes.c_void_p
    q, k, v, o, tau, m = (vp(x) for x in ptrs)
    return L.entmax_attn_fwd(q, k, v, o, tau, m, None, B, H, N, d, dtype, alpha, 1, vp(ws), ws_bytes, None)


def test_forward_argument_errors(L):
    ok = [0x1000] * 6   # never dereferenced: every case below fails validation first
    assert call_fwd(L, [0] + ok[1:]) == -1
    assert call_fwd(L, ok[:5] + [0]) == -1
    assert call_fwd(L, ok, alpha=1.0) == -2
    assert call_fwd(L, ok, alpha=3.5) == -2
    assert call_fwd(L, ok, alpha=float("nan")) == -2
    assert call_fwd(L, ok, N=96) == -3
    assert call_fwd(L, ok, d=32) == -3
    assert call_fwd(L, ok, B=0) == -3
    assert call_fwd(L, ok, dtype=7) == -4
    assert call_fwd(L, ok, ws=0) == -5
    assert call_fwd(L, ok, ws=0x1010) == -5          # misaligned
    assert call_fwd(L, ok, ws_bytes=16) == -5


def test_backward_argument_errors(L):
    vp = ctypes.c_void_p
    a = vp(0x1000)
    def call(q=a, do=a, tau=a, dq=a, N=64, d=64, dtype=1, alpha=1.5, ws=vp(0x1000), nbytes=1 << 30):
        return L.entmax_attn_bwd(q, a, a, None, do, tau, None, dq, a, a, 1, 1, N, d, dtype, alpha, 1, ws, nbytes, None)
    assert call(q=None) == -1 and call(do=None) == -1 and call(tau=None) == -1 and call(dq=None) == -1
    assert call(alpha=0.5) == -2
    assert call(N=0) == -3 and call(d=256) == -3
    assert call(dtype=-1) == -4
    assert call(ws=None) == -5 and call(nbytes=0) == -5


def test_python_binding_refuses_cpu_tensors(L):
    import torch
    x = torch.zeros(1, 1, 64, 64)
    with pytest.raises(ValueError):
        ea.entmax_attn_fwd(x, x, x, 1.5, True)
