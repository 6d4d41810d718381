"""ctypes binding of libentmax_attn.so (same names as the C entry points).

PyTorch is used for device memory and the current HIP stream only.  Outputs are allocated
here; every step of the path runs inside the library's kernels.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libentmax_attn.so")
_lib = None

EA_F32, EA_BF16 = 0, 1
EA_STATS_WORDS = 16
EA_STATS_COPIES = 64
STAT_NAMES = ("tau_subtiles", "out_subtiles", "delta_subtiles", "dq_subtiles", "dkdv_subtiles",
              "sweeps", "mask_subtiles", "out_pv_subtiles", "list_overflow_blocks", "gather_rows", "bwd_list_subtiles", "bwd_gather_rows",
              "f16_clamped")
EA_TIMER_SLOTS = 10
TIMER_NAMES = ("fwd_prep", "tau", "out", "mask", "bwd_prep", "dq", "dkdv", "decode_scores", "bwd_list", "bwd_gather")


class EntmaxAttnError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"entmax_attn error {code}: {text}")
        self.code = code


def lib_path():
    return _LIB_PATH


def lib():
    """Load the built library (build it first with __graft_entry__.build() or
    `python -m paper_2604_15180_amd.build`); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is not built; run `python paper_2604_15180_amd/build.py` (needs hipcc). "
                "There is no fallback path.")
        L = ctypes.CDLL(_LIB_PATH)
        vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        L.entmax_attn_mask_tile.restype = ci
        L.entmax_attn_mask_tile.argtypes = []
        L.entmax_attn_histogram_bins.restype = ci
        L.entmax_attn_histogram_bins.argtypes = []
        L.entmax_attn_last_hip_error.restype = ci
        L.entmax_attn_last_hip_error.argtypes = []
        L.entmax_attn_workspace_bytes.restype = sz
        L.entmax_attn_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci, ci]
        L.entmax_attn_fwd.restype = ci
        L.entmax_attn_fwd.argtypes = [vp] * 7 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
        L.entmax_attn_bwd.restype = ci
        L.entmax_attn_bwd.argtypes = [vp] * 10 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
        L.entmax_attn_bwd_with_lists.restype = ci
        L.entmax_attn_bwd_with_lists.argtypes = [vp] * 8 + [sz] + [vp] * 3 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
        L.entmax_attn_fwd_alpha_per_head.restype = ci
        L.entmax_attn_fwd_alpha_per_head.argtypes = [vp] * 7 + [ci, ci, ci, ci, ci, ctypes.POINTER(cf), ci, vp, sz, vp]
        L.entmax_attn_bwd_alpha_per_head.restype = ci
        L.entmax_attn_bwd_alpha_per_head.argtypes = [vp] * 10 + [ci, ci, ci, ci, ci, ctypes.POINTER(cf), ci, vp, sz, vp]
        L.entmax_attn_timer_enable.restype = ci
        L.entmax_attn_timer_enable.argtypes = [ci]
        L.entmax_attn_gather_enable.restype = ci
        L.entmax_attn_gather_enable.argtypes = [ci]
        L.entmax_attn_right_edge_enable.restype = ci
        L.entmax_attn_right_edge_enable.argtypes = [ci]
        L.entmax_attn_timer_read.restype = ci
        L.entmax_attn_timer_read.argtypes = [ctypes.POINTER(cf), ctypes.POINTER(ci), ci]
        L.entmax_attn_decode_workspace_bytes.restype = sz
        L.entmax_attn_decode_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        L.entmax_attn_decode.restype = ci
        L.entmax_attn_decode.argtypes = [vp] * 7 + [ci, ci, ci, ci, ci, cf, vp, sz, vp]
        L.entmax_attn_decode_static_max_bytes.restype = sz
        L.entmax_attn_decode_static_max_bytes.argtypes = []
        L.entmax_attn_decode_static.restype = ci
        L.entmax_attn_decode_static.argtypes = [vp] * 7 + [ci, ci, ci, ci, ci, cf, vp]
        L.entmax_attn_fwd_histogram_bounds.restype = ci
        L.entmax_attn_fwd_histogram_bounds.argtypes = [vp, sz, ci, ci, ci, ci, ci, vp, vp, vp]
        L.entmax_attn_mfma_probe.restype = ci
        L.entmax_attn_mfma_probe.argtypes = [vp, vp, ci, ci, vp]
        L.entmax_attn_coissue_probe.restype = ci
        L.entmax_attn_coissue_probe.argtypes = [vp, ci, ci, ci, vp]
        L.entmax_attn_strerror.restype = ctypes.c_char_p
        L.entmax_attn_strerror.argtypes = [ci]
        _lib = L
    return _lib


def entmax_attn_mask_tile():
    return int(lib().entmax_attn_mask_tile())


def entmax_attn_histogram_bins():
    return int(lib().entmax_attn_histogram_bins())


def entmax_attn_strerror(code):
    return lib().entmax_attn_strerror(int(code)).decode()


def entmax_attn_workspace_bytes(B, H, N, d, dtype, causal, is_bwd):
    return int(lib().entmax_attn_workspace_bytes(B, H, N, d, _dtype_code(dtype), int(bool(causal)), int(bool(is_bwd))))


def _dtype_code(dtype):
    if dtype in (torch.float32, "f32", EA_F32):
        return EA_F32
    if dtype in (torch.bfloat16, "bf16", EA_BF16):
        return EA_BF16
    return 99   # the library answers EA_ERR_DTYPE


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _check(rc):
    if rc != 0:
        text = entmax_attn_strerror(rc)
        if rc == -6:
            text += f" (hipError {lib().entmax_attn_last_hip_error()})"
        raise EntmaxAttnError(rc, text)


def _workspace(nbytes, device):
    # torch's caching allocator returns 512-byte aligned blocks
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _prep(*tensors):
    first = tensors[0]
    for t in tensors:
        if not t.is_cuda:
            raise ValueError("entmax_attn: tensors must live on the GPU (there is no CPU path)")
        if not t.is_contiguous() or t.shape != first.shape or t.dtype != first.dtype:
            raise ValueError("entmax_attn: Q, K, V, dO must be contiguous [B,H,N,d] of one dtype")
    return first.shape


def _alpha_array(alpha, H):
    """None for a single alpha; else a ctypes array of H floats (one alpha per head)."""
    if isinstance(alpha, (int, float)):
        return None
    vals = [float(a) for a in (alpha.tolist() if hasattr(alpha, "tolist") else alpha)]
    if len(vals) != H:
        raise ValueError(f"entmax_attn: {len(vals)} alphas for {H} heads")
    return (ctypes.c_float * H)(*vals)


def entmax_attn_fwd(Q, K, V, alpha, causal, want_iters=False, workspace=None):
    """-> (O, tau, block_mask) or (O, tau, block_mask, iters).  `alpha`: one float, or a sequence of
    H floats (one per head).  The workspace used is kept in `entmax_attn_fwd.last_workspace` so
    that read_stats() can fetch the tile counters."""
    B, H, N, d = _prep(Q, K, V)
    dev = Q.device
    T = N // 64 if N % 64 == 0 else 0
    O = torch.empty((B, H, N, d), dtype=torch.float32, device=dev)
    tau = torch.empty((B, H, N), dtype=torch.float32, device=dev)
    mask = torch.empty((B, H, max(T, 1), max((T + 31) // 32, 1)), dtype=torch.int32, device=dev)
    iters = torch.empty((B, H, N), dtype=torch.int32, device=dev) if want_iters else None
    nbytes = entmax_attn_workspace_bytes(B, H, N, d, Q.dtype, causal, False)
    ws = workspace if workspace is not None else _workspace(nbytes, dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    per_head = _alpha_array(alpha, H)
    if per_head is None:
        rc = lib().entmax_attn_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(tau), _ptr(mask), _ptr(iters),
                                   B, H, N, d, _dtype_code(Q.dtype), float(alpha), int(bool(causal)),
                                   _ptr(ws), ws.numel(), ctypes.c_void_p(stream))
    else:
        rc = lib().entmax_attn_fwd_alpha_per_head(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(tau), _ptr(mask), _ptr(iters),
                                                  B, H, N, d, _dtype_code(Q.dtype), per_head, int(bool(causal)),
                                                  _ptr(ws), ws.numel(), ctypes.c_void_p(stream))
    _check(rc)
    entmax_attn_fwd.last_workspace = ws
    return (O, tau, mask, iters) if want_iters else (O, tau, mask)


def entmax_attn_fwd_histogram_bounds(workspace, B, H, N, d, dtype):
    """-> (tau0, upper) [B,H,N]: what the histogram stage alone gave in the last forward call that
    used `workspace` (start of the refinement and upper end of its bracket, raw convention)."""
    dev = workspace.device
    tau0 = torch.empty((B, H, N), dtype=torch.float32, device=dev)
    upper = torch.empty_like(tau0)
    _check(lib().entmax_attn_fwd_histogram_bounds(_ptr(workspace), workspace.numel(), B, H, N, d, _dtype_code(dtype),
                                                  _ptr(tau0), _ptr(upper), ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)))
    return tau0, upper


def entmax_attn_bwd(Q, K, V, O, dO, tau, alpha, causal, block_mask=None, workspace=None, fwd_workspace=None):
    """-> (dQ, dK, dV).  block_mask=None makes the library rebuild the mask from tau.  fwd_workspace:
    the forward call's workspace (entmax_attn_bwd_with_lists: the supports the forward listed are
    used instead of being found again; single alpha only)."""
    B, H, N, d = _prep(Q, K, V, dO)
    dev = Q.device
    dQ = torch.empty((B, H, N, d), dtype=torch.float32, device=dev)
    dK = torch.empty_like(dQ)
    dV = torch.empty_like(dQ)
    nbytes = entmax_attn_workspace_bytes(B, H, N, d, Q.dtype, causal, True)
    ws = workspace if workspace is not None else _workspace(nbytes, dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    per_head = _alpha_array(alpha, H)
    if fwd_workspace is not None:
        if per_head is not None:
            raise ValueError("entmax_attn_bwd: fwd_workspace goes with a single alpha")
        rc = lib().entmax_attn_bwd_with_lists(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(tau), _ptr(block_mask),
                                              _ptr(fwd_workspace), fwd_workspace.numel(), _ptr(dQ), _ptr(dK), _ptr(dV),
                                              B, H, N, d, _dtype_code(Q.dtype), float(alpha), int(bool(causal)),
                                              _ptr(ws), ws.numel(), ctypes.c_void_p(stream))
    elif per_head is None:
        rc = lib().entmax_attn_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(tau), _ptr(block_mask),
                                   _ptr(dQ), _ptr(dK), _ptr(dV), B, H, N, d, _dtype_code(Q.dtype), float(alpha),
                                   int(bool(causal)), _ptr(ws), ws.numel(), ctypes.c_void_p(stream))
    else:
        rc = lib().entmax_attn_bwd_alpha_per_head(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(tau), _ptr(block_mask),
                                                  _ptr(dQ), _ptr(dK), _ptr(dV), B, H, N, d, _dtype_code(Q.dtype), per_head,
                                                  int(bool(causal)), _ptr(ws), ws.numel(), ctypes.c_void_p(stream))
    _check(rc)
    entmax_attn_bwd.last_workspace = ws
    return dQ, dK, dV


def entmax_attn_decode_workspace_bytes(B, H, N, d, dtype):
    return int(lib().entmax_attn_decode_workspace_bytes(B, H, N, d, _dtype_code(dtype)))


def entmax_attn_decode_static_max_bytes():
    return int(lib().entmax_attn_decode_static_max_bytes())


def entmax_attn_decode_static(q, K, V, alpha, out=None):
    """entmax_attn_decode through the entry point that allocates nothing: the scratch is the
    library's own static array.  `out` = (O, tau, support, iters) tensors to write into (then this
    function allocates nothing either); without it they are made here with torch."""
    B, H, N, d = _check_decode_args(q, K, V)
    dev = K.device
    O, tau, support, iters = out if out is not None else _decode_outputs(B, H, d, dev)
    _check(lib().entmax_attn_decode_static(_ptr(q), _ptr(K), _ptr(V), _ptr(O), _ptr(tau), _ptr(support), _ptr(iters),
                                           B, H, N, d, _dtype_code(K.dtype), float(alpha),
                                           ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)))
    return O, tau, support, iters


def _decode_outputs(B, H, d, dev):
    return (torch.empty((B, H, d), dtype=torch.float32, device=dev), torch.empty((B, H), dtype=torch.float32, device=dev),
            torch.empty((B, H), dtype=torch.int32, device=dev), torch.empty((B, H), dtype=torch.int32, device=dev))


def _check_decode_args(q, K, V):
    for t in (q, K, V):
        if not t.is_cuda:
            raise ValueError("entmax_attn_decode: tensors must live on the GPU (there is no CPU path)")
    if K.dim() != 4 or K.shape != V.shape or q.shape != K.shape[:2] + K.shape[3:] or not (
            q.is_contiguous() and K.is_contiguous() and V.is_contiguous()) or not (q.dtype == K.dtype == V.dtype):
        raise ValueError("entmax_attn_decode: q [B,H,d], K, V [B,H,N,d], contiguous, of one dtype")
    return K.shape


def entmax_attn_decode(q, K, V, alpha, workspace=None):
    """One query per head against all cached keys: q [B,H,d], K, V [B,H,N,d] -> (O [B,H,d], tau [B,H],
    support [B,H], iters [B,H])."""
    B, H, N, d = _check_decode_args(q, K, V)
    dev = K.device
    O, tau, support, iters = _decode_outputs(B, H, d, dev)
    ws = workspace if workspace is not None else _workspace(entmax_attn_decode_workspace_bytes(B, H, N, d, K.dtype), dev)
    _check(lib().entmax_attn_decode(_ptr(q), _ptr(K), _ptr(V), _ptr(O), _ptr(tau), _ptr(support), _ptr(iters),
                                    B, H, N, d, _dtype_code(K.dtype), float(alpha), _ptr(ws), ws.numel(),
                                    ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)))
    return O, tau, support, iters


def entmax_attn_mfma_probe(data, sink, groups, iters):
    """Enqueue the matrix-core rate probe on the current stream (data: >= 8192 fp16 values on the
    GPU, sink: >= groups * 256 floats). Returns the flops the launch performs."""
    if not (data.is_cuda and sink.is_cuda and data.dtype == torch.float16 and data.numel() >= 8192
            and sink.dtype == torch.float32 and sink.numel() >= groups * 256):
        raise ValueError("entmax_attn_mfma_probe: data = 8192 fp16 values, sink = groups * 256 floats, both on the GPU")
    _check(lib().entmax_attn_mfma_probe(_ptr(data), _ptr(sink), int(groups), int(iters),
                                         ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)))
    return float(groups) * 4 * iters * 32 * 32768.0


def entmax_attn_coissue_probe(sink, iters, valu_per_round, with_mfma):
    """Enqueue the co-issue probe on the current stream (sink: >= 512 * 512 floats on the GPU)."""
    if not (sink.is_cuda and sink.dtype == torch.float32 and sink.numel() >= 512 * 512):
        raise ValueError("entmax_attn_coissue_probe: sink = 512 * 512 floats on the GPU")
    _check(lib().entmax_attn_coissue_probe(_ptr(sink), int(iters), int(valu_per_round), int(bool(with_mfma)),
                                            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)))


def entmax_attn_right_edge_enable(on):
    """Approximate forward from right-edge binning, no refinement (this thread's later forward calls)."""
    _check(lib().entmax_attn_right_edge_enable(int(bool(on))))


def entmax_attn_gather_enable(on):
    _check(lib().entmax_attn_gather_enable(int(bool(on))))


def entmax_attn_timer_enable(on):
    _check(lib().entmax_attn_timer_enable(int(bool(on))))


def entmax_attn_timer_read():
    """-> {kernel name: (summed ms, launches)} since the last read (waits for the events)."""
    ms = (ctypes.c_float * EA_TIMER_SLOTS)()
    cnt = (ctypes.c_int * EA_TIMER_SLOTS)()
    _check(lib().entmax_attn_timer_read(ms, cnt, EA_TIMER_SLOTS))
    return {TIMER_NAMES[k]: (float(ms[k]), int(cnt[k])) for k in range(EA_TIMER_SLOTS) if cnt[k]}


def read_stats(workspace):
    """Executed-tile counters of the last call that used `workspace` (synchronises)."""
    copies = workspace[: EA_STATS_COPIES * EA_STATS_WORDS * 8].view(torch.int64).view(EA_STATS_COPIES, EA_STATS_WORDS)
    return dict(zip(STAT_NAMES, copies.cpu().sum(0).tolist()))
