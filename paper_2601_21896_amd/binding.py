"""ctypes binding of libpafu.so: argument marshalling only.

Every function here has the name and the argument order of its C entry point in
include/pafu.h; tensors are torch CUDA(HIP) tensors whose data pointers are handed
over unchanged.  There is no fallback: if the library is missing or a call fails,
an exception is raised.
"""

from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, c_char_p, c_float, c_int, c_longlong, c_size_t, c_void_p)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpafu.so")

PAFU_BF16, PAFU_F32, PAFU_FP8_E4M3 = 0, 1, 2
PAFU_ACT_SILU, PAFU_ACT_GELU_ERF = 0, 1
PAFU_MODE_SINGLE, PAFU_MODE_ROLLOUT = 0, 1

SYMBOLS = (
    "pafu_strerror", "pafu_last_hip_error", "pafu_version", "pafu_study_build", "pafu_launch_probe",
    "pafu_score_workspace_bytes", "pafu_score", "pafu_score_static",
    "pafu_select_workspace_bytes", "pafu_select_topk", "pafu_select_topk_pinned",
    "pafu_compact_kv", "pafu_compact_kv_counted",
    "pafu_attention_workspace_bytes", "pafu_chunk_attention", "pafu_chunk_attention_gather",
    "pafu_quantize_kv", "pafu_dequantize_kv", "pafu_chunk_attention_fp8",
    "pafu_sse_workspace_bytes", "pafu_sse_score",
    "pafu_step_workspace_bytes", "pafu_step", "pafu_step_layers", "pafu_step_layers_shared",
)


class PafuError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().pafu_strerror(status).decode()
        if status == -7:
            msg += " (hipError %d)" % _lib().pafu_last_hip_error()
        super().__init__("%s failed: %s [%d]" % (where, msg, status))


class pafu_step_args(Structure):
    _fields_ = [
        ("mode", c_int), ("N", c_int), ("D", c_int), ("n", c_int), ("Lc", c_int), ("k", c_int),
        ("block_len", c_int), ("M", c_int), ("n_out", c_int), ("act", c_int), ("n_seg", c_int),
        ("Fs", c_int), ("x_dtype", c_int), ("out_dtype", c_int), ("softmax_scale", c_float),
        ("ld_x", c_longlong), ("ld_cache", c_longlong), ("ld_out", c_longlong),
        ("ld_chunk", c_longlong), ("ld_o", c_longlong),
        ("x_cache", c_void_p * 3), ("x_chunk", c_void_p * 3),
        ("W1", c_void_p), ("b1", c_void_p), ("W2", c_void_p), ("b2", c_void_p),
        ("K_cache", c_void_p), ("V_cache", c_void_p), ("SL_in", c_void_p),
        ("Q", c_void_p), ("K_chunk", c_void_p), ("V_chunk", c_void_p),
        ("scores", c_void_p), ("ids", c_void_p), ("K_out", c_void_p), ("V_out", c_void_p),
        ("SL_out", c_void_p), ("O", c_void_p), ("workspace", c_void_p), ("workspace_bytes", c_size_t),
        ("n_pinned", c_int),
        ("stage_events", c_void_p * 5),
        ("kv_dtype", c_int), ("k_scale_log2", c_int), ("v_scale_log2", c_int),
    ]


_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libpafu.so is not built (%s); run `python -c 'import __graft_entry__ as g; g.build()'` "
                "or `python -m paper_2601_21896_amd.build`" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        lib.pafu_strerror.restype = c_char_p
        lib.pafu_strerror.argtypes = [c_int]
        lib.pafu_last_hip_error.restype = c_int
        lib.pafu_version.restype = c_int
        lib.pafu_study_build.restype = c_int
        lib.pafu_launch_probe.restype = c_int
        lib.pafu_launch_probe.argtypes = [c_void_p]
        lib.pafu_score_workspace_bytes.restype = c_size_t
        lib.pafu_score_workspace_bytes.argtypes = [c_int]
        lib.pafu_score.restype = c_int
        lib.pafu_score.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_longlong, c_int,
                                   c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_void_p, c_void_p,
                                   c_size_t]
        lib.pafu_score_static.restype = c_int
        lib.pafu_score_static.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_longlong, c_int,
                                          c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_void_p]
        lib.pafu_select_workspace_bytes.restype = c_size_t
        lib.pafu_select_workspace_bytes.argtypes = [c_int]
        lib.pafu_select_topk.restype = c_int
        lib.pafu_select_topk.argtypes = [c_void_p, c_void_p, c_int, c_int, c_void_p, c_void_p, c_void_p, c_size_t]
        lib.pafu_select_topk_pinned.restype = c_int
        lib.pafu_select_topk_pinned.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p,
                                                c_size_t]
        lib.pafu_compact_kv.restype = c_int
        lib.pafu_compact_kv.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_longlong, c_int, c_void_p, c_int,
                                        c_int, c_int, c_int, c_void_p, c_void_p, c_void_p, c_longlong]
        lib.pafu_compact_kv_counted.restype = c_int
        lib.pafu_compact_kv_counted.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_longlong, c_int, c_void_p,
                                                c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p,
                                                c_longlong]
        lib.pafu_attention_workspace_bytes.restype = c_size_t
        lib.pafu_attention_workspace_bytes.argtypes = [c_int, c_int, c_int]
        lib.pafu_chunk_attention.restype = c_int
        lib.pafu_chunk_attention.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_int, c_void_p, c_void_p,
                                             c_int, c_int, c_int, c_longlong, c_longlong, c_longlong, c_longlong,
                                             c_int, c_float, c_void_p, c_int, c_void_p, c_size_t]
        lib.pafu_chunk_attention_gather.restype = c_int
        lib.pafu_chunk_attention_gather.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_int, c_void_p,
                                                    c_int, c_void_p, c_void_p, c_int, c_int, c_int, c_longlong,
                                                    c_longlong, c_longlong, c_longlong, c_int, c_float, c_void_p,
                                                    c_int, c_void_p, c_size_t]
        for f in (lib.pafu_quantize_kv, lib.pafu_dequantize_kv):
            f.restype = c_int
            f.argtypes = [c_void_p, c_void_p, c_void_p, c_longlong, c_int, c_int, c_int, c_int, c_int, c_void_p,
                          c_void_p, c_longlong]
        lib.pafu_chunk_attention_fp8.restype = c_int
        lib.pafu_chunk_attention_fp8.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_int, c_void_p,
                                                 c_void_p, c_int, c_int, c_int, c_longlong, c_longlong, c_longlong,
                                                 c_longlong, c_int, c_float, c_int, c_int, c_void_p, c_int, c_void_p,
                                                 c_size_t]
        lib.pafu_step_workspace_bytes.restype = c_size_t
        lib.pafu_step_workspace_bytes.argtypes = [POINTER(pafu_step_args)]
        lib.pafu_step.restype = c_int
        lib.pafu_step.argtypes = [c_void_p, POINTER(pafu_step_args)]
        lib.pafu_step_layers.restype = c_int
        lib.pafu_step_layers.argtypes = [c_void_p, POINTER(pafu_step_args), c_int]
        lib.pafu_sse_workspace_bytes.restype = c_size_t
        lib.pafu_sse_workspace_bytes.argtypes = [c_int, c_int]
        lib.pafu_sse_score.restype = c_int
        lib.pafu_sse_score.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_longlong, c_longlong, c_int,
                                       c_float, c_void_p, c_void_p, c_size_t]
        lib.pafu_step_layers_shared.restype = c_int
        lib.pafu_step_layers_shared.argtypes = [c_void_p, POINTER(pafu_step_args), c_int, c_int]
        _LIB = lib
    return _LIB


def library():
    """The loaded ctypes library (raises if it is not built)."""
    return _lib()


def _ptr(t):
    """Device pointer of a torch tensor (None -> NULL); raw ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return PAFU_BF16
    if t.dtype == torch.float32:
        return PAFU_F32
    raise TypeError("unsupported dtype %s" % t.dtype)


def _check(rc, where):
    if rc != 0:
        raise PafuError(rc, where)


def pafu_version() -> int:
    return _lib().pafu_version()


def pafu_strerror(status: int) -> str:
    return _lib().pafu_strerror(status).decode()


def pafu_study_build() -> int:
    return _lib().pafu_study_build()


def pafu_launch_probe(stream=None):
    _check(_lib().pafu_launch_probe(_stream(stream)), "pafu_launch_probe")


def set_stage_events(args: "pafu_step_args", events):
    """Attaches up to five timing events (torch.cuda.Event objects that have been recorded once, or raw hipEvent_t
    handles, or None) to a step's argument struct."""
    keep = []
    for i in range(5):
        e = events[i] if i < len(events) else None
        if e is None:
            args.stage_events[i] = None
        elif isinstance(e, int):
            args.stage_events[i] = e
        else:
            handle = e.cuda_event
            if not handle:
                raise ValueError("record the event once before attaching it (its handle is created lazily)")
            args.stage_events[i] = handle
            keep.append(e)
    args._keep_events = keep


def pafu_score_workspace_bytes(M: int) -> int:
    return _lib().pafu_score_workspace_bytes(M)


def pafu_score(x_segs, W1, b1, W2, b2, out, act=PAFU_ACT_SILU, workspace=None, stream=None, T=None):
    """x_segs: one tensor [T, Fs] or a tuple of up to three (feature-axis concatenation)."""
    if not isinstance(x_segs, (tuple, list)):
        x_segs = (x_segs,)
    x0 = x_segs[0]
    T = x0.shape[0] if T is None else T
    Fs = x0.shape[1]
    M, n_out = W1.shape[0], W2.shape[0]
    ptrs = [_ptr(x) for x in x_segs] + [None] * (3 - len(x_segs))
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib().pafu_score(_stream(stream), ptrs[0], ptrs[1], ptrs[2], len(x_segs), T, Fs, x0.stride(0),
                           _dtype_code(x0), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), M, n_out, act, _ptr(out),
                           _ptr(workspace), ws_bytes)
    _check(rc, "pafu_score")
    return out


def pafu_score_static(x_segs, W1, b1, W2, b2, out, act=PAFU_ACT_SILU, stream=None, T=None):
    """pafu_score without a workspace: the library's static device scratch holds the folded second layer."""
    if not isinstance(x_segs, (tuple, list)):
        x_segs = (x_segs,)
    x0 = x_segs[0]
    T = x0.shape[0] if T is None else T
    ptrs = [_ptr(x) for x in x_segs] + [None] * (3 - len(x_segs))
    rc = _lib().pafu_score_static(_stream(stream), ptrs[0], ptrs[1], ptrs[2], len(x_segs), T, x0.shape[1],
                                  x0.stride(0), _dtype_code(x0), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), W1.shape[0],
                                  W2.shape[0], act, _ptr(out))
    _check(rc, "pafu_score_static")
    return out


def pafu_select_workspace_bytes(n: int) -> int:
    return _lib().pafu_select_workspace_bytes(n)


def pafu_select_topk(scores, k, out_ids, out_count=None, workspace=None, stream=None, n=None):
    n = scores.shape[0] if n is None else n
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib().pafu_select_topk(_stream(stream), _ptr(scores), n, k, _ptr(out_ids), _ptr(out_count),
                                 _ptr(workspace), ws_bytes)
    _check(rc, "pafu_select_topk")
    return out_ids


def pafu_select_topk_pinned(scores, k, n_pinned, out_ids, out_count=None, workspace=None, stream=None, n=None):
    n = scores.shape[0] if n is None else n
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib().pafu_select_topk_pinned(_stream(stream), _ptr(scores), n, k, n_pinned, _ptr(out_ids),
                                        _ptr(out_count), _ptr(workspace), ws_bytes)
    _check(rc, "pafu_select_topk_pinned")
    return out_ids


def pafu_compact_kv(K, V, SL, ids, count, K_out, V_out, SL_out, stream=None, n=None):
    n = K.shape[0] if n is None else n
    N, D = K.shape[1], K.shape[2]
    rc = _lib().pafu_compact_kv(_stream(stream), _ptr(K), _ptr(V), _ptr(SL), K.stride(0), n, _ptr(ids), count, N, D,
                                _dtype_code(K), _ptr(K_out), _ptr(V_out), _ptr(SL_out), K_out.stride(0))
    _check(rc, "pafu_compact_kv")
    return K_out, V_out, SL_out


def pafu_compact_kv_counted(K, V, SL, ids, count_dev, max_count, K_out, V_out, SL_out, stream=None, n=None):
    """pafu_compact_kv with the row count in a device int32 tensor (as written by pafu_select_topk)."""
    n = K.shape[0] if n is None else n
    N, D = K.shape[1], K.shape[2]
    rc = _lib().pafu_compact_kv_counted(_stream(stream), _ptr(K), _ptr(V), _ptr(SL), K.stride(0), n, _ptr(ids),
                                        _ptr(count_dev), max_count, N, D, _dtype_code(K), _ptr(K_out), _ptr(V_out),
                                        _ptr(SL_out), K_out.stride(0))
    _check(rc, "pafu_compact_kv_counted")
    return K_out, V_out, SL_out


def pafu_attention_workspace_bytes(Lq: int, N: int, D: int) -> int:
    return _lib().pafu_attention_workspace_bytes(Lq, N, D)


def pafu_chunk_attention(Q, Kc, Vc, n_kept, Kn, Vn, block_len, O, softmax_scale=0.0, workspace=None, stream=None):
    Lq, N, D = Q.shape
    Lc = Kn.shape[0]
    ld_c = Kc.stride(0) if Kc is not None else N * D
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib().pafu_chunk_attention(_stream(stream), _ptr(Q), Lq, _ptr(Kc), _ptr(Vc), n_kept, _ptr(Kn), _ptr(Vn),
                                     Lc, N, D, Q.stride(0), ld_c, Kn.stride(0), O.stride(0), block_len,
                                     float(softmax_scale), _ptr(O), _dtype_code(O), _ptr(workspace), ws_bytes)
    _check(rc, "pafu_chunk_attention")
    return O


def pafu_chunk_attention_gather(Q, K_cache, V_cache, ids, n_kept, Kn, Vn, block_len, O, softmax_scale=0.0,
                                workspace=None, stream=None):
    Lq, N, D = Q.shape
    Lc = Kn.shape[0]
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib().pafu_chunk_attention_gather(_stream(stream), _ptr(Q), Lq, _ptr(K_cache), _ptr(V_cache),
                                            K_cache.shape[0], _ptr(ids), n_kept, _ptr(Kn), _ptr(Vn), Lc, N, D,
                                            Q.stride(0), K_cache.stride(0), Kn.stride(0), O.stride(0), block_len,
                                            float(softmax_scale), _ptr(O), _dtype_code(O), _ptr(workspace), ws_bytes)
    _check(rc, "pafu_chunk_attention_gather")
    return O


def pafu_quantize_kv(K, V, k_scale_log2, v_scale_log2, K_q, V_q, stream=None, rows=None):
    """K, V: [rows, N, D] bf16 -> K_q, V_q: [rows, N * D] uint8 E4M3 codes of value / 2^scale_log2."""
    rows = K.shape[0] if rows is None else rows
    N, D = K.shape[1], K.shape[2]
    rc = _lib().pafu_quantize_kv(_stream(stream), _ptr(K), _ptr(V), K.stride(0), rows, N, D, k_scale_log2, v_scale_log2,
                                 _ptr(K_q), _ptr(V_q), K_q.stride(0))
    _check(rc, "pafu_quantize_kv")
    return K_q, V_q


def pafu_dequantize_kv(K_q, V_q, k_scale_log2, v_scale_log2, K, V, stream=None, rows=None):
    """The exact way back: K, V [rows, N, D] bf16 = code * 2^scale_log2."""
    rows = K.shape[0] if rows is None else rows
    N, D = K.shape[1], K.shape[2]
    rc = _lib().pafu_dequantize_kv(_stream(stream), _ptr(K_q), _ptr(V_q), K_q.stride(0), rows, N, D, k_scale_log2,
                                   v_scale_log2, _ptr(K), _ptr(V), K.stride(0))
    _check(rc, "pafu_dequantize_kv")
    return K, V


def pafu_chunk_attention_fp8(Q, Kc_q, Vc_q, n_kept, Kn_q, Vn_q, block_len, k_scale_log2, v_scale_log2, O,
                             softmax_scale=0.0, workspace=None, stream=None):
    """Q [Lq, N, D] bf16; Kc_q / Vc_q [n_kept, N * D] and Kn_q / Vn_q [Lc, N * D] uint8 codes."""
    Lq, N, D = Q.shape
    Lc = Kn_q.shape[0]
    ld_c = Kc_q.stride(0) if Kc_q is not None else N * D
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib().pafu_chunk_attention_fp8(_stream(stream), _ptr(Q), Lq, _ptr(Kc_q), _ptr(Vc_q), n_kept, _ptr(Kn_q),
                                         _ptr(Vn_q), Lc, N, D, Q.stride(0), ld_c, Kn_q.stride(0), O.stride(0), block_len,
                                         float(softmax_scale), k_scale_log2, v_scale_log2, _ptr(O), _dtype_code(O),
                                         _ptr(workspace), ws_bytes)
    _check(rc, "pafu_chunk_attention_fp8")
    return O


def make_step_args(mode, N, D, n, Lc, k, block_len, x_cache, x_chunk, W1, b1, W2, b2, K_cache, V_cache, SL_in, Q,
                   K_chunk, V_chunk, scores, ids, K_out, V_out, SL_out, O, act=PAFU_ACT_SILU, workspace=None,
                   softmax_scale=0.0, n_pinned=0, kv_dtype=PAFU_BF16, k_scale_log2=0, v_scale_log2=0) -> pafu_step_args:
    """Fills a pafu_step_args from torch tensors (x_cache / x_chunk: tensor or tuple of segments)."""
    a = pafu_step_args()
    xs_cache = x_cache if isinstance(x_cache, (tuple, list)) else ((x_cache,) if x_cache is not None else ())
    xs_chunk = x_chunk if isinstance(x_chunk, (tuple, list)) else (x_chunk,)
    a.mode, a.N, a.D, a.n, a.Lc, a.k, a.block_len = mode, N, D, n, Lc, k, block_len
    a.M, a.n_out, a.act = W1.shape[0], W2.shape[0], act
    a.n_seg, a.Fs = len(xs_chunk), xs_chunk[0].shape[1]
    a.x_dtype, a.out_dtype = _dtype_code(xs_chunk[0]), _dtype_code(O)
    a.softmax_scale = float(softmax_scale)
    a.n_pinned = int(n_pinned)
    a.kv_dtype, a.k_scale_log2, a.v_scale_log2 = int(kv_dtype), int(k_scale_log2), int(v_scale_log2)
    a.ld_x = xs_chunk[0].stride(0)
    a.ld_cache = K_cache.stride(0) if K_cache is not None else N * D
    a.ld_out = K_out.stride(0)
    a.ld_chunk = Q.stride(0)
    a.ld_o = O.stride(0)
    for i in range(3):
        a.x_cache[i] = _ptr(xs_cache[i]) if i < len(xs_cache) else None
        a.x_chunk[i] = _ptr(xs_chunk[i]) if i < len(xs_chunk) else None
    a.W1, a.b1, a.W2, a.b2 = _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2)
    a.K_cache, a.V_cache, a.SL_in = _ptr(K_cache), _ptr(V_cache), _ptr(SL_in)
    a.Q, a.K_chunk, a.V_chunk = _ptr(Q), _ptr(K_chunk), _ptr(V_chunk)
    a.scores, a.ids = _ptr(scores), _ptr(ids)
    a.K_out, a.V_out, a.SL_out, a.O = _ptr(K_out), _ptr(V_out), _ptr(SL_out), _ptr(O)
    a.workspace = _ptr(workspace)
    a.workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    # the struct holds raw device pointers; keep the tensors alive for as long as the struct lives
    a._keep = (xs_cache, xs_chunk, W1, b1, W2, b2, K_cache, V_cache, SL_in, Q, K_chunk, V_chunk, scores, ids, K_out,
               V_out, SL_out, O, workspace)
    return a


def pafu_step_workspace_bytes(args: pafu_step_args) -> int:
    return _lib().pafu_step_workspace_bytes(ctypes.byref(args))


def pafu_step(args: pafu_step_args, stream=None):
    _check(_lib().pafu_step(_stream(stream), ctypes.byref(args)), "pafu_step")


def pafu_step_layers(args_list, stream=None):
    arr = (pafu_step_args * len(args_list))(*args_list)
    _check(_lib().pafu_step_layers(_stream(stream), arr, len(args_list)), "pafu_step_layers")


def pafu_step_layers_shared(args_list, index_layer, stream=None):
    arr = (pafu_step_args * len(args_list))(*args_list)
    _check(_lib().pafu_step_layers_shared(_stream(stream), arr, len(args_list), index_layer),
           "pafu_step_layers_shared")


def pafu_sse_workspace_bytes(L: int, N: int) -> int:
    return _lib().pafu_sse_workspace_bytes(L, N)


def pafu_sse_score(Q, K, block_len, out, workspace, softmax_scale=0.0, stream=None):
    """Q, K: [L, N, D] bf16; out: [L] fp32; workspace: at least pafu_sse_workspace_bytes(L, N) bytes."""
    L, N, D = Q.shape
    rc = _lib().pafu_sse_score(_stream(stream), _ptr(Q), _ptr(K), L, N, D, Q.stride(0), K.stride(0), block_len,
                               float(softmax_scale), _ptr(out), _ptr(workspace),
                               workspace.numel() * workspace.element_size())
    _check(rc, "pafu_sse_score")
    return out
