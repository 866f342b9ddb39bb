"""ctypes binding of librtp.so -- argument marshalling only.

Every function has the name and argument order of its C entry point (see
include/rtp.h); tensors are torch tensors on the GPU (only their data_ptr() is
used), sizes are Python ints, and the HIP stream defaults to torch's current
stream.  A non-zero return code raises RtpError with the library's message.
There is no fallback: if the library cannot be loaded, importing succeeds but
the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("RTP_LIB", os.path.join(HERE, "librtp.so"))

RTP_OK, RTP_ERR_INVALID_ARG, RTP_ERR_UNSUPPORTED, RTP_ERR_WORKSPACE, RTP_ERR_HIP = 0, -1, -2, -3, -4

EXPORTS = [
    "rtp_last_error", "rtp_version", "rtp_profile_start", "rtp_profile_stop", "rtp_index_score_traffic_probe",
    "rtp_index_score",
    "rtp_topp_workspace_bytes", "rtp_topp_workspace_init", "rtp_topp_select", "rtp_topp_select_noalloc",
    "rtp_sparse_attn_decode_workspace_bytes", "rtp_sparse_attn_decode",
    "rtp_sparse_attn_prefill_workspace_bytes", "rtp_sparse_attn_prefill", "rtp_sparse_attn_prefill_tile_stats",
    "rtp_local_attn_workspace_bytes", "rtp_local_attn",
    "rtp_dense_attn_workspace_bytes", "rtp_dense_attn",
    "rtp_index_project", "rtp_topk_select",
    "rtp_block_topp_workspace_bytes", "rtp_block_topp_select", "rtp_sparsity_stats",
    "rtp_select_attend_decode_workspace_bytes", "rtp_select_attend_decode",
    "rtp_decode_attention", "rtp_decode_attention_paged", "rtp_sparse_attn_decode_paged",
    "rtp_kv_ring_heads", "rtp_kv_ring_append", "rtp_kv_ring_fill",
    "rtp_local_attn_ring_workspace_bytes", "rtp_local_attn_ring",
]
RTP_SIDE_QUERY, RTP_SIDE_KEY = 0, 1
RTP_DTYPE_BF16, RTP_DTYPE_FP16 = 0, 1


class RtpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"rtp error {code}: {msg}")
        self.code = code


class rtp_launch_time(C.Structure):
    _fields_ = [("kernel", C.c_char_p), ("us", C.c_float)]


class rtp_layer_desc(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("index_dim", C.c_int32),
        ("n_ret", C.c_int32), ("ret_heads", C.POINTER(C.c_int32)),
        ("sink", C.c_int32), ("window", C.c_int32),
        ("softmax_scale", C.c_float), ("index_scale", C.c_float), ("kv_dtype", C.c_int32),
    ]


def layer_desc(n_q_heads: int, n_kv_heads: int, ret_heads: Sequence[int], sink: int, window: int,
               head_dim: int = 128, index_dim: int = 16, softmax_scale: float = 0.0,
               index_scale: float = 0.0, kv_dtype: int = 0) -> rtp_layer_desc:
    arr = (C.c_int32 * max(len(ret_heads), 1))(*ret_heads)
    d = rtp_layer_desc(n_q_heads, n_kv_heads, head_dim, index_dim, len(ret_heads),
                       C.cast(arr, C.POINTER(C.c_int32)), sink, window, softmax_scale, index_scale, kv_dtype)
    d._keepalive = arr
    return d


_lib = None


def lib() -> C.CDLL:
    """Loads librtp.so (built by paper_2605_16928_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RtpError(-100, f"{LIB_PATH} is missing: build it with `python -m paper_2605_16928_amd.build` "
                             f"(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    dp = C.POINTER(rtp_layer_desc)
    L.rtp_last_error.restype = C.c_char_p
    L.rtp_last_error.argtypes = []
    L.rtp_version.restype = C.c_char_p
    L.rtp_version.argtypes = []
    L.rtp_index_score.restype = i32
    L.rtp_index_score.argtypes = [dp, vp, vp, vp, i64, vp, vp, vp, i32, i32, i64, vp, i64, vp, vp, sz, vp]
    L.rtp_topp_workspace_bytes.restype = sz
    L.rtp_topp_workspace_bytes.argtypes = [i32, i64]
    L.rtp_topp_select.restype = i32
    L.rtp_topp_select.argtypes = [vp, i64, vp, vp, i32, i64, vp, i64, vp, vp, vp, i32, vp, sz, vp]
    L.rtp_index_score_traffic_probe.restype = i32
    L.rtp_index_score_traffic_probe.argtypes = [dp, vp, vp, vp, i64, vp, vp, vp, i32, i32, i64, vp, i64, vp]
    L.rtp_profile_start.restype = i32
    L.rtp_profile_start.argtypes = [i32]
    L.rtp_profile_stop.restype = i32
    L.rtp_profile_stop.argtypes = [C.POINTER(rtp_launch_time), i32, C.POINTER(i32)]
    L.rtp_topp_select_noalloc.restype = i32
    L.rtp_topp_select_noalloc.argtypes = [vp, i64, vp, vp, i32, i64, vp, i64, vp, vp, vp, vp]
    L.rtp_topp_workspace_init.restype = i32
    L.rtp_topp_workspace_init.argtypes = [vp, sz, vp]
    L.rtp_sparse_attn_decode_workspace_bytes.restype = sz
    L.rtp_sparse_attn_decode_workspace_bytes.argtypes = [dp, i32, i64]
    L.rtp_sparse_attn_decode.restype = i32
    L.rtp_sparse_attn_decode.argtypes = [dp, vp, vp, vp, i64, i64, vp, vp, i64, vp, i64, i32, vp, vp, vp, sz, vp]
    L.rtp_sparse_attn_prefill_workspace_bytes.restype = sz
    L.rtp_sparse_attn_prefill_workspace_bytes.argtypes = [dp, i32, i64]
    L.rtp_sparse_attn_prefill_tile_stats.restype = i32
    L.rtp_sparse_attn_prefill_tile_stats.argtypes = [dp, i32, i64, vp, sz, vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    L.rtp_sparse_attn_prefill.restype = i32
    L.rtp_sparse_attn_prefill.argtypes = [dp, vp, vp, vp, vp, i64, vp, vp, i64, i64, i64, i32, C.c_float,
                                          vp, vp, vp, vp, vp, vp, sz, vp]
    for name in ("rtp_local_attn", "rtp_dense_attn"):
        getattr(L, name + "_workspace_bytes").restype = sz
        getattr(L, name + "_workspace_bytes").argtypes = [dp, i32, i32, i64]
        getattr(L, name).restype = i32
        getattr(L, name).argtypes = [dp, vp, vp, vp, i64, i64, vp, vp, vp, i32, i32, i64, vp, vp, vp, sz, vp]
    L.rtp_index_project.restype = i32
    L.rtp_index_project.argtypes = [dp, vp, vp, i32, i32, vp, i64, i64, vp]
    L.rtp_topk_select.restype = i32
    L.rtp_topk_select.argtypes = [vp, i64, vp, vp, i32, i64, vp, i64, vp, vp, vp, sz, vp]
    L.rtp_block_topp_workspace_bytes.restype = sz
    L.rtp_block_topp_workspace_bytes.argtypes = [i32, i64]
    L.rtp_block_topp_select.restype = i32
    L.rtp_block_topp_select.argtypes = [vp, i64, vp, vp, i32, i64, i32, C.c_float, C.c_float, vp, i64, vp, vp, vp,
                                        vp, i64, vp, sz, vp]
    L.rtp_select_attend_decode_workspace_bytes.restype = sz
    L.rtp_select_attend_decode_workspace_bytes.argtypes = [dp, i32, i64]
    L.rtp_select_attend_decode.restype = i32
    L.rtp_select_attend_decode.argtypes = [dp, vp, i64, vp, vp, i32, i64, vp, vp, vp, i64, i64, vp, vp, i64, vp, vp, vp,
                                           i32, vp, vp, vp, sz, vp, sz, vp]
    L.rtp_sparse_attn_decode_paged.restype = i32
    L.rtp_sparse_attn_decode_paged.argtypes = [dp, vp, vp, vp, i64, i64, vp, i64, i32, vp, i64, vp, i64, i32, vp, vp, vp, sz, vp]
    L.rtp_decode_attention.restype = i32
    L.rtp_decode_attention.argtypes = [dp, vp, i64, vp, vp, vp, i32, i64, vp, vp, vp, i64, i64, vp, vp, i64, vp, vp, vp,
                                       i32, vp, vp, vp, sz, vp, sz, vp, sz, vp]
    L.rtp_decode_attention_paged.restype = i32
    L.rtp_decode_attention_paged.argtypes = [dp, vp, i64, vp, vp, vp, i32, i64, vp, vp, vp, i64, i64, vp, i64, i32, vp, i64,
                                             vp, vp, vp, i32, vp, vp, vp, sz, vp, sz, vp, sz, vp]
    L.rtp_kv_ring_heads.restype = i32
    L.rtp_kv_ring_heads.argtypes = [dp, vp]
    L.rtp_kv_ring_append.restype = i32
    L.rtp_kv_ring_append.argtypes = [dp, vp, vp, vp, i32, vp, vp, i64, i64, vp, vp]
    L.rtp_kv_ring_fill.restype = i32
    L.rtp_kv_ring_fill.argtypes = [dp, vp, vp, i64, i64, vp, vp, i32, vp, vp, i64, i64, vp, vp]
    L.rtp_local_attn_ring_workspace_bytes.restype = sz
    L.rtp_local_attn_ring_workspace_bytes.argtypes = [dp, i32, i64]
    L.rtp_local_attn_ring.restype = i32
    L.rtp_local_attn_ring.argtypes = [dp, vp, vp, vp, i64, i64, vp, vp, vp, i64, i64, vp, vp, i32, i64, vp, vp, vp, sz, vp]
    L.rtp_sparsity_stats.restype = i32
    L.rtp_sparsity_stats.argtypes = [dp, vp, vp, i64, vp, vp, vp, i32, vp, vp, vp]
    _lib = L
    return L


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc: int):
    if rc != 0:
        raise RtpError(rc, lib().rtp_last_error().decode())


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def rtp_version() -> str:
    return lib().rtp_version().decode()


def rtp_last_error() -> str:
    return lib().rtp_last_error().decode()


def rtp_index_score(layer, q_in, WQ, kI, kI_head_stride, seq_start, ctx_len, q_start, B, n_q, max_ctx,
                    scores, score_stride, qI_out=None, topp_ws=None, stream=None):
    _check(lib().rtp_index_score(C.byref(layer), _ptr(q_in), _ptr(WQ), _ptr(kI), kI_head_stride, _ptr(seq_start),
                                 _ptr(ctx_len), _ptr(q_start), B, n_q, max_ctx, _ptr(scores), score_stride,
                                 _ptr(qI_out), _ptr(topp_ws), _nbytes(topp_ws), _stream(stream)))


def rtp_topp_workspace_bytes(R, max_len) -> int:
    return lib().rtp_topp_workspace_bytes(R, max_len)


def rtp_topp_workspace_init(ws, stream=None):
    _check(lib().rtp_topp_workspace_init(_ptr(ws), _nbytes(ws), _stream(stream)))


def rtp_topp_select(scores, score_stride, row_len, p, R, max_len, sel_idx, sel_stride, sel_count,
                    tau, mass, ws, level1_ready=0, stream=None):
    _check(lib().rtp_topp_select(_ptr(scores), score_stride, _ptr(row_len), _ptr(p), R, max_len, _ptr(sel_idx),
                                 sel_stride, _ptr(sel_count), _ptr(tau), _ptr(mass), level1_ready, _ptr(ws),
                                 _nbytes(ws), _stream(stream)))


def rtp_index_score_traffic_probe(layer, q_in, WQ, kI, kI_head_stride, seq_start, ctx_len, q_start, B, n_q, max_ctx,
                                  scores, score_stride, stream=None):
    _check(lib().rtp_index_score_traffic_probe(C.byref(layer), _ptr(q_in), _ptr(WQ), _ptr(kI), kI_head_stride,
                                               _ptr(seq_start), _ptr(ctx_len), _ptr(q_start), B, n_q, max_ctx,
                                               _ptr(scores), score_stride, _stream(stream)))


def rtp_profile_start(max_launches: int) -> None:
    _check(lib().rtp_profile_start(max_launches))


def rtp_profile_stop(max_launches: int = 1 << 16):
    """[(kernel name, microseconds)] of the launches recorded since rtp_profile_start, in launch order."""
    buf = (rtp_launch_time * max_launches)()
    n = C.c_int32(0)
    _check(lib().rtp_profile_stop(buf, max_launches, C.byref(n)))
    return [(buf[i].kernel.decode().strip("()"), float(buf[i].us)) for i in range(n.value)]


def rtp_topp_select_noalloc(scores, score_stride, row_len, p, R, max_len, sel_idx, sel_stride, sel_count,
                            tau, mass, stream=None):
    _check(lib().rtp_topp_select_noalloc(_ptr(scores), score_stride, _ptr(row_len), _ptr(p), R, max_len, _ptr(sel_idx),
                                         sel_stride, _ptr(sel_count), _ptr(tau), _ptr(mass), _stream(stream)))


def rtp_sparse_attn_decode_workspace_bytes(layer, B, max_sel) -> int:
    return lib().rtp_sparse_attn_decode_workspace_bytes(C.byref(layer), B, max_sel)


def rtp_sparse_attn_decode(layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, sel_idx, sel_stride,
                           sel_count, max_sel, B, out, lse, ws, stream=None):
    _check(lib().rtp_sparse_attn_decode(C.byref(layer), _ptr(q), _ptr(K), _ptr(V), kv_row_stride, kv_head_stride,
                                        _ptr(seq_start), _ptr(sel_idx), sel_stride, _ptr(sel_count), max_sel, B,
                                        _ptr(out), _ptr(lse), _ptr(ws), _nbytes(ws), _stream(stream)))


def rtp_select_attend_decode_workspace_bytes(layer, B, max_ctx) -> int:
    return lib().rtp_select_attend_decode_workspace_bytes(C.byref(layer), B, max_ctx)


def rtp_select_attend_decode(layer, scores, score_stride, row_len, p, B, max_ctx, q, K, V, kv_row_stride,
                             kv_head_stride, seq_start, sel_idx, sel_stride, sel_count, tau, mass, out, lse,
                             topp_ws, attn_ws, level1_ready=0, stream=None):
    _check(lib().rtp_select_attend_decode(C.byref(layer), _ptr(scores), score_stride, _ptr(row_len), _ptr(p), B,
                                          max_ctx, _ptr(q), _ptr(K), _ptr(V), kv_row_stride, kv_head_stride,
                                          _ptr(seq_start), _ptr(sel_idx), sel_stride, _ptr(sel_count), _ptr(tau),
                                          _ptr(mass), level1_ready, _ptr(out), _ptr(lse), _ptr(topp_ws),
                                          _nbytes(topp_ws), _ptr(attn_ws), _nbytes(attn_ws), _stream(stream)))


def rtp_sparse_attn_decode_paged(layer, q, K, V, kv_row_stride, kv_head_stride, page_table, pt_stride, page_size,
                                 sel_idx, sel_stride, sel_count, max_sel, B, out, lse, ws, stream=None):
    _check(lib().rtp_sparse_attn_decode_paged(C.byref(layer), _ptr(q), _ptr(K), _ptr(V), kv_row_stride, kv_head_stride,
                                              _ptr(page_table), pt_stride, page_size, _ptr(sel_idx), sel_stride,
                                              _ptr(sel_count), max_sel, B, _ptr(out), _ptr(lse), _ptr(ws), _nbytes(ws),
                                              _stream(stream)))


def rtp_decode_attention_paged(layer, scores, score_stride, row_len, p, ctx_len, B, max_ctx, q, K, V, kv_row_stride,
                               kv_head_stride, page_table, pt_stride, page_size, sel_idx, sel_stride, sel_count, tau, mass,
                               out, lse, topp_ws, attn_ws, local_ws, level1_ready=0, stream=None):
    _check(lib().rtp_decode_attention_paged(C.byref(layer), _ptr(scores), score_stride, _ptr(row_len), _ptr(p),
                                            _ptr(ctx_len), B, max_ctx, _ptr(q), _ptr(K), _ptr(V), kv_row_stride,
                                            kv_head_stride, _ptr(page_table), pt_stride, page_size, _ptr(sel_idx),
                                            sel_stride, _ptr(sel_count), _ptr(tau), _ptr(mass), level1_ready, _ptr(out),
                                            _ptr(lse), _ptr(topp_ws), _nbytes(topp_ws), _ptr(attn_ws), _nbytes(attn_ws),
                                            _ptr(local_ws), _nbytes(local_ws), _stream(stream)))


def rtp_decode_attention(layer, scores, score_stride, row_len, p, ctx_len, B, max_ctx, q, K, V, kv_row_stride,
                         kv_head_stride, seq_start, sel_idx, sel_stride, sel_count, tau, mass, out, lse,
                         topp_ws, attn_ws, local_ws, level1_ready=0, stream=None):
    _check(lib().rtp_decode_attention(C.byref(layer), _ptr(scores), score_stride, _ptr(row_len), _ptr(p), _ptr(ctx_len),
                                      B, max_ctx, _ptr(q), _ptr(K), _ptr(V), kv_row_stride, kv_head_stride,
                                      _ptr(seq_start), _ptr(sel_idx), sel_stride, _ptr(sel_count), _ptr(tau), _ptr(mass),
                                      level1_ready, _ptr(out), _ptr(lse), _ptr(topp_ws), _nbytes(topp_ws), _ptr(attn_ws),
                                      _nbytes(attn_ws), _ptr(local_ws), _nbytes(local_ws), _stream(stream)))


def rtp_kv_ring_heads(layer) -> list:
    """The KV heads whose query heads are all local (they may live in the bounded cache), ascending."""
    buf = (C.c_int32 * max(1, layer.n_kv_heads))()
    n = lib().rtp_kv_ring_heads(C.byref(layer), buf)
    if n < 0:
        raise RtpError(RTP_ERR_INVALID_ARG, lib().rtp_last_error().decode())
    return [int(buf[i]) for i in range(n)]


def rtp_kv_ring_append(layer, k_new, v_new, pos, B, ring_K, ring_V, ring_row_stride, ring_head_stride, ring_seq_start,
                       stream=None):
    _check(lib().rtp_kv_ring_append(C.byref(layer), _ptr(k_new), _ptr(v_new), _ptr(pos), B, _ptr(ring_K), _ptr(ring_V),
                                    ring_row_stride, ring_head_stride, _ptr(ring_seq_start), _stream(stream)))


def rtp_kv_ring_fill(layer, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len, B, ring_K, ring_V,
                     ring_row_stride, ring_head_stride, ring_seq_start, stream=None):
    _check(lib().rtp_kv_ring_fill(C.byref(layer), _ptr(K), _ptr(V), kv_row_stride, kv_head_stride, _ptr(seq_start),
                                  _ptr(ctx_len), B, _ptr(ring_K), _ptr(ring_V), ring_row_stride, ring_head_stride,
                                  _ptr(ring_seq_start), _stream(stream)))


def rtp_local_attn_ring_workspace_bytes(layer, B, max_ctx) -> int:
    return lib().rtp_local_attn_ring_workspace_bytes(C.byref(layer), B, max_ctx)


def rtp_local_attn_ring(layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ring_K, ring_V, ring_row_stride,
                        ring_head_stride, ring_seq_start, ctx_len, B, max_ctx, out, lse, ws, stream=None):
    _check(lib().rtp_local_attn_ring(C.byref(layer), _ptr(q), _ptr(K), _ptr(V), kv_row_stride, kv_head_stride,
                                     _ptr(seq_start), _ptr(ring_K), _ptr(ring_V), ring_row_stride, ring_head_stride,
                                     _ptr(ring_seq_start), _ptr(ctx_len), B, max_ctx, _ptr(out), _ptr(lse), _ptr(ws),
                                     _nbytes(ws), _stream(stream)))


def rtp_sparse_attn_prefill_workspace_bytes(layer, T, chunk_start) -> int:
    return lib().rtp_sparse_attn_prefill_workspace_bytes(C.byref(layer), T, chunk_start)


def rtp_sparse_attn_prefill(layer, q_pre, q, WQ, kI, kI_head_stride, K, V, kv_row_stride, kv_head_stride,
                            chunk_start, T, p, out, lse, tau, count, mass, ws, stream=None):
    _check(lib().rtp_sparse_attn_prefill(C.byref(layer), _ptr(q_pre), _ptr(q), _ptr(WQ), _ptr(kI), kI_head_stride,
                                         _ptr(K), _ptr(V), kv_row_stride, kv_head_stride, chunk_start, T, p,
                                         _ptr(out), _ptr(lse), _ptr(tau), _ptr(count), _ptr(mass), _ptr(ws),
                                         _nbytes(ws), _stream(stream)))


def rtp_sparse_attn_prefill_tile_stats(layer, T, chunk_start, ws, stream=None):
    """(tiles_visited, tiles_causal) of the last p < 1 call on this workspace."""
    vis, causal = C.c_int64(0), C.c_int64(0)
    _check(lib().rtp_sparse_attn_prefill_tile_stats(C.byref(layer), T, chunk_start, _ptr(ws), _nbytes(ws), _stream(stream),
                                                    C.byref(vis), C.byref(causal)))
    return vis.value, causal.value


def rtp_local_attn_workspace_bytes(layer, B, n_q, max_ctx) -> int:
    return lib().rtp_local_attn_workspace_bytes(C.byref(layer), B, n_q, max_ctx)


def rtp_dense_attn_workspace_bytes(layer, B, n_q, max_ctx) -> int:
    return lib().rtp_dense_attn_workspace_bytes(C.byref(layer), B, n_q, max_ctx)


def rtp_local_attn(layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len, q_start, B, n_q, max_ctx,
                   out, lse, ws, stream=None):
    _check(lib().rtp_local_attn(C.byref(layer), _ptr(q), _ptr(K), _ptr(V), kv_row_stride, kv_head_stride,
                                _ptr(seq_start), _ptr(ctx_len), _ptr(q_start), B, n_q, max_ctx, _ptr(out), _ptr(lse),
                                _ptr(ws), _nbytes(ws), _stream(stream)))


def rtp_dense_attn(layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len, q_start, B, n_q, max_ctx,
                   out, lse, ws, stream=None):
    _check(lib().rtp_dense_attn(C.byref(layer), _ptr(q), _ptr(K), _ptr(V), kv_row_stride, kv_head_stride,
                                _ptr(seq_start), _ptr(ctx_len), _ptr(q_start), B, n_q, max_ctx, _ptr(out), _ptr(lse),
                                _ptr(ws), _nbytes(ws), _stream(stream)))


def rtp_index_project(layer, W, x_pre, side, T, xI_out, out_head_stride, out_t0=0, stream=None):
    _check(lib().rtp_index_project(C.byref(layer), _ptr(W), _ptr(x_pre), side, T, _ptr(xI_out), out_head_stride,
                                   out_t0, _stream(stream)))


def rtp_topk_select(scores, score_stride, row_len, k, R, max_len, sel_idx, sel_stride, sel_count, tau, ws,
                    stream=None):
    _check(lib().rtp_topk_select(_ptr(scores), score_stride, _ptr(row_len), _ptr(k), R, max_len, _ptr(sel_idx),
                                 sel_stride, _ptr(sel_count), _ptr(tau), _ptr(ws), _nbytes(ws), _stream(stream)))


def rtp_block_topp_workspace_bytes(R, max_len) -> int:
    return lib().rtp_block_topp_workspace_bytes(R, max_len)


def rtp_block_topp_select(scores, score_stride, row_len, p, R, max_len, block, bin_lo, bin_width, sel_idx,
                          sel_stride, sel_count, threshold_bin, mass, block_mask, mask_stride, ws, stream=None):
    _check(lib().rtp_block_topp_select(_ptr(scores), score_stride, _ptr(row_len), _ptr(p), R, max_len, block,
                                       bin_lo, bin_width, _ptr(sel_idx), sel_stride, _ptr(sel_count),
                                       _ptr(threshold_bin), _ptr(mass), _ptr(block_mask), mask_stride,
                                       _ptr(ws), _nbytes(ws), _stream(stream)))


def rtp_sparsity_stats(layer, ctx_len, sel_idx, sel_stride, sel_count, lse_selected, lse_full, B, stats,
                       union_size=None, stream=None):
    _check(lib().rtp_sparsity_stats(C.byref(layer), _ptr(ctx_len), _ptr(sel_idx), sel_stride, _ptr(sel_count),
                                    _ptr(lse_selected), _ptr(lse_full), B, _ptr(stats), _ptr(union_size),
                                    _stream(stream)))
