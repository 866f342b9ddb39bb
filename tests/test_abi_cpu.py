"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
public header declares, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

from paper_2605_16928_amd import rtp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 0x10000  # a fake, well-aligned, non-NULL "device pointer": argument checks fail before any use


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rtp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rtp_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = rtp.lib()
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), f"{n} is declared in include/rtp.h but not exported"
    assert sorted(rtp.EXPORTS) == names
    assert rtp.rtp_version().startswith("rtp-gfx950")


def test_binding_has_one_function_per_entry_point():
    for n in declared_symbols():
        assert callable(getattr(rtp, n))


def _layer(**kw):
    d = dict(n_q_heads=8, n_kv_heads=2, ret_heads=[0, 4], sink=4, window=64)
    d.update(kw)
    return rtp.layer_desc(**d)


def _expect(code, fn, *a, **k):
    with pytest.raises(rtp.RtpError) as e:
        fn(*a, **k)
    assert e.value.code == code, str(e.value)
    assert rtp.rtp_last_error() != ""
    return str(e.value)


def test_layer_descriptor_checks():
    good = dict(q_in=A, WQ=None, kI=A, kI_head_stride=16 * 64, seq_start=A, ctx_len=A, q_start=None, B=1, n_q=1,
                max_ctx=64, scores=A, score_stride=64, qI_out=None, stream=0)
    call = lambda layer: rtp.rtp_index_score(layer, **good)
    assert "head_dim" in _expect(rtp.RTP_ERR_UNSUPPORTED, call, _layer(head_dim=64))
    assert "index_dim" in _expect(rtp.RTP_ERR_UNSUPPORTED, call, _layer(index_dim=32))
    _expect(rtp.RTP_ERR_INVALID_ARG, call, _layer(n_q_heads=6, n_kv_heads=4))
    _expect(rtp.RTP_ERR_UNSUPPORTED, call, _layer(n_q_heads=32, n_kv_heads=2))       # group of 16
    assert "ascending" in _expect(rtp.RTP_ERR_INVALID_ARG, call, _layer(ret_heads=[4, 0]))
    _expect(rtp.RTP_ERR_INVALID_ARG, call, _layer(ret_heads=[0, 8]))
    _expect(rtp.RTP_ERR_INVALID_ARG, call, _layer(sink=0, window=0))
    _expect(rtp.RTP_ERR_INVALID_ARG, call, _layer(sink=-1))


def test_index_score_argument_checks():
    L = _layer()
    good = dict(q_in=A, WQ=None, kI=A, kI_head_stride=16 * 64, seq_start=A, ctx_len=A, q_start=None, B=1, n_q=1,
                max_ctx=64, scores=A, score_stride=64, qI_out=None, stream=0)
    for k, v in [("q_in", None), ("kI", None), ("scores", None), ("B", 0), ("max_ctx", 0), ("n_q", 2),
                 ("score_stride", 63), ("score_stride", 66), ("scores", A + 4), ("kI_head_stride", 12),
                 ("max_ctx", (1 << 24) + 1)]:
        bad = dict(good)
        bad[k] = v
        if k == "max_ctx" and v > 64:
            bad["score_stride"] = v + 3
        _expect(rtp.RTP_ERR_INVALID_ARG, rtp.rtp_index_score, L, **bad)
    # a top-p workspace handed to the score pass must be large enough
    lib = rtp.lib()
    rc = lib.rtp_index_score(C.byref(L), C.c_void_p(A), None, C.c_void_p(A), 16 * 64, C.c_void_p(A), C.c_void_p(A), None,
                             1, 1, 64, C.c_void_p(A), 64, None, C.c_void_p(A), 256, None)
    assert rc == rtp.RTP_ERR_WORKSPACE


def test_topp_argument_and_workspace_checks():
    need = rtp.rtp_topp_workspace_bytes(4, 1000)
    assert need > 0 and need % 256 == 0
    assert rtp.rtp_topp_workspace_bytes(8, 1000) > need
    lib = rtp.lib()
    vp = C.c_void_p

    def call(scores=A, stride=1000, row_len=A, p=A, R=4, max_len=1000, sel=A, sel_stride=1000, cnt=A, ws=A,
             ws_bytes=need, ready=0):
        return lib.rtp_topp_select(vp(scores), stride, vp(row_len), vp(p), R, max_len, vp(sel), sel_stride, vp(cnt),
                                   None, None, ready, vp(ws), ws_bytes, None)

    assert call(scores=None) == rtp.RTP_ERR_INVALID_ARG
    assert call(R=0) == rtp.RTP_ERR_INVALID_ARG
    assert call(stride=999) == rtp.RTP_ERR_INVALID_ARG
    assert call(stride=1002) == rtp.RTP_ERR_INVALID_ARG
    assert call(sel_stride=999) == rtp.RTP_ERR_INVALID_ARG
    assert call(max_len=(1 << 24) + 4, stride=(1 << 24) + 4, sel_stride=(1 << 24) + 4) == rtp.RTP_ERR_INVALID_ARG
    assert call(ready=2) == rtp.RTP_ERR_INVALID_ARG
    assert call(ws=None) == rtp.RTP_ERR_WORKSPACE
    assert call(ws=A + 8) == rtp.RTP_ERR_WORKSPACE
    assert call(ws_bytes=need - 1) == rtp.RTP_ERR_WORKSPACE
    assert b"workspace" in lib.rtp_last_error()
    assert lib.rtp_topp_workspace_init(None, 1024, None) == rtp.RTP_ERR_WORKSPACE
    assert lib.rtp_topp_workspace_init(vp(A + 8), 1024, None) == rtp.RTP_ERR_WORKSPACE
    assert lib.rtp_topp_workspace_init(vp(A), 1023, None) == rtp.RTP_ERR_WORKSPACE


def test_attention_argument_and_workspace_checks():
    lib = rtp.lib()
    L = _layer()
    vp = C.c_void_p
    need = rtp.rtp_sparse_attn_decode_workspace_bytes(L, 2, 4096)
    assert need > 0 and need % 256 == 0

    def sparse(q=A, K=A, V=A, rs=128, hs=128 * 100, sel_stride=4096, max_sel=4096, B=2, ws=A, wsb=need, layer=L):
        return lib.rtp_sparse_attn_decode(C.byref(layer), vp(q), vp(K), vp(V), rs, hs, vp(A), vp(A), sel_stride, vp(A),
                                          max_sel, B, vp(A), None, vp(ws), wsb, None)

    assert sparse(q=None) == rtp.RTP_ERR_INVALID_ARG
    assert sparse(rs=64) == rtp.RTP_ERR_INVALID_ARG
    assert sparse(rs=132) == rtp.RTP_ERR_INVALID_ARG
    assert sparse(K=A + 2) == rtp.RTP_ERR_INVALID_ARG
    assert sparse(sel_stride=100) == rtp.RTP_ERR_INVALID_ARG
    assert sparse(B=0) == rtp.RTP_ERR_INVALID_ARG
    assert sparse(wsb=need - 256) == rtp.RTP_ERR_WORKSPACE
    assert sparse(ws=None) == rtp.RTP_ERR_WORKSPACE
    assert sparse(B=1000, wsb=1 << 40) == rtp.RTP_ERR_UNSUPPORTED          # more rows than one plan holds

    for name in ("rtp_local_attn", "rtp_dense_attn"):
        fn = getattr(lib, name)
        need2 = getattr(rtp, name + "_workspace_bytes")(L, 2, 1, 4096)
        assert need2 > 0 and need2 % 256 == 0

        def rng(q=A, n_q=1, q_start=None, ws=A, wsb=need2, max_ctx=4096, ctx=A):
            return fn(C.byref(L), vp(q), vp(A), vp(A), 128, 128 * 100, vp(A), vp(ctx), vp(q_start), 2, n_q, max_ctx,
                      vp(A), None, vp(ws), wsb, None)

        assert rng(q=None) == rtp.RTP_ERR_INVALID_ARG
        assert rng(n_q=2) == rtp.RTP_ERR_INVALID_ARG           # decode mode takes one query per sequence
        assert rng(n_q=0) == rtp.RTP_ERR_INVALID_ARG
        assert rng(ctx=None) == rtp.RTP_ERR_INVALID_ARG
        assert rng(max_ctx=0) == rtp.RTP_ERR_INVALID_ARG
        assert rng(wsb=0) == rtp.RTP_ERR_WORKSPACE


def test_widened_entry_points_argument_checks():
    lib = rtp.lib()
    L = _layer()
    vp = C.c_void_p
    # index-key build
    proj = lambda W=A, x=A, side=rtp.RTP_SIDE_KEY, T=8, out=A, hs=16 * 64, t0=0: lib.rtp_index_project(
        C.byref(L), vp(W), vp(x), side, T, vp(out), hs, t0, None)
    assert proj(W=None) == rtp.RTP_ERR_INVALID_ARG
    assert proj(side=2) == rtp.RTP_ERR_INVALID_ARG
    assert proj(T=0) == rtp.RTP_ERR_INVALID_ARG
    assert proj(x=A + 8) == rtp.RTP_ERR_INVALID_ARG
    assert proj(hs=6) == rtp.RTP_ERR_INVALID_ARG
    assert proj(t0=-1) == rtp.RTP_ERR_INVALID_ARG
    # static top-k shares the top-p workspace rule
    need = rtp.rtp_topp_workspace_bytes(4, 1000)
    topk = lambda scores=A, k=A, ws=A, wsb=need, R=4: lib.rtp_topk_select(
        vp(scores), 1000, vp(A), vp(k), R, 1000, vp(A), 1000, vp(A), None, vp(ws), wsb, None)
    assert topk(k=None) == rtp.RTP_ERR_INVALID_ARG
    assert topk(scores=None) == rtp.RTP_ERR_INVALID_ARG
    assert topk(R=0) == rtp.RTP_ERR_INVALID_ARG
    assert topk(wsb=need - 1) == rtp.RTP_ERR_WORKSPACE
    # block-wise selector
    needb = rtp.rtp_block_topp_workspace_bytes(4, 1000)
    assert needb > 0 and needb % 256 == 0 and rtp.rtp_block_topp_workspace_bytes(4, 100000) > needb
    blk = lambda scores=A, block=64, lo=-32.0, width=0.25, mask=None, mstride=0, ws=A, wsb=needb: lib.rtp_block_topp_select(
        vp(scores), 1000, vp(A), vp(A), 4, 1000, block, lo, width, vp(A), 1000, vp(A), None, None, vp(mask), mstride,
        vp(ws), wsb, None)
    assert blk(scores=None) == rtp.RTP_ERR_INVALID_ARG
    assert blk(block=32) == rtp.RTP_ERR_UNSUPPORTED
    assert blk(width=0.0) == rtp.RTP_ERR_INVALID_ARG
    assert blk(width=float("nan")) == rtp.RTP_ERR_INVALID_ARG
    assert blk(mask=A, mstride=3) == rtp.RTP_ERR_INVALID_ARG
    assert blk(ws=None) == rtp.RTP_ERR_WORKSPACE
    assert blk(wsb=needb - 1) == rtp.RTP_ERR_WORKSPACE
    # sparsity figures
    st = lambda ctx=A, sel=A, cnt=A, ls=None, lf=None, B=2, out=A: lib.rtp_sparsity_stats(
        C.byref(L), vp(ctx), vp(sel), 1000, vp(cnt), vp(ls), vp(lf), B, vp(out), None, None)
    assert st(ctx=None) == rtp.RTP_ERR_INVALID_ARG
    assert st(sel=None) == rtp.RTP_ERR_INVALID_ARG
    assert st(ls=A) == rtp.RTP_ERR_INVALID_ARG             # one log-sum-exp array without the other
    assert st(B=0) == rtp.RTP_ERR_INVALID_ARG
    assert st(out=None) == rtp.RTP_ERR_INVALID_ARG
    # selection + attention in one call: both workspaces and both argument groups are checked
    needt = rtp.rtp_topp_workspace_bytes(2 * 2, 1000)
    needa = rtp.rtp_select_attend_decode_workspace_bytes(L, 2, 1000)
    assert needa > 0 and needa % 256 == 0
    assert rtp.rtp_select_attend_decode_workspace_bytes(L, 2, 100000) > needa
    fa = lambda scores=A, p=A, q=A, rs=128, B=2, tws=A, twsb=needt, aws=A, awsb=needa: lib.rtp_select_attend_decode(
        C.byref(L), vp(scores), 1000, vp(A), vp(p), B, 1000, vp(q), vp(A), vp(A), rs, 128 * 1000, vp(A),
        vp(A), 1000, vp(A), None, None, 0, vp(A), None, vp(tws), twsb, vp(aws), awsb, None)
    assert fa(scores=None) == rtp.RTP_ERR_INVALID_ARG
    assert fa(p=None) == rtp.RTP_ERR_INVALID_ARG
    assert fa(q=None) == rtp.RTP_ERR_INVALID_ARG
    assert fa(q=A + 8) == rtp.RTP_ERR_INVALID_ARG
    assert fa(rs=100) == rtp.RTP_ERR_INVALID_ARG
    assert fa(B=0) == rtp.RTP_ERR_INVALID_ARG
    assert fa(aws=None) == rtp.RTP_ERR_WORKSPACE
    assert fa(awsb=needa - 1) == rtp.RTP_ERR_WORKSPACE
    assert fa(twsb=needt - 1) == rtp.RTP_ERR_WORKSPACE
    # ... and with the local heads in the same call
    needl = rtp.rtp_local_attn_workspace_bytes(L, 2, 1, 1000)
    da = lambda scores=A, ctx=A, q=A, aws=A, awsb=needa, lws=A, lwsb=needl, twsb=needt: lib.rtp_decode_attention(
        C.byref(L), vp(scores), 1000, vp(A), vp(A), vp(ctx), 2, 1000, vp(q), vp(A), vp(A), 128, 128 * 1000, vp(A),
        vp(A), 1000, vp(A), None, None, 0, vp(A), None, vp(A), twsb, vp(aws), awsb, vp(lws), lwsb, None)
    assert da(scores=None) == rtp.RTP_ERR_INVALID_ARG
    assert da(ctx=None) == rtp.RTP_ERR_INVALID_ARG
    assert da(q=A + 2) == rtp.RTP_ERR_INVALID_ARG
    assert da(aws=None) == rtp.RTP_ERR_WORKSPACE
    assert da(lws=None) == rtp.RTP_ERR_WORKSPACE
    assert da(lwsb=needl - 1) == rtp.RTP_ERR_WORKSPACE
    assert da(twsb=needt - 1) == rtp.RTP_ERR_WORKSPACE


def test_bounded_cache_entry_points_host_side():
    lib = rtp.lib()
    vp = C.c_void_p
    # which KV heads may live in the bounded cache: computed on the host
    assert rtp.rtp_kv_ring_heads(rtp.layer_desc(n_q_heads=32, n_kv_heads=8, ret_heads=[0, 8, 16, 24], sink=4, window=64)) == [1, 3, 5, 7]
    assert rtp.rtp_kv_ring_heads(_layer()) == []                     # both KV heads serve a retrieval head
    assert rtp.rtp_kv_ring_heads(_layer(ret_heads=[])) == [0, 1]
    L = rtp.layer_desc(n_q_heads=8, n_kv_heads=4, ret_heads=[0, 5], sink=4, window=64)
    assert rtp.rtp_kv_ring_heads(L) == [1, 3]
    app = lambda k=A, pos=A, B=2, rk=A, rs=128, hs=128 * 200, rss=A, layer=L: lib.rtp_kv_ring_append(
        C.byref(layer), vp(k), vp(A), vp(pos), B, vp(rk), vp(A), rs, hs, vp(rss), None)
    assert app(k=None) == rtp.RTP_ERR_INVALID_ARG
    assert app(pos=None) == rtp.RTP_ERR_INVALID_ARG
    assert app(B=0) == rtp.RTP_ERR_INVALID_ARG
    assert app(rk=None) == rtp.RTP_ERR_INVALID_ARG
    assert app(rk=A + 4) == rtp.RTP_ERR_INVALID_ARG
    assert app(rs=100) == rtp.RTP_ERR_INVALID_ARG
    assert app(rss=None) == rtp.RTP_ERR_INVALID_ARG
    assert app(layer=rtp.layer_desc(n_q_heads=8, n_kv_heads=4, ret_heads=[0, 5], sink=4, window=0)) == rtp.RTP_ERR_INVALID_ARG
    fill = lambda K=A, krs=128, ctx=A, B=2, rk=A: lib.rtp_kv_ring_fill(
        C.byref(L), vp(K), vp(A), krs, 128 * 1000, vp(A), vp(ctx), B, vp(rk), vp(A), 128, 128 * 200, vp(A), None)
    assert fill(K=None) == rtp.RTP_ERR_INVALID_ARG
    assert fill(krs=64) == rtp.RTP_ERR_INVALID_ARG
    assert fill(ctx=None) == rtp.RTP_ERR_INVALID_ARG
    assert fill(B=0) == rtp.RTP_ERR_INVALID_ARG
    assert fill(rk=None) == rtp.RTP_ERR_INVALID_ARG
    need = rtp.rtp_local_attn_ring_workspace_bytes(L, 2, 1000)
    assert need == rtp.rtp_local_attn_workspace_bytes(L, 2, 1, 1000)
    att = lambda q=A, rk=A, rrs=128, ws=A, wsb=need: lib.rtp_local_attn_ring(
        C.byref(L), vp(q), vp(A), vp(A), 128, 128 * 1000, vp(A), vp(rk), vp(A), rrs, 128 * 200, vp(A), vp(A), 2, 1000,
        vp(A), None, vp(ws), wsb, None)
    assert att(q=None) == rtp.RTP_ERR_INVALID_ARG
    assert att(rk=None) == rtp.RTP_ERR_INVALID_ARG
    assert att(rrs=120) == rtp.RTP_ERR_INVALID_ARG
    assert att(ws=None) == rtp.RTP_ERR_WORKSPACE
    assert att(wsb=need - 1) == rtp.RTP_ERR_WORKSPACE


def test_paged_sparse_attention_argument_checks():
    lib = rtp.lib()
    L = _layer()
    vp = C.c_void_p
    need = rtp.rtp_sparse_attn_decode_workspace_bytes(L, 2, 1000)
    pg = lambda pt=A, pts=16, ps=64, K=A, sel=A, ws=A, wsb=need: lib.rtp_sparse_attn_decode_paged(
        C.byref(L), vp(A), vp(K), vp(A), 128, 128 * 4096, vp(pt), pts, ps, vp(sel), 1000, vp(A), 1000, 2, vp(A), None,
        vp(ws), wsb, None)
    assert pg(pt=None) == rtp.RTP_ERR_INVALID_ARG
    assert pg(ps=48) == rtp.RTP_ERR_INVALID_ARG              # not a power of two
    assert pg(ps=8) == rtp.RTP_ERR_INVALID_ARG               # below 16
    assert pg(pts=15) == rtp.RTP_ERR_INVALID_ARG             # 15 pages of 64 do not cover 1000 tokens
    assert pg(K=None) == rtp.RTP_ERR_INVALID_ARG
    assert pg(sel=None) == rtp.RTP_ERR_INVALID_ARG
    assert pg(ws=None) == rtp.RTP_ERR_WORKSPACE
    assert pg(wsb=need - 1) == rtp.RTP_ERR_WORKSPACE


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    monkeypatch.setattr(rtp, "_lib", None)
    monkeypatch.setattr(rtp, "LIB_PATH", "/nonexistent/librtp.so")
    with pytest.raises(rtp.RtpError):
        rtp.rtp_version()


def test_prefill_calls_reject_a_row_stride_beyond_the_tile_offset_range():
    """The prefill kernels address a lane's place inside a 64-row tile with 32 bits: kv_row_stride above 2^24
    elements is refused before anything is launched."""
    lib = rtp.lib()
    L = _layer()
    vp = C.c_void_p
    need = rtp.rtp_dense_attn_workspace_bytes(L, 1, 64, 4096)

    def dense(rs):
        return lib.rtp_dense_attn(C.byref(L), vp(A), vp(A), vp(A), rs, 1 << 40, vp(A), vp(A), vp(A), 1, 64, 4096,
                                  vp(A), None, vp(A), need, None)

    assert dense((1 << 24) + 8) == rtp.RTP_ERR_INVALID_ARG
    assert "2^24" in rtp.rtp_last_error()


def test_decode_range_calls_refuse_more_than_1024_units():
    """The range-source decode calls plan at most 1024 (sequence, KV head) units per call: a larger batch is
    refused as unsupported before anything is launched (the header states the limit)."""
    lib = rtp.lib()
    L = _layer()                      # 2 KV heads
    vp = C.c_void_p
    for name in ("rtp_local_attn", "rtp_dense_attn"):
        fn = getattr(lib, name)
        ok_B, bad_B = 512, 513
        assert fn(C.byref(L), vp(A), vp(A), vp(A), 128, 128 * 100, vp(A), vp(A), None, bad_B, 1, 4096,
                  vp(A), None, vp(A), 1 << 40, None) == rtp.RTP_ERR_UNSUPPORTED
        assert "exceeds 1024" in rtp.rtp_last_error()
        assert getattr(rtp, name + "_workspace_bytes")(L, ok_B, 1, 4096) > 0


def test_sparse_prefill_refuses_an_oversized_chunk_before_any_launch():
    """T beyond what one launch's grid holds is an argument error like the others: with index projections given
    (WQ != NULL) the call must not have enqueued its projection launch first -- the pointers here are fake, a
    launch would fault."""
    lib = rtp.lib()
    L = _layer()
    vp = C.c_void_p
    T = 128 * 65535 + 1
    rc = lib.rtp_sparse_attn_prefill(C.byref(L), vp(A), vp(A), vp(A), vp(A), 16 * 64, vp(A), vp(A), 128, 1 << 40,
                                     0, T, C.c_float(0.9), vp(A), None, None, None, None, vp(A), 1 << 50, None)
    assert rc == rtp.RTP_ERR_INVALID_ARG and b"too large" in lib.rtp_last_error()


def test_paged_decode_attention_and_dtype_argument_checks():
    lib = rtp.lib()
    vp = C.c_void_p
    L = _layer()
    _expect(rtp.RTP_ERR_UNSUPPORTED, lambda: rtp.rtp_index_score(_layer(kv_dtype=7), q_in=A, WQ=None, kI=A, kI_head_stride=1024,
                                                                  seq_start=A, ctx_len=A, q_start=None, B=1, n_q=1, max_ctx=64,
                                                                  scores=A, score_stride=64, qI_out=None, stream=0))
    assert "kv_dtype" in rtp.rtp_last_error()
    ws = 1 << 30

    def call(table=A, page_size=64, pt_stride=64, q=A):
        return lib.rtp_decode_attention_paged(C.byref(L), vp(A), 4096, vp(A), vp(A), vp(A), 2, 4096, vp(q), vp(A), vp(A), 128,
                                              128 * 100, vp(table), pt_stride, page_size, vp(A), 4096, vp(A), None, None, 0,
                                              vp(A), None, vp(A), ws, vp(A), ws, vp(A), ws, None)

    assert call(table=None) == rtp.RTP_ERR_INVALID_ARG
    assert call(page_size=48) == rtp.RTP_ERR_INVALID_ARG and b"power of two" in lib.rtp_last_error()
    assert call(page_size=8) == rtp.RTP_ERR_INVALID_ARG
    assert call(pt_stride=63) == rtp.RTP_ERR_INVALID_ARG and b"pt_stride" in lib.rtp_last_error()
    assert call(q=None) == rtp.RTP_ERR_INVALID_ARG


def test_prefill_tile_statistics_argument_checks():
    """rtp_sparse_attn_prefill_tile_stats checks its arguments and the workspace size before it touches the
    device (the pointers here are fake)."""
    lib = rtp.lib()
    L = _layer()
    vp = C.c_void_p
    vis, causal = C.c_int64(-1), C.c_int64(-1)
    need = lib.rtp_sparse_attn_prefill_workspace_bytes(C.byref(L), 300, 3000)
    assert need > 0
    rc = lib.rtp_sparse_attn_prefill_tile_stats(C.byref(L), 0, 3000, vp(A), need, None, C.byref(vis), C.byref(causal))
    assert rc == rtp.RTP_ERR_INVALID_ARG
    rc = lib.rtp_sparse_attn_prefill_tile_stats(C.byref(L), 300, 3000, vp(A), need, None, None, C.byref(causal))
    assert rc == rtp.RTP_ERR_INVALID_ARG
    rc = lib.rtp_sparse_attn_prefill_tile_stats(C.byref(L), 300, 3000, vp(A), need - 256, None, C.byref(vis), C.byref(causal))
    assert rc == rtp.RTP_ERR_WORKSPACE and b"workspace" in lib.rtp_last_error()
    rc = lib.rtp_sparse_attn_prefill_tile_stats(C.byref(L), 300, 3000, None, need, None, C.byref(vis), C.byref(causal))
    assert rc == rtp.RTP_ERR_WORKSPACE
    # a layer without retrieval heads has nothing to visit
    L0 = _layer(ret_heads=[])
    rc = lib.rtp_sparse_attn_prefill_tile_stats(C.byref(L0), 300, 3000, None, 0, None, C.byref(vis), C.byref(causal))
    assert rc == rtp.RTP_OK and vis.value == 0 and causal.value == 0
