"""Device-side drivers of the hot path: buffers for one workload and the C-ABI calls on them, in
the order a decode step (indexer scores -> top-p -> sparse attention, local heads beside them) or a
prefill chunk issues them.  Argument marshalling only; every computation happens in librtp.so."""
from __future__ import annotations

import numpy as np
import torch

from . import rtp, workloads as wl

DEV = "cuda:0"


def layer_desc_of(layer: wl.Layer):
    return rtp.layer_desc(layer.n_q_heads, layer.n_kv_heads, layer.ret_heads, layer.sink, layer.window,
                          softmax_scale=layer.softmax_scale, index_scale=layer.index_scale,
                          kv_dtype=rtp.RTP_DTYPE_FP16 if layer.kv_dtype == "fp16" else rtp.RTP_DTYPE_BF16)


def ws_alloc(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=DEV)


def i32(x):
    return torch.tensor(list(x), dtype=torch.int32, device=DEV)


def i64(x):
    return torch.tensor(list(x), dtype=torch.int64, device=DEV)


class DecodeRun:
    """Device buffers for one decode workload and the C-ABI calls on them."""

    def __init__(self, w: wl.DecodeWorkload, fuse_level1: bool = True, interleaved: bool = False):
        """fuse_level1: the score pass accumulates the selector's first histogram level (the
        configuration the benchmark times); False runs the two calls independently.
        interleaved: keep the K and V rows of a token next to each other ([Hkv, T, 2, 128], one
        512-byte piece per gathered token) instead of in two tensors; the workload's own K and V
        are released."""
        self.w = w
        self.fuse_level1 = fuse_level1
        if interleaved:
            self.kv = torch.stack([w.K, w.V], dim=2).contiguous()
            T = w.K.shape[1]
            self.Kp, self.Vp, self.kv_rs, self.kv_hs = self.kv.data_ptr(), self.kv.data_ptr() + 256, 256, T * 256
        else:
            self.Kp, self.Vp, self.kv_rs, self.kv_hs = w.K, w.V, 128, w.K.shape[1] * 128
        L = w.layer
        self.desc = layer_desc_of(L)
        self.B, self.n_ret = w.B, L.n_ret
        self.R = self.B * self.n_ret
        self.max_ctx = max(w.ctx_len)
        self.stride = (self.max_ctx + 3) // 4 * 4
        self.seq_start, self.ctx_len = i64(w.seq_start), i32(w.ctx_len)
        self.row_len = i32([w.ctx_len[b] for b in range(self.B) for _ in range(self.n_ret)])
        self.scores = torch.full((max(self.R, 1), self.stride), float("nan"), dtype=torch.float32, device=DEV)
        self.qI_out = torch.zeros((self.B, max(self.n_ret, 1), 16), dtype=torch.bfloat16, device=DEV)
        self.sel_idx = torch.full((max(self.R, 1), self.stride), -7, dtype=torch.int32, device=DEV)
        self.sel_count = torch.full((max(self.R, 1),), -7, dtype=torch.int32, device=DEV)
        self.tau = torch.zeros((max(self.R, 1),), dtype=torch.float32, device=DEV)
        self.mass = torch.zeros((max(self.R, 1),), dtype=torch.float32, device=DEV)
        self.out = torch.zeros((self.B, L.n_q_heads, 128), dtype=w.q.dtype, device=DEV)
        self.lse = torch.zeros((self.B, L.n_q_heads), dtype=torch.float32, device=DEV)
        self.ws_topp = ws_alloc(rtp.rtp_topp_workspace_bytes(max(self.R, 1), self.max_ctx))
        rtp.rtp_topp_workspace_init(self.ws_topp)
        self._level1_pending = False
        self._fork, self._join = (torch.cuda.Event(), torch.cuda.Event()) if torch.cuda.is_available() else (None, None)
        self.ws_sparse = ws_alloc(rtp.rtp_sparse_attn_decode_workspace_bytes(self.desc, self.B, self.max_ctx))
        self.ws_fused = ws_alloc(rtp.rtp_select_attend_decode_workspace_bytes(self.desc, self.B, self.max_ctx))
        self.ws_local = ws_alloc(rtp.rtp_local_attn_workspace_bytes(self.desc, self.B, 1, self.max_ctx))
        self.ws_dense = ws_alloc(rtp.rtp_dense_attn_workspace_bytes(self.desc, self.B, 1, self.max_ctx))
        self.T_tot = w.T_tot

    # ---- the five calls -------------------------------------------------------------------
    def index_score(self):
        w = self.w
        q_in = w.q_pre if w.WQ is not None else w.qI
        fuse = self.fuse_level1 and not self._level1_pending and self.R > 0
        rtp.rtp_index_score(self.desc, q_in, w.WQ, w.kI, self.T_tot * 16, self.seq_start, self.ctx_len, None,
                            self.B, 1, self.max_ctx, self.scores, self.stride, self.qI_out,
                            self.ws_topp if fuse else None)
        self._level1_pending = self._level1_pending or fuse

    def index_score_fused_timing(self, scratch):
        """The fused score pass on its own, for timing: level 1 goes to a scratch workspace."""
        w = self.w
        q_in = w.q_pre if w.WQ is not None else w.qI
        rtp.rtp_index_score(self.desc, q_in, w.WQ, w.kI, self.T_tot * 16, self.seq_start, self.ctx_len, None,
                            self.B, 1, self.max_ctx, self.scores, self.stride, self.qI_out, scratch)

    def index_score_plain_timing(self):
        """The score pass without the selector's histogram level, for timing."""
        w = self.w
        q_in = w.q_pre if w.WQ is not None else w.qI
        rtp.rtp_index_score(self.desc, q_in, w.WQ, w.kI, self.T_tot * 16, self.seq_start, self.ctx_len, None,
                            self.B, 1, self.max_ctx, self.scores, self.stride, self.qI_out, None)

    def index_score_traffic_probe(self, dst):
        """The score pass's loads and stores without its arithmetic (a measurement; dst gets meaningless words)."""
        w = self.w
        q_in = w.q_pre if w.WQ is not None else w.qI
        rtp.rtp_index_score_traffic_probe(self.desc, q_in, w.WQ, w.kI, self.T_tot * 16, self.seq_start, self.ctx_len, None,
                                          self.B, 1, self.max_ctx, dst, self.stride)

    def topp(self, scores=None, p_rows=None):
        s = self.scores if scores is None else scores
        p = self.w.p_rows if p_rows is None else p_rows
        ready = 1 if (self._level1_pending and scores is None) else 0
        rtp.rtp_topp_select(s, self.stride, self.row_len, p, self.R, self.max_ctx, self.sel_idx, self.stride,
                            self.sel_count, self.tau, self.mass, self.ws_topp, level1_ready=ready)
        if ready:
            self._level1_pending = False

    def topk(self, k: int):
        """Static top-k over the scores of the last index_score call (the fixed-budget rule)."""
        if not hasattr(self, "_k_rows") or self._k_val != k:
            self._k_rows, self._k_val = i32([k] * max(self.R, 1)), k
        rtp.rtp_topk_select(self.scores, self.stride, self.row_len, self._k_rows, self.R, self.max_ctx, self.sel_idx,
                            self.stride, self.sel_count, self.tau, self.ws_topp)

    def block_topp(self, bin_lo: float = -32.0, bin_width: float = 0.25):
        """Block-wise histogram top-p (blocks of 64) over the scores of the last index_score call."""
        if not hasattr(self, "ws_block"):
            self.ws_block = ws_alloc(rtp.rtp_block_topp_workspace_bytes(max(self.R, 1), self.max_ctx))
            self.thr_bin = torch.zeros((max(self.R, 1),), dtype=torch.int32, device=DEV)
        rtp.rtp_block_topp_select(self.scores, self.stride, self.row_len, self.w.p_rows, self.R, self.max_ctx, 64,
                                  bin_lo, bin_width, self.sel_idx, self.stride, self.sel_count, self.thr_bin,
                                  self.mass, None, 0, self.ws_block)

    def sparsity_stats(self, lse_full=None):
        """[B, 4] compute sparsity, memory sparsity, active tokens, attention mass of the current selection
        (the mass needs the log-sum-exps of the last sparse call in self.lse and of a dense call in lse_full)."""
        if not hasattr(self, "stats"):
            self.stats = torch.zeros((self.B, 4), dtype=torch.float32, device=DEV)
        rtp.rtp_sparsity_stats(self.desc, self.ctx_len, self.sel_idx, self.stride, self.sel_count,
                               self.lse if lse_full is not None else None, lse_full, self.B, self.stats)
        return self.stats

    def sparse_attn(self, sel_idx=None, sel_count=None, max_sel=None):
        w = self.w
        rtp.rtp_sparse_attn_decode(self.desc, w.q, self.Kp, self.Vp, self.kv_rs, self.kv_hs, self.seq_start,
                                   self.sel_idx if sel_idx is None else sel_idx, self.stride,
                                   self.sel_count if sel_count is None else sel_count,
                                   self.max_ctx if max_sel is None else max_sel, self.B, self.out, self.lse,
                                   self.ws_sparse)

    def select_attend(self):
        """Top-p selection and the retrieval heads' attention as one call (same outputs as topp() followed
        by sparse_attn())."""
        w = self.w
        ready = 1 if self._level1_pending else 0
        rtp.rtp_select_attend_decode(self.desc, self.scores, self.stride, self.row_len, w.p_rows, self.B, self.max_ctx,
                                     w.q, self.Kp, self.Vp, self.kv_rs, self.kv_hs, self.seq_start,
                                     self.sel_idx, self.stride, self.sel_count, self.tau, self.mass,
                                     self.out, self.lse, self.ws_topp, self.ws_fused, level1_ready=ready)
        if ready:
            self._level1_pending = False

    def decode_attention(self):
        """Everything of the step after the score pass as one call: selection, retrieval-head attention and the
        local heads (their work items travel inside the selector's launches)."""
        w = self.w
        ready = 1 if self._level1_pending else 0
        rtp.rtp_decode_attention(self.desc, self.scores, self.stride, self.row_len, w.p_rows, self.ctx_len, self.B,
                                 self.max_ctx, w.q, self.Kp, self.Vp, self.kv_rs, self.kv_hs, self.seq_start,
                                 self.sel_idx, self.stride, self.sel_count, self.tau, self.mass, self.out, self.lse,
                                 self.ws_topp, self.ws_fused, self.ws_local, level1_ready=ready)
        if ready:
            self._level1_pending = False

    def step_one_stream(self):
        """One decode step as two calls on one stream: the score pass, then rtp_decode_attention."""
        self.index_score()
        self.decode_attention()

    @property
    def carries_local_heads(self) -> bool:
        """Whether rtp_decode_attention carries the local heads inside the selector's launches for this layer
        (2, 4 or 8 query heads per KV head -- 8 only for small batches, see the library --, at least one
        retrieval and one local head); where it does not, the call still works and runs its parts in turn."""
        L = self.w.layer
        return L.n_q_heads // L.n_kv_heads in (2, 4, 8) and 0 < L.n_ret < L.n_q_heads

    def step_fastest(self, side: "torch.cuda.Stream"):
        """The step in the form the benchmark times: one stream where the local heads can be carried, else the
        local heads on a second stream."""
        if self.carries_local_heads:
            self.step_one_stream()
        else:
            self.step_two_streams(side)

    def local_attn(self, stream=None):
        w = self.w
        rtp.rtp_local_attn(self.desc, w.q, self.Kp, self.Vp, self.kv_rs, self.kv_hs, self.seq_start, self.ctx_len, None,
                           self.B, 1, self.max_ctx, self.out, self.lse, self.ws_local, stream=stream)

    def make_ring(self):
        """Bounded (sink + window rows) cache of the all-local KV heads, filled from the full cache."""
        L = self.w.layer
        self.ring_heads = rtp.rtp_kv_ring_heads(self.desc)
        cap = L.sink + L.window
        n = max(len(self.ring_heads), 1)
        self.ring_K = torch.zeros((n, self.B * cap, 128), dtype=torch.bfloat16, device=DEV)
        self.ring_V = torch.zeros_like(self.ring_K)
        self.ring_start = i64([b * cap for b in range(self.B)])
        self.ring_hs = self.B * cap * 128
        rtp.rtp_kv_ring_fill(self.desc, self.Kp, self.Vp, self.kv_rs, self.kv_hs, self.seq_start, self.ctx_len, self.B,
                             self.ring_K, self.ring_V, 128, self.ring_hs, self.ring_start)

    def ring_append(self, k_new, v_new, pos):
        rtp.rtp_kv_ring_append(self.desc, k_new, v_new, pos, self.B, self.ring_K, self.ring_V, 128, self.ring_hs,
                               self.ring_start)

    def local_attn_ring(self, stream=None):
        """local_attn with the bounded cache as the source of the all-local KV heads."""
        rtp.rtp_local_attn_ring(self.desc, self.w.q, self.Kp, self.Vp, self.kv_rs, self.kv_hs, self.seq_start,
                                self.ring_K, self.ring_V, 128, self.ring_hs, self.ring_start, self.ctx_len, self.B,
                                self.max_ctx, self.out, self.lse, self.ws_local, stream=stream)

    def dense_attn(self, out=None, lse=None):
        w = self.w
        rtp.rtp_dense_attn(self.desc, w.q, self.Kp, self.Vp, self.kv_rs, self.kv_hs, self.seq_start, self.ctx_len, None,
                           self.B, 1, self.max_ctx, self.out if out is None else out,
                           self.lse if lse is None else lse, self.ws_dense)

    def select_then_attend(self, fused: bool):
        if fused:
            self.select_attend()
        else:
            self.topp()
            self.sparse_attn()

    def step(self, fused: bool = True):
        """One decode step; fused: selection and retrieval-head attention as one call."""
        self.index_score()
        self.select_then_attend(fused)
        self.local_attn()

    def step_two_streams(self, side: "torch.cuda.Stream", fused: bool = True):
        """The same step with the local heads on a second stream: they do not depend on the
        indexer / top-p chain and write disjoint output rows."""
        main = torch.cuda.current_stream()
        # (the two events are made once and the side stream is passed to the call rather than made current:
        # the host has about as much to do per step as the GPU, so its share is kept small)
        fork, join = self._fork, self._join
        # the score pass saturates HBM on its own; the local heads start once it is done and overlap
        # the top-p launches, which leave HBM idle
        self.index_score()
        fork.record(main)
        side.wait_event(fork)
        self.local_attn(stream=side)
        join.record(side)
        self.select_then_attend(fused)
        main.wait_event(join)

    # ---- results as numpy -----------------------------------------------------------------
    def sel_sets(self):
        torch.cuda.synchronize()
        cnt = self.sel_count.cpu().numpy()
        idx = self.sel_idx.cpu().numpy()
        return [np.sort(idx[r, :max(cnt[r], 0)]) for r in range(self.R)], cnt

    def out_f64(self):
        torch.cuda.synchronize()
        return self.out.float().cpu().numpy().astype(np.float64)


class PrefillRun:
    """Device buffers for one prefill chunk of one sequence and the C-ABI calls on it."""

    def __init__(self, w: "wl.PrefillWorkload", interleaved: bool = False):
        self.w = w
        L = w.layer
        self.desc = layer_desc_of(L)
        self.seq_start, self.ctx_len, self.q_start = i64([0]), i32([w.N]), i32([w.chunk_start])
        self.out = torch.zeros((w.T, L.n_q_heads, 128), dtype=w.q.dtype, device=DEV)
        self.lse = torch.zeros((w.T, L.n_q_heads), dtype=torch.float32, device=DEV)
        self.tau = torch.zeros((max(L.n_ret, 1), w.T), dtype=torch.float32, device=DEV)
        self.mass = torch.zeros((max(L.n_ret, 1), w.T), dtype=torch.float32, device=DEV)
        self.count = torch.zeros((max(L.n_ret, 1), w.T), dtype=torch.int32, device=DEV)
        self.ws = ws_alloc(max(rtp.rtp_sparse_attn_prefill_workspace_bytes(self.desc, w.T, w.chunk_start),
                               rtp.rtp_local_attn_workspace_bytes(self.desc, 1, w.T, w.N)))
        if interleaved:
            self.kv = torch.cat([w.K, w.V], dim=2).contiguous()
            self.Kp, self.Vp, self.rs, self.hs = self.kv.data_ptr(), self.kv.data_ptr() + 256, 256, w.N * 256
        else:
            self.Kp, self.Vp, self.rs, self.hs = w.K, w.V, 128, w.N * 128

    def local_attn(self, out=None, lse=None):
        w = self.w
        rtp.rtp_local_attn(self.desc, w.q, self.Kp, self.Vp, self.rs, self.hs, self.seq_start, self.ctx_len,
                           self.q_start, 1, w.T, w.N, self.out if out is None else out,
                           self.lse if lse is None else lse, self.ws)

    def dense_attn(self, out=None, lse=None):
        w = self.w
        rtp.rtp_dense_attn(self.desc, w.q, self.Kp, self.Vp, self.rs, self.hs, self.seq_start, self.ctx_len,
                           self.q_start, 1, w.T, w.N, self.out if out is None else out,
                           self.lse if lse is None else lse, self.ws)

    def sparse_prefill(self, p=None, out=None, lse=None):
        w = self.w
        q_in = w.q_pre if w.WQ is not None else w.qI
        rtp.rtp_sparse_attn_prefill(self.desc, q_in, w.q, w.WQ, w.kI, w.N * 16, self.Kp, self.Vp, self.rs, self.hs,
                                    w.chunk_start, w.T, w.p if p is None else p, self.out if out is None else out,
                                    self.lse if lse is None else lse, self.tau, self.count, self.mass, self.ws)

    def tile_stats(self):
        """(64-key tiles visited, tiles of plain causal attention) of the last sparse_prefill call with p < 1."""
        return rtp.rtp_sparse_attn_prefill_tile_stats(self.desc, self.w.T, self.w.chunk_start, self.ws)
