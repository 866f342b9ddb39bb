"""Helpers shared by the GPU parity tests: run the decode path through the C-ABI on cuda:0,
hand the same inputs to the oracle, and compare with the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

from oracle import rtp_oracle as orc
from paper_2605_16928_amd import rtp, workloads as wl

DEV = "cuda:0"

# tolerances (benchmark spec; forms fixed here)
SCORE_RTOL = 1e-5          # |d| <= 1e-5 * max(|s_ref|, sum_i |qI_i kI_i|)
BAND_RTOL = 1e-5           # tokens with |s - tau| <= 1e-5 * max(1, |tau|) may differ
OUT_ATOL, OUT_RTOL = 2e-2, 1e-2


def layer_desc_of(layer: wl.Layer):
    return rtp.layer_desc(layer.n_q_heads, layer.n_kv_heads, layer.ret_heads, layer.sink, layer.window)


def ws_alloc(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=DEV)


def i32(x):
    return torch.tensor(list(x), dtype=torch.int32, device=DEV)


def i64(x):
    return torch.tensor(list(x), dtype=torch.int64, device=DEV)


class DecodeRun:
    """Device buffers for one decode workload and the C-ABI calls on them."""

    def __init__(self, w: wl.DecodeWorkload, fuse_level1: bool = True):
        """fuse_level1: the score pass accumulates the selector's first histogram level (the
        configuration the benchmark times); False runs the two calls independently."""
        self.w = w
        self.fuse_level1 = fuse_level1
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
        self.out = torch.zeros((self.B, L.n_q_heads, 128), dtype=torch.bfloat16, device=DEV)
        self.lse = torch.zeros((self.B, L.n_q_heads), dtype=torch.float32, device=DEV)
        self.ws_topp = ws_alloc(rtp.rtp_topp_workspace_bytes(max(self.R, 1), self.max_ctx))
        rtp.rtp_topp_workspace_init(self.ws_topp)
        self._level1_pending = False
        self.ws_sparse = ws_alloc(rtp.rtp_sparse_attn_decode_workspace_bytes(self.desc, self.B, self.max_ctx))
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

    def topp(self, scores=None, p_rows=None):
        s = self.scores if scores is None else scores
        p = self.w.p_rows if p_rows is None else p_rows
        ready = 1 if (self._level1_pending and scores is None) else 0
        rtp.rtp_topp_select(s, self.stride, self.row_len, p, self.R, self.max_ctx, self.sel_idx, self.stride,
                            self.sel_count, self.tau, self.mass, self.ws_topp, level1_ready=ready)
        if ready:
            self._level1_pending = False

    def sparse_attn(self, sel_idx=None, sel_count=None, max_sel=None):
        w = self.w
        rtp.rtp_sparse_attn_decode(self.desc, w.q, w.K, w.V, 128, self.T_tot * 128, self.seq_start,
                                   self.sel_idx if sel_idx is None else sel_idx, self.stride,
                                   self.sel_count if sel_count is None else sel_count,
                                   self.max_ctx if max_sel is None else max_sel, self.B, self.out, self.lse,
                                   self.ws_sparse)

    def local_attn(self):
        w = self.w
        rtp.rtp_local_attn(self.desc, w.q, w.K, w.V, 128, self.T_tot * 128, self.seq_start, self.ctx_len, None,
                           self.B, 1, self.max_ctx, self.out, self.lse, self.ws_local)

    def dense_attn(self, out=None, lse=None):
        w = self.w
        rtp.rtp_dense_attn(self.desc, w.q, w.K, w.V, 128, self.T_tot * 128, self.seq_start, self.ctx_len, None,
                           self.B, 1, self.max_ctx, self.out if out is None else out,
                           self.lse if lse is None else lse, self.ws_dense)

    def step(self):
        self.index_score()
        self.topp()
        self.sparse_attn()
        self.local_attn()

    def step_two_streams(self, side: "torch.cuda.Stream"):
        """The same step with the local heads on a second stream: they do not depend on the
        indexer / top-p chain and write disjoint output rows."""
        main = torch.cuda.current_stream()
        fork, join = torch.cuda.Event(), torch.cuda.Event()
        # the score pass saturates HBM on its own; the local heads start once it is done and overlap
        # the top-p launches, which leave HBM idle
        self.index_score()
        fork.record(main)
        side.wait_event(fork)
        with torch.cuda.stream(side):
            self.local_attn()
            join.record(side)
        self.topp()
        self.sparse_attn()
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


def oracle_inputs(w: wl.DecodeWorkload) -> dict:
    L = w.layer
    d = dict(q_bits=wl.bf16_bits(w.q), K_bits=wl.bf16_bits(w.K), V_bits=wl.bf16_bits(w.V),
             kI_bits=wl.bf16_bits(w.kI), seq_start=w.seq_start, ctx_len=w.ctx_len,
             n_q_heads=L.n_q_heads, n_kv_heads=L.n_kv_heads, ret_heads=L.ret_heads, sink=L.sink,
             window=L.window, p_rows=w.p_rows.cpu().numpy().astype(np.float64))
    if w.WQ is not None:
        d.update(WQ=w.WQ.cpu().numpy(), q_pre_bits=wl.bf16_bits(w.q_pre))
    else:
        d.update(qI_bits=wl.bf16_bits(w.qI))
    return d


# ---- comparators ------------------------------------------------------------------------------
def check_scores(s_gpu: np.ndarray, s_ref: np.ndarray, qI_bits, kI_bits, what=""):
    q = orc.bf16_to_f64(qI_bits)
    k = orc.bf16_to_f64(kI_bits)
    mag = np.abs(k) @ np.abs(q)
    tol = SCORE_RTOL * np.maximum(np.abs(s_ref), mag)
    bad = np.abs(s_gpu.astype(np.float64) - s_ref) > tol
    assert not bad.any(), f"{what}: {bad.sum()} scores outside 1e-5 relative; worst {np.abs(s_gpu - s_ref).max()}"


def check_selection(sel_gpu: np.ndarray, s: np.ndarray, ref: dict, p: float, what=""):
    """`s`: the float64 scores the reference selection `ref` was computed from."""
    tau = ref["tau"]
    band = np.abs(s - tau) <= BAND_RTOL * max(1.0, abs(tau))
    g = np.zeros(s.shape[0], dtype=bool)
    g[sel_gpu] = True
    r = np.zeros(s.shape[0], dtype=bool)
    r[ref["idx"]] = True
    diff = (g != r) & ~band
    assert not diff.any(), (f"{what}: {diff.sum()} tokens outside the threshold band differ "
                            f"(gpu {g.sum()} vs ref {r.sum()} tokens, tau {tau})")
    w = np.exp(s - s.max())
    Z = w.sum()
    assert w[g].sum() / Z >= p - 1e-6, f"{what}: selected mass {w[g].sum() / Z} below p={p}"
    assert w[g & ~band].sum() / Z < p + 1e-6, f"{what}: selection is not minimal"
    assert len(np.unique(sel_gpu)) == len(sel_gpu), f"{what}: duplicate indices"


def check_selection_valid(sel_gpu: np.ndarray, s: np.ndarray, p: float, slack: float, what=""):
    """End-to-end form: the GPU chose its set from ITS fp32 scores, `s` are the oracle's fp64 scores
    (they differ by up to `slack`).  The set must still be a top-p set of `s` up to that slack:
    upward closed in score, mass >= p, and not reaching p without its lowest-scored band."""
    g = np.zeros(s.shape[0], dtype=bool)
    g[sel_gpu] = True
    tau_g = s[g].min()
    band = BAND_RTOL * max(1.0, abs(tau_g)) + 2.0 * slack
    missing = (~g) & (s > tau_g + band)
    assert not missing.any(), f"{what}: {missing.sum()} tokens above the threshold band are not selected"
    w = np.exp(s - s.max())
    Z = w.sum()
    assert w[g].sum() / Z >= p - 1e-6, f"{what}: selected mass {w[g].sum() / Z} below p={p}"
    assert w[g & (s > tau_g + band)].sum() / Z < p + 1e-6, f"{what}: selection is not minimal"


def check_out(o_gpu: np.ndarray, o_ref: np.ndarray, what="", tight=True):
    """The stated bar is 2e-2 absolute + 1e-2 relative.  `tight` additionally holds the kernels to
    what their arithmetic should give: True = fp32 accumulation + one bf16 rounding of the output
    (1e-3 + 2^-8*|ref|, the decode kernels); "mfma" = probabilities also rounded to bf16 before the
    PV product (6e-3 + 2^-7*|ref|, the prefill kernels)."""
    err = np.abs(o_gpu - o_ref)
    tol = OUT_ATOL + OUT_RTOL * np.abs(o_ref)
    assert (err <= tol).all(), f"{what}: max abs err {err.max()} (tolerance 2e-2 + 1e-2*|ref|)"
    if tight:
        tol = (6e-3 + 2.0 ** -7 * np.abs(o_ref)) if tight == "mfma" else (1e-3 + 2.0 ** -8 * np.abs(o_ref))
        assert (err <= tol).all(), f"{what}: max abs err {err.max()} exceeds the rounding budget"
    return float(err.max())


class PrefillRun:
    """Device buffers for one prefill chunk of one sequence and the C-ABI calls on it."""

    def __init__(self, w: "wl.PrefillWorkload", interleaved: bool = False):
        self.w = w
        L = w.layer
        self.desc = layer_desc_of(L)
        self.seq_start, self.ctx_len, self.q_start = i64([0]), i32([w.N]), i32([w.chunk_start])
        self.out = torch.zeros((w.T, L.n_q_heads, 128), dtype=torch.bfloat16, device=DEV)
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


def prefill_oracle_inputs(w: "wl.PrefillWorkload") -> dict:
    L = w.layer
    d = dict(q_bits=wl.bf16_bits(w.q), K_bits=wl.bf16_bits(w.K), V_bits=wl.bf16_bits(w.V),
             kI_bits=wl.bf16_bits(w.kI), chunk_start=w.chunk_start, n_q_heads=L.n_q_heads,
             n_kv_heads=L.n_kv_heads, ret_heads=L.ret_heads, sink=L.sink, window=L.window)
    if w.WQ is not None:
        d.update(WQ=w.WQ.cpu().numpy(), q_pre_bits=wl.bf16_bits(w.q_pre))
    else:
        d.update(qI_bits=wl.bf16_bits(w.qI))
    return d
