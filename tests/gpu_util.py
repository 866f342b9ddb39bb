"""Helpers shared by the GPU parity tests: run the path through the C-ABI on cuda:0 (the drivers
live in paper_2605_16928_amd.pipeline), hand the same inputs to the oracle, and compare with the
stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

from oracle import rtp_oracle as orc
from paper_2605_16928_amd import rtp, workloads as wl
from paper_2605_16928_amd.pipeline import DEV, DecodeRun, PrefillRun, layer_desc_of, ws_alloc, i32, i64  # noqa: F401

# tolerances (benchmark spec; forms fixed here)
SCORE_RTOL = 1e-5          # |d| <= 1e-5 * max(|s_ref|, sum_i |qI_i kI_i|)
BAND_RTOL = 1e-5           # tokens with |s - tau| <= 1e-5 * max(1, |tau|) may differ
OUT_ATOL, OUT_RTOL = 2e-2, 1e-2


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
