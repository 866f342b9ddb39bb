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
             window=L.window, p_rows=w.p_rows.cpu().numpy().astype(np.float64),
             softmax_scale=L.softmax_scale, index_scale=L.index_scale, kv_dtype=L.kv_dtype)
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


def attend_reference(w: wl.DecodeWorkload, oi: dict, sets) -> dict:
    """The oracle's attention of every retrieval row over the given sets: {(b, h): (out, lse)}."""
    L = w.layer
    sc = L.softmax_scale if L.softmax_scale else 1.0 / np.sqrt(128.0)
    ref = {}
    for b in range(w.B):
        t0, n = w.seq_start[b], w.ctx_len[b]
        for j, h in enumerate(L.ret_heads):
            kvh = h // (L.n_q_heads // L.n_kv_heads)
            if len(sets[b * L.n_ret + j]) == 0:
                continue
            ref[(b, h)] = orc.attend(oi["q_bits"][b, h], oi["K_bits"][kvh, t0:t0 + n], oi["V_bits"][kvh, t0:t0 + n],
                                     sets[b * L.n_ret + j], sc, L.kv_dtype)
    return ref


def check_layer(out: np.ndarray, lse: np.ndarray, w: wl.DecodeWorkload, oi: dict, ref: dict, sets, what=""):
    """One decode step's output, every (sequence, head) row, against the oracle.  Local rows and retrieval
    rows whose set IS the oracle's: the oracle's layer.  A retrieval row whose set differs from the oracle's
    can only differ inside the threshold band (the selection checks establish that; the library keeps every
    token tied with the threshold score where the oracle keeps the lower indices), so its output is held to
    the oracle's attention over the set the library reports.  Returns the number of such rows."""
    L = w.layer
    other = 0
    att = None
    for b in range(w.B):
        for h in range(L.n_q_heads):
            o, l = ref["out"][b, h], ref["lse"][b, h]
            if h in L.ret_heads:
                r = b * L.n_ret + list(L.ret_heads).index(h)
                if not np.array_equal(np.sort(ref["sel"][r]["idx"]), np.asarray(sets[r])):
                    att = attend_reference(w, oi, sets) if att is None else att
                    o, l = att[(b, h)]
                    other += 1
            check_out(out[b, h], o, f"{what} b{b} h{h}")
            assert abs(lse[b, h] - l) < 2e-3, f"{what} b{b} h{h}: lse {lse[b, h]} vs {l}"
    return other


def reported_sets(s: np.ndarray, tau_rep: float, count_rep: int, band: float, what=""):
    """The sets a prefill report (threshold, count) of the library can stand for, given the oracle's fp64 scores
    `s`.  The reported threshold and the kernel's keep test are fp32 roundings of the same bound, so a token whose
    score lies within `band` of the reported threshold may be on either side: any set between {s > tau + band}
    and {s >= tau - band} is a legal reading.  The reported count says how many band tokens are in; the keep test
    is monotone in the score, so the first candidate is the highest-scoring ones; band tokens closer to each other
    than fp32 resolves may swap, so every other choice of that many follows (for small bands only)."""
    import itertools
    certain = np.nonzero(s > tau_rep + band)[0]
    band_ids = np.nonzero(np.abs(s - tau_rep) <= band)[0]
    band_ids = band_ids[np.argsort(-s[band_ids], kind="stable")]
    k_in = int(count_rep) - len(certain)
    assert 0 <= k_in <= len(band_ids), f"{what}: count {count_rep} outside [{len(certain)}, {len(certain) + len(band_ids)}]"
    yield np.sort(np.concatenate([certain, band_ids[:k_in]]))
    if 0 < k_in < len(band_ids) and len(band_ids) <= 12:
        for extra in itertools.combinations(band_ids.tolist(), k_in):
            if list(extra) != band_ids[:k_in].tolist():
                yield np.sort(np.concatenate([certain, np.asarray(extra, dtype=np.int64)]))


MASS_EPS = 3e-7      # the library's weights are fp32 exponentials (relative error up to 2^-22 each), summed in fp64


def count_range(s: np.ndarray, p: float):
    """Sizes of the top-p set of scores `s` that fp32 weights can justify: from the smallest set whose fp64 mass
    reaches p - MASS_EPS to the smallest whose mass reaches p + MASS_EPS.  For ordinary p and set sizes the two
    coincide with the exact count; they part when single tokens weigh less than the rounding of the heaviest ones
    (p within 1e-5 of 1 on peaked rows)."""
    w = np.exp(s - s.max())
    cum = np.cumsum(np.sort(w)[::-1]) / w.sum()
    lo = int(np.searchsorted(cum, p - MASS_EPS, side="left")) + 1
    hi = int(np.searchsorted(cum, min(p + MASS_EPS, cum[-1]), side="left")) + 1
    return min(lo, len(s)), min(hi, len(s))


def check_out_any(o_gpu: np.ndarray, candidates, attend_fn, what="", attend_abs_fn=None):
    """o_gpu must match attend_fn(ids) for one of the candidate sets (the first is the expected one): to the
    stated bar, and to the rounding budget of the prefill kernels, which round every probability to bf16 before the
    PV product and the output once more: |err| <= 1e-3 + 2^-8 * sum_i p_i |v_i| + 2^-8 * |ref| per coordinate
    (attend_abs_fn(ids) returns sum_i p_i |v_i|, i.e. the same attention over |V|)."""
    first = None
    for ids in candidates:
        try:
            ref = attend_fn(ids)
            err = check_out(o_gpu, ref, what, tight=False)
            if attend_abs_fn is not None:
                budget = 1e-3 + 2.0 ** -8 * attend_abs_fn(ids) + 2.0 ** -8 * np.abs(ref)
                assert (np.abs(o_gpu - ref) <= budget).all(), \
                    f"{what}: max abs err {err} exceeds the rounding budget of bf16 probabilities"
            return err
        except AssertionError as e:
            first = first or e
    raise first


def prefill_oracle_inputs(w: "wl.PrefillWorkload") -> dict:
    L = w.layer
    d = dict(q_bits=wl.bf16_bits(w.q), K_bits=wl.bf16_bits(w.K), V_bits=wl.bf16_bits(w.V),
             kI_bits=wl.bf16_bits(w.kI), chunk_start=w.chunk_start, n_q_heads=L.n_q_heads,
             n_kv_heads=L.n_kv_heads, ret_heads=L.ret_heads, sink=L.sink, window=L.window,
             softmax_scale=L.softmax_scale, index_scale=L.index_scale, kv_dtype=L.kv_dtype)
    if w.WQ is not None:
        d.update(WQ=w.WQ.cpu().numpy(), q_pre_bits=wl.bf16_bits(w.q_pre))
    else:
        d.update(qI_bits=wl.bf16_bits(w.qI))
    return d
