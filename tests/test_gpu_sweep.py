"""Seeded, bounded sweeps of the decode step and of a prefill chunk over random layer shapes, head roles,
context lengths, windows and p, every case compared with the CPU oracle stage by stage (index query bits,
index scores, selection, attention), plus the two configurations an earlier sweep tripped over as named cases.

The workloads of the sweeps are drawn on the CPU (a seed replays bit for bit on any machine, under the oracle
alone as well) and moved to the GPU.  A sweep prints every case before it runs and stops at its first failure.
"""
import json

import numpy as np
import pytest
import torch

from oracle import rtp_oracle as orc
from paper_2605_16928_amd import workloads as wl
from gpu_util import (DEV, DecodeRun, PrefillRun, oracle_inputs, prefill_oracle_inputs, check_scores, check_selection,
                      check_selection_valid, check_out, check_layer)
import test_gpu_prefill as tp

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------------------------------------------
# decode
# ---------------------------------------------------------------------------------------------------
def check_decode_case(w: wl.DecodeWorkload, name: str, fuse_two: bool = True):
    """Every form of the decode step (five calls, selection + attention in one call, everything after the score
    pass in one call) on one workload: index query bits and scores against the oracle, the selection against
    the oracle's on the same scores and end to end, the forms against each other bit for bit, the layer output
    against the oracle.  Returns the number of retrieval rows whose set differs from the oracle's inside the
    threshold band (ties, fp32 scores)."""
    L = w.layer
    oi = oracle_inputs(w)
    ref = orc.decode_layer(**oi)
    two = DecodeRun(w, fuse_level1=fuse_two)
    two.index_score()
    torch.cuda.synchronize()
    if L.n_ret:
        assert np.array_equal(wl.bf16_bits(two.qI_out), ref["qI_bits"]), f"{name}: index query bits differ"
    s_gpu = two.scores.cpu().numpy()
    for r in range(two.R):
        b, j = divmod(r, L.n_ret)
        t0, n = w.seq_start[b], w.ctx_len[b]
        check_scores(s_gpu[r, :n] / (L.index_scale or 1.0), ref["scores"][r] / (L.index_scale or 1.0),
                     ref["qI_bits"][b, j], oi["kI_bits"][j, t0:t0 + n], f"{name} row {r}")
    two.topp()
    two.sparse_attn()
    two.local_attn()
    sets2, cnt2 = two.sel_sets()
    for r in range(two.R):
        n = w.ctx_len[r // L.n_ret]
        s64 = s_gpu[r, :n].astype(np.float64)
        pr = float(w.p_rows[r])
        check_selection(sets2[r], s64, orc.topp_select(s64, pr), pr, f"{name} row {r} (same scores)")
        slack = float(np.abs(s64 - ref["scores"][r]).max())
        check_selection_valid(sets2[r], ref["scores"][r], pr, slack, f"{name} row {r} (end to end)")
    other = check_layer(two.out_f64(), two.lse.cpu().numpy(), w, oi, ref, sets2, f"{name} five calls")
    run = DecodeRun(w)
    for form in ("one_call", "fused", "one_call"):
        run.sel_idx.fill_(-1)
        run.out.fill_(9.0)
        run.lse.fill_(9.0)
        if form == "one_call":
            run.step_one_stream()
        else:
            run.step()
        sets, cnt = run.sel_sets()
        assert torch.equal(run.sel_count, two.sel_count), f"{name} {form}: counts differ between forms"
        for r in range(run.R):
            assert torch.equal(run.sel_idx[r, :max(cnt[r], 0)], two.sel_idx[r, :max(cnt[r], 0)]), \
                f"{name} {form}: sets differ between forms"
        assert torch.equal(run.tau, two.tau) and torch.equal(run.mass, two.mass)
        check_layer(run.out_f64(), run.lse.cpu().numpy(), w, oi, ref, sets, f"{name} {form}")
    return other


def test_decode_tie_at_the_threshold_with_eight_heads_on_one_kv_head():
    """The configuration an earlier sweep reported as a 0.228 output error: 8 query heads on 1 KV head, the
    retrieval head in the middle of the group, contexts [13, 2213] with 16 sinks (more than the first context),
    p = [0.99, 0.5].  Two planted tokens of the second row carry identical bf16 index keys, their common score is
    the threshold: the oracle keeps the lower index (7 tokens), the library both (8 tokens) -- a legal set
    inside the band, so the retrieval row is held to the oracle's attention over the reported set.  The
    workload is drawn by the device generator, as it was then."""
    print("[case] decode, tie at the threshold, G = 8 on one KV head", flush=True)
    w = wl.small_decode(DEV, seed=141038683, ctx=(13, 2213), n_q_heads=8, n_kv_heads=1, ret_heads=(3,), sink=16,
                        window=4096, p=(0.99, 0.5, 0.8, 0.95), index_mode="direct", n_planted=8)
    check_decode_case(w, "tie_g8")


def test_decode_forced_tie_replayable():
    """The same situation built by hand on a CPU-drawn workload: the eight planted tokens of a row (60 % of its
    mass) get identical index keys, and p = 0.5 is reached inside that tie."""
    print("[case] decode, forced tie", flush=True)
    w = wl.small_decode("cpu", seed=77, ctx=(13, 3000), n_q_heads=8, n_kv_heads=1, ret_heads=(3,), sink=16, window=4096,
                        p=(0.99, 0.5), index_mode="direct", n_planted=8)
    pos = w.planted[(1, 0)]
    t0 = w.seq_start[1]
    w.kI[0, t0 + pos] = w.kI[0, t0 + pos[0]].clone()
    w = w.to(DEV)
    other = check_decode_case(w, "forced_tie")
    assert other >= 1, "the tie was meant to make the library's set larger than the oracle's"


def _decode_desc(rng):
    while True:
        nkv = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 2, 4, 8]))
        nq = nkv * G
        if nq <= 32:
            break
    n_ret = int(rng.integers(1, max(2, min(nq, 4) + 1)))
    ret = tuple(sorted(rng.choice(nq, size=min(n_ret, nq), replace=False).tolist()))
    B = int(rng.integers(1, 5))
    ctx = tuple(int(x) for x in np.exp(rng.uniform(np.log(5), np.log(30000), size=B)).astype(int))
    return dict(nq=nq, nkv=nkv, ret=ret, ctx=ctx, sink=int(rng.choice([0, 1, 4, 16])),
                window=int(rng.choice([1, 7, 64, 500, 4096])),
                p=tuple(float(x) for x in rng.choice([0.5, 0.8, 0.9, 0.95, 0.99, 1.0], size=4)),
                mode=str(rng.choice(["direct", "proj"])), seed=int(rng.integers(1 << 30)),
                n_planted=int(rng.choice([0, 1, 8])), fuse=bool(rng.integers(2)),
                index_scale=float(rng.choice([0.0, 0.0, 0.5, 3.0])), kv_dtype=str(rng.choice(["bf16", "bf16", "fp16"])))


def test_decode_sweep():
    rng = np.random.default_rng(20260531)
    n_other = 0
    for case in range(100):
        d = _decode_desc(rng)
        print("[case] decode sweep", case, json.dumps(d), flush=True)
        w = wl.small_decode("cpu", seed=d["seed"], ctx=d["ctx"], n_q_heads=d["nq"], n_kv_heads=d["nkv"],
                            ret_heads=d["ret"], sink=d["sink"], window=d["window"], p=d["p"], index_mode=d["mode"],
                            n_planted=d["n_planted"], kv_dtype=d["kv_dtype"])
        w.layer.index_scale = d["index_scale"]
        n_other += check_decode_case(w.to(DEV), f"sweep{case}", fuse_two=d["fuse"])
    print(f"   decode sweep: {n_other} retrieval rows differed from the oracle's set inside the band", flush=True)


# ---------------------------------------------------------------------------------------------------
# prefill
# ---------------------------------------------------------------------------------------------------
def check_prefill_case(w: wl.PrefillWorkload, name: str, p: float):
    """Retrieval heads with per-query top-p against the oracle (thresholds, counts, masses, attention over the
    kept sets, exact sets where no score is near the threshold), then the local heads and the paper's dense
    retrieval rule (p = 1) on every row."""
    tp._check_sparse_prefill(w, name, p)
    L = w.layer
    run = PrefillRun(w)
    oi = prefill_oracle_inputs(w)
    rows = [(t, h) for t in range(w.T) for h in range(L.n_q_heads)]
    run.out.fill_(9.0)
    run.local_attn()
    run.sparse_prefill(p=1.0)
    torch.cuda.synchronize()
    out = run.out.float().cpu().numpy().astype(np.float64)
    ref = orc.prefill_rows(rows=rows, p=1.0, **oi)
    o_ref = np.zeros_like(out)
    for r in ref:
        o_ref[r["t"], r["h"]] = r["out"]
    check_out(out, o_ref, f"{name} local + p1", tight="mfma")


def test_prefill_threshold_beside_a_score():
    """The configuration an earlier sweep reported as a 0.0214 same-set error: query 228 of head 2 has a token
    2.4e-7 above the REPORTED threshold that the kernel's keep test (an fp32 rounding of the same bound) leaves
    out; the output is the exact top-p set's.  Any set between {s > tau + band} and {s >= tau - band} with the
    reported count is a legal reading of the report.  Drawn by the device generator, as it was then."""
    print("[case] prefill, a score beside the reported threshold", flush=True)
    for mode in ("proj", "direct"):
        w = wl.small_prefill(DEV, seed=263203685, chunk_start=3000, T=300, p=0.99, n_q_heads=16, n_kv_heads=4,
                             ret_heads=(2, 3), sink=4, window=8192, index_mode=mode)
        check_prefill_case(w, f"beside_{mode}", 0.99)


def _prefill_desc(rng):
    while True:
        nkv = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 2, 4, 8]))
        nq = nkv * G
        if nq <= 16:
            break
    n_ret = int(rng.integers(1, min(nq, 3) + 1))
    return dict(nq=nq, nkv=nkv, ret=tuple(sorted(rng.choice(nq, size=n_ret, replace=False).tolist())),
                T=int(rng.choice([1, 17, 64, 100, 129, 200, 300])), start=int(rng.choice([0, 5, 100, 700, 1500, 3000])),
                sink=int(rng.choice([0, 4, 40])), window=int(rng.choice([8, 100, 600, 8192])),
                p=float(rng.choice([0.5, 0.8, 0.9, 0.99])), seed=int(rng.integers(1 << 30)),
                mode=str(rng.choice(["direct", "proj"])), index_scale=float(rng.choice([0.0, 0.0, 0.5, 3.0])),
                kv_dtype=str(rng.choice(["bf16", "bf16", "fp16"])))


def _peaked_prefill_desc(rng):
    """Laws on which most key tiles hold no kept pair: a small own cluster with nearly all the mass, runs of
    queries sharing a cluster, contexts of up to 200 key tiles, chunk lengths around the 256-query tile."""
    d = _prefill_desc(rng)
    d.update(T=int(rng.choice([31, 100, 256, 257, 300, 520])), start=int(rng.choice([0, 700, 4000, 9000, 12500])),
             mode="direct", own_frac=float(rng.choice([0.97, 0.99, 0.995])), pick_run=int(rng.choice([1, 8, 32, 64])),
             p=float(rng.choice([0.5, 0.8, 0.9])), cluster_len=int(rng.choice([4, 8, 32])))
    return d


def test_prefill_sweep():
    rng = np.random.default_rng(20260601)
    for case in range(100):
        d = _prefill_desc(rng)
        print("[case] prefill sweep", case, json.dumps(d), flush=True)
        w = wl.small_prefill("cpu", seed=d["seed"], chunk_start=d["start"], T=d["T"], p=d["p"], n_q_heads=d["nq"],
                             n_kv_heads=d["nkv"], ret_heads=d["ret"], sink=d["sink"], window=d["window"],
                             index_mode=d["mode"], kv_dtype=d["kv_dtype"])
        w.layer.index_scale = d["index_scale"]
        check_prefill_case(w.to(DEV), f"sweep{case}", d["p"])


def test_prefill_sweep_peaked_laws():
    """The tile lists of the selecting attention launch under random shapes: every case against the oracle, and
    over the sweep most key tiles must have been left out."""
    rng = np.random.default_rng(20260602)
    visited = causal = 0
    for case in range(40):
        d = _peaked_prefill_desc(rng)
        print("[case] prefill sweep, peaked", case, json.dumps(d), flush=True)
        w = wl.small_prefill("cpu", seed=d["seed"], chunk_start=d["start"], T=d["T"], p=d["p"], n_q_heads=d["nq"],
                             n_kv_heads=d["nkv"], ret_heads=d["ret"], sink=d["sink"], window=d["window"],
                             index_mode="direct", kv_dtype=d["kv_dtype"], own_frac=d["own_frac"], pick_run=d["pick_run"],
                             cluster_len=d["cluster_len"])
        w.layer.index_scale = d["index_scale"]
        w = w.to(DEV)
        tp._check_sparse_prefill(w, f"peaked{case}", d["p"])
        run = PrefillRun(w)
        run.sparse_prefill()
        v, c = run.tile_stats()
        assert 0 < v <= c
        visited += v
        causal += c
    print(f"   peaked sweep: {visited} of {causal} key tiles visited", flush=True)
    assert visited < 0.8 * causal
