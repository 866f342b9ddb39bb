"""GPU parity of the prefill path (MFMA tiles): local sink+window attention, the dense comparison,
and the retrieval heads' chunk kernel, against the CPU oracle row by row."""
import numpy as np
import pytest
import torch

from oracle import rtp_oracle as orc
from paper_2605_16928_amd import rtp, workloads as wl
from gpu_util import (DEV, PrefillRun, prefill_oracle_inputs, check_out, check_out_any, reported_sets, count_range, i32, i64,
                      layer_desc_of, ws_alloc)

pytestmark = pytest.mark.gpu


def _cases():
    return {
        # two query tiles with a ragged tail, band crossing several key tiles, sinks outside the band
        "small": dict(),
        # first chunk of a sequence: queries below the sink count, below one key tile
        "first_chunk": dict(chunk_start=0, T=130, seed=42),
        # window narrower than a key tile, no sinks
        "narrow": dict(chunk_start=300, T=100, sink=0, window=30, seed=43),
        # more sinks than one key tile holds
        "many_sinks": dict(chunk_start=900, T=64, sink=70, window=100, seed=44),
        # window wider than the context: local == dense
        "wide": dict(chunk_start=200, T=129, sink=4, window=4096, seed=45),
        # group sizes 1 and 8
        "g1": dict(n_q_heads=4, n_kv_heads=4, ret_heads=(2,), chunk_start=257, T=65, seed=46),
        "g8": dict(n_q_heads=16, n_kv_heads=2, ret_heads=(0, 8), chunk_start=1000, T=96, seed=47),
        # a single query
        "one_query": dict(chunk_start=333, T=1, seed=48),
        # fp16 attention tensors
        "small_f16": dict(seed=49, kv_dtype="fp16"),
        "g8_f16": dict(n_q_heads=16, n_kv_heads=2, ret_heads=(0, 8), chunk_start=1000, T=96, seed=50, kv_dtype="fp16"),
        "first_chunk_f16": dict(chunk_start=0, T=130, seed=51, kv_dtype="fp16"),
    }


@pytest.mark.parametrize("name", list(_cases()))
def test_prefill_local_dense_and_retrieval_p1(name):
    print(f"[case] prefill {name}", flush=True)
    w = wl.small_prefill(DEV, **_cases()[name])
    L = w.layer
    run = PrefillRun(w)
    oi = prefill_oracle_inputs(w)
    rows = [(t, h) for t in range(w.T) for h in range(L.n_q_heads)]

    # local heads + retrieval heads with p = 1 (the paper's prefill rule) fill the whole output
    run.out.fill_(9.0)
    run.local_attn()
    run.sparse_prefill(p=1.0)
    torch.cuda.synchronize()
    out = run.out.float().cpu().numpy().astype(np.float64)
    lse = run.lse.cpu().numpy()
    ref = orc.prefill_rows(rows=rows, p=1.0, **oi)
    o_ref = np.zeros_like(out)
    l_ref = np.zeros_like(lse)
    for r in ref:
        o_ref[r["t"], r["h"]] = r["out"]
        l_ref[r["t"], r["h"]] = r["lse"]
    check_out(out, o_ref, f"{name} local + retrieval(p=1)", tight="mfma")
    assert np.allclose(lse, l_ref, atol=3e-3, rtol=0)

    # dense comparison over all heads
    dout = torch.zeros_like(run.out)
    dlse = torch.zeros_like(run.lse)
    run.dense_attn(dout, dlse)
    torch.cuda.synchronize()
    dref = orc.dense_rows(rows=rows, q_bits=oi["q_bits"], K_bits=oi["K_bits"], V_bits=oi["V_bits"],
                          chunk_start=w.chunk_start, n_q_heads=L.n_q_heads, n_kv_heads=L.n_kv_heads, kv_dtype=L.kv_dtype)
    o_ref = np.zeros_like(out)
    for r in dref:
        o_ref[r["t"], r["h"]] = r["out"]
    check_out(dout.float().cpu().numpy().astype(np.float64), o_ref, f"{name} dense", tight="mfma")


def test_prefill_two_sequences_and_interleaved_kv():
    """B = 2 packed sequences with different chunk positions; K|V interleaved rows."""
    print("[case] prefill two sequences / interleaved", flush=True)
    d = wl.small_decode(DEV, seed=51, ctx=(900, 1300), sink=4, window=200, n_planted=0)
    L = d.layer
    n_q = 70
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    q = torch.randn((2, n_q, L.n_q_heads, 128), generator=g, device=DEV).to(torch.bfloat16)
    q_start = [900 - n_q, 1300 - n_q - 37]
    desc = layer_desc_of(L)
    out = torch.zeros((2, n_q, L.n_q_heads, 128), dtype=torch.bfloat16, device=DEV)
    dout = torch.zeros_like(out)
    ws = ws_alloc(rtp.rtp_local_attn_workspace_bytes(desc, 2, n_q, 1300))
    kv = torch.cat([d.K, d.V], dim=2).contiguous()
    T = d.T_tot
    rtp.rtp_local_attn(desc, q, kv.data_ptr(), kv.data_ptr() + 256, 256, T * 256, i64(d.seq_start), i32(d.ctx_len),
                       i32(q_start), 2, n_q, 1300, out, None, ws)
    rtp.rtp_dense_attn(desc, q, d.K, d.V, 128, T * 128, i64(d.seq_start), i32(d.ctx_len), i32(q_start), 2, n_q, 1300,
                       dout, None, ws)
    torch.cuda.synchronize()
    Kb, Vb, qb = wl.bf16_bits(d.K), wl.bf16_bits(d.V), wl.bf16_bits(q)
    local_heads = [h for h in range(L.n_q_heads) if h not in L.ret_heads]
    for b in range(2):
        s0, n = d.seq_start[b], d.ctx_len[b]
        common = dict(q_bits=qb[b], K_bits=Kb[:, s0:s0 + n], V_bits=Vb[:, s0:s0 + n], chunk_start=q_start[b],
                      n_q_heads=L.n_q_heads, n_kv_heads=L.n_kv_heads)
        rows = [(t, h) for t in range(n_q) for h in local_heads]
        ref = orc.prefill_rows(rows=rows, kI_bits=None, ret_heads=L.ret_heads, sink=L.sink, window=L.window, p=1.0,
                               **common)
        got = out[b].float().cpu().numpy().astype(np.float64)
        for r in ref:
            check_out(got[r["t"], r["h"]], r["out"], f"local b{b} t{r['t']} h{r['h']}", tight="mfma")
        for h in L.ret_heads:
            assert np.all(got[:, h] == 0)                       # retrieval rows untouched by the local call
        rows = [(t, h) for t in range(n_q) for h in range(L.n_q_heads)]
        dref = orc.dense_rows(rows=rows, **common)
        dgot = dout[b].float().cpu().numpy().astype(np.float64)
        for r in dref:
            check_out(dgot[r["t"], r["h"]], r["out"], f"dense b{b} t{r['t']} h{r['h']}", tight="mfma")


def _dense_vs_oracle(w, what):
    L = w.layer
    run = PrefillRun(w)
    oi = prefill_oracle_inputs(w)
    rows = [(t, h) for t in range(w.T) for h in range(L.n_q_heads)]
    dout = torch.zeros_like(run.out)
    dlse = torch.zeros_like(run.lse)
    run.dense_attn(dout, dlse)
    torch.cuda.synchronize()
    dref = orc.dense_rows(rows=rows, q_bits=oi["q_bits"], K_bits=oi["K_bits"], V_bits=oi["V_bits"],
                          chunk_start=w.chunk_start, n_q_heads=L.n_q_heads, n_kv_heads=L.n_kv_heads)
    got = dout.float().cpu().numpy().astype(np.float64)
    o_ref = np.zeros_like(got)
    for r in dref:
        o_ref[r["t"], r["h"]] = r["out"]
    assert np.isfinite(got).all(), what
    check_out(got, o_ref, what, tight="mfma")


def test_dense_prefill_scores_far_above_the_first_tile():
    """The dense kernel takes every query's reference maximum from the first key tile.  Here the late
    keys score ~90 (natural units) above it: exp overflows against that reference and the workgroup
    has to notice and repeat its keys with the running-maximum recurrence."""
    print("[case] dense prefill, reference outrun upwards", flush=True)
    w = wl.small_prefill(DEV, seed=91, chunk_start=600, T=150)
    w.q[:] = 2.0
    w.K[:, 300:, :] = 4.0                     # q.k * scale = 128 * 8 / sqrt(128) ~ 90.5 for keys >= 300
    _dense_vs_oracle(w, "reference outrun upwards")


def test_dense_prefill_reference_above_every_visible_score():
    """First chunk: keys 32..63 score ~90 above the rest but the first 32 queries cannot see them, so
    their reference (taken over the whole first tile, masks ignored) is far above everything they
    attend to; their probabilities underflow and the repeat pass has to produce them."""
    print("[case] dense prefill, reference outrun downwards", flush=True)
    w = wl.small_prefill(DEV, seed=92, chunk_start=0, T=100)
    w.q[:] = 2.0
    w.K[:, :, :] = (torch.randn_like(w.K.float()) * 0.05).to(w.K.dtype)
    w.K[:, 32:64, :] = 4.0
    _dense_vs_oracle(w, "reference outrun downwards")


# ---------------------------------------------------------------------------------------------
# per-query top-p in prefill (p < 1)
# ---------------------------------------------------------------------------------------------
FINE = 2.0 ** -17           # threshold resolution of the prefill selector (score units)
BAND = 3e-5                 # fp32 rounding of (max - score) and of the MFMA index scores


def _sparse_cases():
    return {
        "small_p90": (dict(), 0.9),
        "small_p50": (dict(seed=61), 0.5),
        "small_p999": (dict(seed=62), 0.999),
        "first_chunk": (dict(chunk_start=0, T=150, seed=63), 0.9),
        "proj": (dict(index_mode="proj", chunk_start=500, T=70, seed=64), 0.8),
        "zipf_g8": (dict(n_q_heads=16, n_kv_heads=2, ret_heads=(0, 8), chunk_start=1800, T=96, seed=65, zipf=1.1), 0.9),
        "p_to_one": (dict(chunk_start=300, T=40, seed=66), 0.9999999),
        # fp16 attention tensors: the matrix-core variants on binary16 operands
        "small_f16": (dict(seed=68, kv_dtype="fp16"), 0.9),
        "g8_f16": (dict(n_q_heads=16, n_kv_heads=2, ret_heads=(0, 8), chunk_start=1800, T=96, seed=69, kv_dtype="fp16"), 0.8),
    }


@pytest.mark.parametrize("name", list(_sparse_cases()))
def test_sparse_prefill_matches_oracle(name):
    print(f"[case] sparse prefill {name}", flush=True)
    kw, p = _sparse_cases()[name]
    w = wl.small_prefill(DEV, p=p, **kw)
    _check_sparse_prefill(w, name, p)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp16"])
def test_sparse_prefill_peaked_law_skips_key_tiles(kv_dtype):
    """A peaked indexer law: the own cluster of 8 tokens holds nearly all the mass, runs of 32 queries share a
    cluster, so p = 0.9 keeps a handful of tokens per query and most 64-key tiles hold no kept pair of a whole
    query tile.  The attention launch leaves those tiles out; everything it reports still matches the oracle,
    and the tile statistics show the skipping."""
    print(f"[case] sparse prefill, peaked law, {kv_dtype}", flush=True)
    w = wl.small_prefill(DEV, p=0.9, chunk_start=9000, T=600, seed=70, own_frac=0.99, pick_run=32, kv_dtype=kv_dtype)
    cnt = _check_sparse_prefill(w, f"peaked_{kv_dtype}", 0.9)
    assert np.median(cnt) <= 16
    run = PrefillRun(w)
    run.sparse_prefill(p=0.9)
    visited, causal = run.tile_stats()
    n_ret = w.layer.n_ret
    assert causal == n_ret * sum((9000 + min(t0 + 256, 600) - 1) // 64 + 1 for t0 in range(0, 600, 256))
    print(f"   tiles visited {visited} of {causal}", flush=True)
    assert 0 < visited < causal // 2
    # p close to 1 reaches every tile: the list is the whole causal range again
    run.sparse_prefill(p=0.9999999)
    assert run.tile_stats()[0] > causal // 2


def test_sparse_prefill_key_ranges_without_a_kept_key():
    """Long context, few heads: the launch cuts every query tile's key range in two, and with a small p the
    few kept tokens of a query leave whole ranges empty -- a legitimate zero partial, not a failed reference."""
    print("[case] sparse prefill, empty key ranges", flush=True)
    w = wl.small_prefill(DEV, p=0.3, chunk_start=6000, T=64, seed=67)
    cnt = _check_sparse_prefill(w, "empty_ranges", 0.3)
    assert cnt.min() < 64                     # some query keeps less than one tile's worth of keys


def test_sparse_prefill_reference_outrun_repeats_exactly():
    """The selecting mode on inputs whose late keys score ~90 above the first tile: the fixed reference
    overflows and the workgroup repeats its keys with the running maximum, keep test included."""
    print("[case] sparse prefill, reference outrun upwards", flush=True)
    w = wl.small_prefill(DEV, p=0.9, chunk_start=600, T=150, seed=93)
    w.q[:] = 2.0
    w.K[:, 300:, :] = 4.0
    _check_sparse_prefill(w, "sparse_outrun", 0.9)


def _check_sparse_prefill(w, name, p):
    L = w.layer
    run = PrefillRun(w)
    oi = prefill_oracle_inputs(w)
    run.out.fill_(5.0)
    run.sparse_prefill()
    torch.cuda.synchronize()
    out = run.out.float().cpu().numpy().astype(np.float64)
    tau, cnt, mass = run.tau.cpu().numpy(), run.count.cpu().numpy(), run.mass.cpu().numpy()
    p32 = float(np.float32(p))
    rows = [(t, h) for t in range(w.T) for h in L.ret_heads]
    ref = orc.prefill_rows(rows=rows, p=p32, **oi)
    sc = 1.0 / np.sqrt(128.0)
    worst = 0.0
    for r in ref:
        t, h, m = r["t"], r["h"], r["m"]
        j = L.ret_heads.index(h)
        s = r["scores"]
        wgt = np.exp(s - s.max())
        Z = wgt.sum()
        tg = float(tau[j, t])
        # (a) the kept set reaches p, and the threshold is never above the exact one
        keep = s > tg
        amb = np.abs(s - tg) <= BAND
        assert tg <= r["sel"]["tau"] + BAND, f"{name} t{t} h{h}: threshold {tg} above the exact {r['sel']['tau']}"
        assert wgt[keep | amb].sum() / Z >= p32 - 1e-6, f"{name} t{t} h{h}: kept mass below p"
        # (b) ... and not lower than one fine bin
        if np.isfinite(tg):
            above = s > tg + FINE + BAND
            assert wgt[above].sum() / Z < p32 + 1e-6, \
                f"{name} t{t} h{h}: threshold {tg} is more than one fine bin below the exact one"
        # (c) statistics
        assert abs(int(cnt[j, t]) - int(keep.sum())) <= int(amb.sum()), f"{name} t{t} h{h}: count {cnt[j, t]} vs {keep.sum()}"
        assert abs(mass[j, t] - wgt[keep].sum() / Z) <= 1e-5 + wgt[amb].sum() / Z
        # (d) attention over the set the library kept.  The reported threshold and the kernel's keep test are
        # fp32 roundings of the same bound, so a token whose fp64 score lies within the band of the reported
        # threshold may be on either side: any set between {s > tau + band} and {s >= tau - band} is a legal
        # reading of the report.  The reported count says how many band tokens are in; the test is
        # monotone in the score, so they are the highest-scoring ones (band tokens whose scores differ by less
        # than fp32 resolves may swap: then any choice of that many is accepted).
        kvh = h // (L.n_q_heads // L.n_kv_heads)

        def att(ids):
            return orc.attend(oi["q_bits"][t, h], oi["K_bits"][kvh, :m + 1], oi["V_bits"][kvh, :m + 1], ids, sc, L.kv_dtype)[0]

        def att_abs(ids):
            return orc.attend(oi["q_bits"][t, h], oi["K_bits"][kvh, :m + 1], oi["V_bits"][kvh, :m + 1] & 0x7fff, ids, sc,
                              L.kv_dtype)[0]

        worst = max(worst, check_out_any(out[t, h], reported_sets(s, tg, int(cnt[j, t]), BAND, f"{name} t{t} h{h}"), att,
                                         f"{name} t{t} h{h} (same set)", att_abs))
        # (e) end to end against the exact top-p set: the stated tolerance.  Tokens within 1e-5 of the
        # exact threshold may legitimately differ; rows that have such a token are only held to (d).
        near = np.abs(s - r["sel"]["tau"]) <= 1e-5 * max(1.0, abs(r["sel"]["tau"]))
        if near.sum() <= 1:
            k_lo, k_hi = count_range(s, p32)
            assert k_lo <= int(cnt[j, t]) <= k_hi, f"{name} t{t} h{h}: set differs ({cnt[j, t]} kept, exact {r['sel']['count']})"
            if k_lo == k_hi:
                assert int(cnt[j, t]) == r["sel"]["count"]
                check_out(out[t, h], r["out"], f"{name} t{t} h{h} (exact top-p)", tight=False)
    for h in range(L.n_q_heads):
        if h not in L.ret_heads:
            assert np.all(out[:, h] == 5.0)
    print(f"   worst abs err vs same-set oracle {worst:.2e}; kept tokens min/mean/max "
          f"{cnt.min()}/{cnt.mean():.1f}/{cnt.max()}", flush=True)
    return cnt


def test_sparse_prefill_p1_statistics_and_dense_equivalence():
    """p = 1 with statistics requested runs the selecting kernel with nothing to select:
    the dense path's output up to rounding (the two kernels block the keys differently),
    count = m + 1, mass = 1."""
    print("[case] sparse prefill p=1 statistics", flush=True)
    w = wl.small_prefill(DEV, seed=71, chunk_start=260, T=90)
    run = PrefillRun(w)
    L = w.layer
    run.sparse_prefill(p=1.0)
    torch.cuda.synchronize()
    a = run.out.clone()
    cnt = run.count.cpu().numpy()
    assert np.array_equal(cnt, np.tile(w.chunk_start + np.arange(w.T) + 1, (L.n_ret, 1)))
    assert np.all(run.mass.cpu().numpy() == 1.0)
    dout = torch.zeros_like(run.out)
    run.dense_attn(dout)
    torch.cuda.synchronize()
    ga = a[:, L.ret_heads].float().cpu().numpy().astype(np.float64)
    gd = dout[:, L.ret_heads].float().cpu().numpy().astype(np.float64)
    assert (np.abs(ga - gd) <= 2e-3 + 2.0 ** -7 * np.abs(gd)).all(), np.abs(ga - gd).max()


def test_retrieval_dense_split_keys_matches_unsplit():
    """Few heads and a long context: the dense rule cuts every query tile's key range into parts and
    merges them.  With a workspace the split path runs, without one the unsplit path: same result."""
    print("[case] dense retrieval rule with key-range splits", flush=True)
    w = wl.small_prefill(DEV, seed=81, chunk_start=6000, T=130, n_q_heads=4, n_kv_heads=2, ret_heads=(1,))
    run = PrefillRun(w)
    L = w.layer
    need = rtp.rtp_sparse_attn_prefill_workspace_bytes(run.desc, w.T, w.chunk_start)
    assert need > L.n_ret * w.T * 132 * 4            # room for at least two partials per row
    a = torch.zeros_like(run.out)
    b = torch.zeros_like(run.out)
    la, lb = torch.zeros_like(run.lse), torch.zeros_like(run.lse)
    args = (run.desc, w.qI, w.q, None, w.kI, w.N * 16, run.Kp, run.Vp, run.rs, run.hs, w.chunk_start, w.T, 1.0)
    rtp.rtp_sparse_attn_prefill(*args, a, la, None, None, None, run.ws)
    rtp.rtp_sparse_attn_prefill(*args, b, lb, None, None, None, None)
    torch.cuda.synchronize()
    oi = prefill_oracle_inputs(w)
    rows = [(t, 1) for t in range(w.T)]
    ref = orc.dense_rows(rows=rows, q_bits=oi["q_bits"], K_bits=oi["K_bits"], V_bits=oi["V_bits"],
                         chunk_start=w.chunk_start, n_q_heads=L.n_q_heads, n_kv_heads=L.n_kv_heads)
    ga = a.float().cpu().numpy().astype(np.float64)
    gb = b.float().cpu().numpy().astype(np.float64)
    for r in ref:
        check_out(ga[r["t"], 1], r["out"], "split", tight="mfma")
        check_out(gb[r["t"], 1], r["out"], "unsplit", tight="mfma")
        assert abs(la[r["t"], 1].item() - r["lse"]) < 3e-3 and abs(lb[r["t"], 1].item() - r["lse"]) < 3e-3


@pytest.mark.parametrize("scale,p", [(2.0, 0.999999), (2.5, 0.9999999), (3.0, 0.999999)])
def test_sparse_prefill_threshold_far_below_the_row_maximum(scale, p):
    """Score rows whose bulk lies 13 to 22 below the row maximum, with p so close to 1 that the threshold falls
    into that bulk: the search's first digit covers 15.875 below its reference, so it must lower the reference
    and repeat for such queries instead of keeping every candidate (fp32 p cannot push a threshold much deeper
    than that at these lengths; every repeat runs the same code).  Checked like every
    other case: exact sets away from the threshold band, counts, masses, attention over the kept set."""
    print(f"[case] sparse prefill, threshold far below the maximum, scale {scale} p {p}", flush=True)
    w = wl.small_prefill("cpu", p=p, chunk_start=2500, T=96, seed=97)
    w.layer.index_scale = scale
    w = w.to(DEV)
    cnt = _check_sparse_prefill(w, f"far_{scale}", p)
    # the case does what it is meant to: for most queries the threshold lies more than 15.875 below the maximum,
    # and the kept set is neither tiny nor the whole candidate set
    run = PrefillRun(w)
    run.sparse_prefill()
    torch.cuda.synchronize()
    oi = prefill_oracle_inputs(w)
    ref = orc.prefill_rows(rows=[(t, w.layer.ret_heads[0]) for t in range(0, w.T, 8)], p=float(np.float32(p)), **oi)
    deep = [r["sel"]["smax"] - r["sel"]["tau"] for r in ref]
    assert max(deep) > 15.875 and (scale > 2.75 or np.median(deep) > 15.875), deep
    assert all(r["sel"]["count"] < r["m"] + 1 for r in ref)
