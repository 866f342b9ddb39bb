"""Parity at the full sizes of the baseline configurations, in the launch configuration the benchmark
times.  Decode rows are cheap for the oracle, so every retrieval row is checked; prefill checks a
sample of (query, head) rows that includes the chunk edges (rows are independent, so sampling is sound).
"""
import numpy as np
import pytest
import torch

from oracle import rtp_oracle as orc
from paper_2605_16928_amd import rtp, workloads as wl
from gpu_util import (DEV, DecodeRun, PrefillRun, check_scores, check_selection, check_selection_valid, check_out,
                      check_out_any, reported_sets, count_range)

pytestmark = pytest.mark.gpu
SC = 1.0 / np.sqrt(128.0)


def _decode_fullsize(w, n_local_samples=24, n_dense_samples=2, seed=0):
    L = w.layer
    G = L.n_q_heads // L.n_kv_heads
    run = DecodeRun(w)
    side = torch.cuda.Stream()
    run.step_fastest(side)
    torch.cuda.synchronize()
    s_gpu = run.scores.cpu().numpy()
    sets, cnt = run.sel_sets()
    out = run.out_f64()
    kI, qI = wl.bf16_bits(w.kI), wl.bf16_bits(w.qI)
    qb = wl.bf16_bits(w.q)
    rng = np.random.default_rng(seed)
    sizes = []

    def kv_slice(kvh, t0, ids):
        ids_t = torch.as_tensor(np.asarray(ids) + t0, device=DEV)
        return wl.bf16_bits(w.K[kvh].index_select(0, ids_t)), wl.bf16_bits(w.V[kvh].index_select(0, ids_t))

    for b in range(w.B):
        t0, n = w.seq_start[b], w.ctx_len[b]
        for j, h in enumerate(L.ret_heads):
            r = b * L.n_ret + j
            p = float(w.p_rows[r])
            s_ref = orc.index_score(qI[b, j], kI[j, t0:t0 + n])
            check_scores(s_gpu[r, :n], s_ref, qI[b, j], kI[j, t0:t0 + n], f"row {r}")
            s64 = s_gpu[r, :n].astype(np.float64)
            check_selection(sets[r], s64, orc.topp_select(s64, p), p, f"row {r} (same scores)")
            check_selection_valid(sets[r], s_ref, p, float(np.abs(s64 - s_ref).max()), f"row {r} (end to end)")
            Ks, Vs = kv_slice(h // G, t0, sets[r])
            o, _ = orc.attend(qb[b, h], Ks, Vs, np.arange(len(sets[r])), SC, L.kv_dtype)
            check_out(out[b, h], o, f"sparse b{b} h{h}")
            sizes.append(len(sets[r]))
    local_heads = [h for h in range(L.n_q_heads) if h not in L.ret_heads]
    for _ in range(n_local_samples):
        b = int(rng.integers(w.B))
        h = int(rng.choice(local_heads))
        ids = orc.local_set(w.ctx_len[b] - 1, L.sink, L.window)
        Ks, Vs = kv_slice(h // G, w.seq_start[b], ids)
        o, _ = orc.attend(qb[b, h], Ks, Vs, np.arange(len(ids)), SC, L.kv_dtype)
        check_out(out[b, h], o, f"local b{b} h{h}")
    dout = torch.zeros_like(run.out)
    run.dense_attn(dout)
    torch.cuda.synchronize()
    dgot = dout.float().cpu().numpy().astype(np.float64)
    for _ in range(n_dense_samples):
        b = int(rng.integers(w.B))
        h = int(rng.integers(L.n_q_heads))
        t0, n = w.seq_start[b], w.ctx_len[b]
        o, _ = orc.attend(qb[b, h], wl.bf16_bits(w.K[h // G, t0:t0 + n]), wl.bf16_bits(w.V[h // G, t0:t0 + n]),
                          np.arange(n), SC, L.kv_dtype)
        check_out(dgot[b, h], o, f"dense b{b} h{h}")

    # selection and attention as two calls: the same sets bit for bit, the same outputs up to summation order
    sel1, cnt1, tau1, out1 = run.sel_idx.clone(), run.sel_count.clone(), run.tau.clone(), run.out.clone()
    run.step_two_streams(side, fused=False)
    torch.cuda.synchronize()
    assert torch.equal(cnt1, run.sel_count) and torch.equal(tau1, run.tau)
    for r in range(run.R):
        assert torch.equal(sel1[r, :cnt[r]], run.sel_idx[r, :cnt[r]])
    assert (out1.float() - run.out.float()).abs().max().item() <= 2e-2
    return sizes


@pytest.mark.parametrize("p", [0.8, 0.9, 0.95])
def test_c2_full_size(p):
    print(f"[case] c2 full size p={p}", flush=True)
    sizes = _decode_fullsize(wl.c2(DEV, p=p))
    print(f"   selected tokens per row: min {min(sizes)} mean {np.mean(sizes):.0f} max {max(sizes)}", flush=True)
    assert len(sizes) == 32


def test_c2_full_size_with_clustered_kept_tokens():
    """Configuration 2 at full size with the scores of every row's last 8192 tokens raised by 2 (what bench.py
    reports as extra.clustered_law): most rows then have one overfull chunk and the one-call form shares the
    gather out by rank.  Selection against the oracle on the same scores, attention against the oracle over
    the selected rows, and both bit for bit / within tolerance of the two separate calls."""
    print("[case] c2 full size, clustered law", flush=True)
    w = wl.c2(DEV, seed=5)
    L = w.layer
    G = L.n_q_heads // L.n_kv_heads
    N = w.ctx_len[0]
    qb = wl.bf16_bits(w.q)

    def prepared():
        run = DecodeRun(w, fuse_level1=False)
        run.index_score()
        run.scores.view(-1, run.stride)[:, N - 8192:N] += 2.0
        return run

    two = prepared()
    two.topp()
    two.sparse_attn()
    two.local_attn()
    run = prepared()
    run.decode_attention()
    torch.cuda.synchronize()
    sets, cnt = run.sel_sets()
    assert torch.equal(run.sel_count, two.sel_count) and torch.equal(run.tau, two.tau)
    overfull = 0
    for r in range(run.R):
        assert torch.equal(run.sel_idx[r, :cnt[r]], two.sel_idx[r, :cnt[r]])
        per_chunk = np.bincount(np.asarray(sets[r]) // 8192, minlength=16)
        overfull += int(per_chunk.max() > 5 * (cnt[r] // 16) // 4 + 400)
    assert overfull >= run.R // 2, "the law no longer clusters the kept tokens"
    assert (run.out.float() - two.out.float()).abs().max().item() <= 2e-2
    s_gpu = run.scores.cpu().numpy()
    out = run.out_f64()
    for r in range(0, run.R, 5):                              # a sample of rows against the oracle
        b, j = divmod(r, L.n_ret)
        h = L.ret_heads[j]
        s64 = s_gpu[r, :N].astype(np.float64)
        pr = float(w.p_rows[r])
        check_selection(sets[r], s64, orc.topp_select(s64, pr), pr, f"clustered row {r}")
        ids_t = torch.as_tensor(np.asarray(sets[r]) + w.seq_start[b], device=DEV)
        Ks, Vs = wl.bf16_bits(w.K[h // G].index_select(0, ids_t)), wl.bf16_bits(w.V[h // G].index_select(0, ids_t))
        o, _ = orc.attend(qb[b, h], Ks, Vs, np.arange(len(sets[r])), SC)
        check_out(out[b, h], o, f"clustered sparse b{b} h{h}")


def test_c5_full_size():
    print("[case] c5 full size (ragged batch of 32, 64 query heads)", flush=True)
    w = wl.c5(DEV)
    sizes = _decode_fullsize(w, n_local_samples=16, n_dense_samples=1)
    print(f"   selected tokens per row: min {min(sizes)} mean {np.mean(sizes):.0f} max {max(sizes)}", flush=True)
    assert max(sizes) >= 100 * max(min(sizes), 1)          # the recipe spans two orders of magnitude


def test_c4_decode_full_size():
    print("[case] decode at 1,048,576 tokens", flush=True)
    sizes = _decode_fullsize(wl.c4_decode(DEV), n_local_samples=8, n_dense_samples=1)
    print(f"   selected tokens per row: {sizes}", flush=True)


def _prefill_fullsize(w, rows_local, rows_ret, rows_dense, what):
    L = w.layer
    G = L.n_q_heads // L.n_kv_heads
    run = PrefillRun(w)
    run.local_attn()
    run.sparse_prefill()
    torch.cuda.synchronize()
    out = run.out.float().cpu().numpy().astype(np.float64)
    tau, cnt = run.tau.cpu().numpy(), run.count.cpu().numpy()
    qb, kI, qI = wl.bf16_bits(w.q), wl.bf16_bits(w.kI), wl.bf16_bits(w.qI)
    p32 = float(np.float32(w.p))

    def kv_rows(kvh, ids):
        ids_t = torch.as_tensor(np.asarray(ids), device=DEV)
        return wl.bf16_bits(w.K[kvh].index_select(0, ids_t)), wl.bf16_bits(w.V[kvh].index_select(0, ids_t))

    for (t, h) in rows_local:
        m = w.chunk_start + t
        ids = orc.local_set(m, L.sink, L.window)
        Ks, Vs = kv_rows(h // G, ids)
        o, _ = orc.attend(qb[t, h], Ks, Vs, np.arange(len(ids)), SC)
        check_out(out[t, h], o, f"{what} local t{t} h{h}", tight="mfma")
    kept = []
    for (t, h) in rows_ret:
        m = w.chunk_start + t
        j = L.ret_heads.index(h)
        s = orc.index_score(qI[j, t], kI[j, :m + 1])
        ref = orc.topp_select(s, p32)
        tg = float(tau[j, t])
        keep = s > tg
        amb = np.abs(s - tg) <= 3e-5
        wgt = np.exp(s - s.max())
        Z = wgt.sum()
        assert tg <= ref["tau"] + 3e-5 and wgt[keep | amb].sum() / Z >= p32 - 1e-6
        assert wgt[s > tg + 2.0 ** -17 + 3e-5].sum() / Z < p32 + 1e-6
        assert abs(int(cnt[j, t]) - int(keep.sum())) <= int(amb.sum())
        def att(ids):
            Ks, Vs = kv_rows(h // G, ids)
            return orc.attend(qb[t, h], Ks, Vs, np.arange(len(ids)), SC)[0]

        def att_abs(ids):
            Ks, Vs = kv_rows(h // G, ids)
            return orc.attend(qb[t, h], Ks, Vs & 0x7fff, np.arange(len(ids)), SC)[0]

        check_out_any(out[t, h], reported_sets(s, tg, int(cnt[j, t]), 3e-5, f"{what} t{t} h{h}"), att,
                      f"{what} sparse t{t} h{h}", att_abs)
        near = np.abs(s - ref["tau"]) <= 1e-5 * max(1.0, abs(ref["tau"]))
        if near.sum() <= 1:
            k_lo, k_hi = count_range(s, p32)
            assert k_lo <= int(cnt[j, t]) <= k_hi, f"{what} t{t} h{h}: set differs from exact top-p"
        kept.append(int(keep.sum()))
    if rows_dense:
        dout = torch.zeros_like(run.out)
        run.dense_attn(dout)
        torch.cuda.synchronize()
        dgot = dout.float().cpu().numpy().astype(np.float64)
        for (t, h) in rows_dense:
            m = w.chunk_start + t
            o, _ = orc.attend(qb[t, h], wl.bf16_bits(w.K[h // G, :m + 1]), wl.bf16_bits(w.V[h // G, :m + 1]),
                              np.arange(m + 1), SC)
            check_out(dgot[t, h], o, f"{what} dense t{t} h{h}", tight="mfma")
    return kept


def _sample_rows(w, n, heads, rng, edges=True):
    ts = set(rng.integers(0, w.T, size=n).tolist())
    if edges:
        ts |= {0, 1, 63, 64, 127, 128, w.T - 1, w.T - 2, w.T // 2}
    ts = sorted(t for t in ts if 0 <= t < w.T)
    return [(t, int(heads[i % len(heads)])) for i, t in enumerate(ts)]


def test_c3_chunks_sampled_rows():
    """Configuration 3: first chunk (queries below one key tile, below the sink count) and last chunk."""
    rng = np.random.default_rng(7)
    for chunk in (0, 31):
        print(f"[case] c3 chunk {chunk}", flush=True)
        w = wl.c3_chunk(DEV, chunk=chunk)
        L = w.layer
        local_heads = [h for h in range(L.n_q_heads) if h not in L.ret_heads]
        kept = _prefill_fullsize(w, _sample_rows(w, 96, local_heads, rng), _sample_rows(w, 120, L.ret_heads, rng),
                                 _sample_rows(w, 6, list(range(L.n_q_heads)), rng, edges=False), f"c3 chunk {chunk}")
        print(f"   kept tokens over {len(kept)} sampled retrieval rows: min {min(kept)} mean {np.mean(kept):.0f} "
              f"max {max(kept)}", flush=True)


def test_c4_last_chunk_sampled_rows():
    """Configuration 4: the 8192-query chunk that sees the whole 1,048,576-token context."""
    print("[case] c4 last chunk", flush=True)
    rng = np.random.default_rng(8)
    w = wl.c4_chunk(DEV, chunk=127)
    L = w.layer
    local_heads = [h for h in range(L.n_q_heads) if h not in L.ret_heads]
    rows_local, rows_ret = _sample_rows(w, 125, local_heads, rng), _sample_rows(w, 125, L.ret_heads, rng)
    assert len(rows_local) + len(rows_ret) >= 256            # chunk edges and the last row of the sequence included
    kept = _prefill_fullsize(w, rows_local, rows_ret, _sample_rows(w, 3, list(range(L.n_q_heads)), rng, edges=False),
                             "c4 last chunk")
    print(f"   kept tokens over {len(kept)} sampled retrieval rows: min {min(kept)} mean {np.mean(kept):.0f} "
          f"max {max(kept)}", flush=True)


@pytest.mark.parametrize("law", ["peaked", "peaked_hard"])
def test_c4_last_chunk_peaked_laws_sampled_rows(law):
    """Configuration 4 under the peaked indexer laws (about 20 kept tokens per query; "peaked_hard" adds a few
    queries that keep up to hundreds of thousands): the launch that leaves out the key tiles without a kept pair,
    sampled retrieval rows -- the rows with the most kept tokens among them -- against the oracle."""
    print(f"[case] c4 last chunk, {law} law", flush=True)
    rng = np.random.default_rng(9)
    w = wl.c4_chunk(DEV, chunk=127, law=law)
    L = w.layer
    run = PrefillRun(w)
    run.sparse_prefill()
    cnt = run.count.cpu().numpy()
    visited, causal = run.tile_stats()
    print(f"   64-key tiles visited: {visited} of {causal}", flush=True)
    assert visited < causal // 2
    rows = _sample_rows(w, 60, L.ret_heads, rng)
    order = np.argsort(cnt, axis=None)[::-1][:6]              # the deepest rows of the chunk
    rows += [(int(i % w.T), int(L.ret_heads[i // w.T])) for i in order]
    del run
    kept = _prefill_fullsize(w, [], rows, [], f"c4 {law}")
    print(f"   kept tokens over {len(kept)} sampled retrieval rows: min {min(kept)} median {np.median(kept):.0f} "
          f"max {max(kept)}", flush=True)
    assert np.median(kept) < 200


def test_c2_full_size_fp16():
    """Configuration 2 with fp16 attention tensors (the format the paper's decode kernel loads): the timed
    step, every row against the oracle."""
    print("[case] c2 full size, fp16 K/V", flush=True)
    w = wl.c2(DEV, p=0.9, kv_dtype="fp16")
    sizes = _decode_fullsize(w, 9)
    assert min(sizes) > 1000
