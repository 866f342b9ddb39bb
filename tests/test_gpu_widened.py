"""GPU parity tests of the entry points beside the five core ones: index-key build, static top-k,
block-wise histogram top-p and the sparsity figures -- each through the C-ABI against the CPU oracle
on the same seeded inputs.  Integer and index results are compared bit for bit."""
import numpy as np
import pytest
import torch

from oracle import rtp_oracle as orc
from paper_2605_16928_amd import rtp, workloads as wl
from gpu_util import DEV, DecodeRun, oracle_inputs, i32, i64, ws_alloc, layer_desc_of

pytestmark = pytest.mark.gpu


def _bits(t):
    return wl.bf16_bits(t)


# ---------------------------------------------------------------------------------------------------
# index-key build (Sec. 3.2, indexer equation)
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("T,Hq,Hkv,ret", [(1, 8, 2, [0, 4]), (197, 8, 2, [1, 2, 6]), (4096 + 33, 32, 8, [0, 8, 16, 24]),
                                          (70, 64, 8, list(range(0, 64, 8)))])
def test_index_project_key_and_query_side_bit_exact(T, Hq, Hkv, ret):
    print(f"[case] index_project T={T} Hq={Hq} Hkv={Hkv}", flush=True)
    g = torch.Generator(device="cpu").manual_seed(1000 + T)
    n_ret = len(ret)
    W = (torch.randn((n_ret, 16, 128), generator=g) / 128 ** 0.5).float()
    k_pre = torch.randn((T, Hkv, 128), generator=g).to(torch.bfloat16)
    q_pre = torch.randn((T, Hq, 128), generator=g).to(torch.bfloat16)
    desc = rtp.layer_desc(Hq, Hkv, ret, 4, 64)
    t0, cap = 5, T + 9                                    # append at token offset 5 of a larger cache
    kI = torch.full((n_ret, cap, 16), 7.0, dtype=torch.bfloat16, device=DEV)
    rtp.rtp_index_project(desc, W.to(DEV), k_pre.to(DEV), rtp.RTP_SIDE_KEY, T, kI, cap * 16, t0)
    qI = torch.zeros((n_ret, T, 16), dtype=torch.bfloat16, device=DEV)
    rtp.rtp_index_project(desc, W.to(DEV), q_pre.to(DEV), rtp.RTP_SIDE_QUERY, T, qI, T * 16, 0)
    torch.cuda.synchronize()
    want_k = orc.build_index_keys(W.numpy(), _bits(k_pre), ret, Hq, Hkv)
    got_k = _bits(kI)
    assert np.array_equal(got_k[:, t0:t0 + T], want_k)
    seven = _bits(torch.tensor([7.0], dtype=torch.bfloat16))[0]
    assert np.all(got_k[:, :t0] == seven) and np.all(got_k[:, t0 + T:] == seven)      # nothing else touched
    want_q = np.stack([orc.index_project(W.numpy()[j], _bits(q_pre)[:, h]) for j, h in enumerate(ret)])
    assert np.array_equal(_bits(qI), want_q)


# ---------------------------------------------------------------------------------------------------
# static top-k (Sec. 4.1 baseline)
# ---------------------------------------------------------------------------------------------------
def _score_rows(rng):
    rows = [rng.standard_normal(5000) * 2, rng.standard_normal(9001), np.full(300, -3.0),
            np.concatenate([[30.0], rng.standard_normal(3000)]), rng.standard_normal(1), rng.standard_normal(8193) * 0.01,
            np.round(rng.standard_normal(6000) * 4) / 4]                         # heavy ties
    s = rng.standard_normal(8191) * 2
    s[100:200] = -np.inf
    rows.append(s)
    return [r.astype(np.float32) for r in rows]


def test_topk_select_matches_oracle_with_ties_and_edge_budgets():
    print("[case] topk_select", flush=True)
    rng = np.random.default_rng(7)
    rows = _score_rows(rng)
    ks_per_row = [[1, 17, 4096, 4999, 5000, 6000], [1, 4096, 9001], [1, 10, 300, 301], [1, 2, 3001], [1, 5], [4096], [1, 100, 3000],
                  [1, 8000, 8091, 8092]]
    cases = [(r, k) for r, ks in enumerate(ks_per_row) for k in ks] + [(0, 0), (1, -3)]
    R = len(cases)
    n_max = max(len(s) for s in rows)
    stride = (n_max + 3) // 4 * 4
    sc = torch.full((R, stride), float("nan"), dtype=torch.float32)
    for i, (r, k) in enumerate(cases):
        sc[i, :len(rows[r])] = torch.from_numpy(rows[r])
    sc = sc.to(DEV)
    row_len = i32([len(rows[r]) for r, _ in cases])
    kk = i32([k for _, k in cases])
    sel = torch.full((R, stride), -1, dtype=torch.int32, device=DEV)
    cnt = torch.full((R,), -9, dtype=torch.int32, device=DEV)
    tau = torch.zeros(R, device=DEV)
    ws = torch.empty(rtp.rtp_topp_workspace_bytes(R, n_max), dtype=torch.uint8, device=DEV)
    for rep in range(2):                                  # twice: the workspace is reused dirty
        rtp.rtp_topk_select(sc, stride, row_len, kk, R, n_max, sel, stride, cnt, tau, ws)
        torch.cuda.synchronize()
        c, idx, t = cnt.cpu().numpy(), sel.cpu().numpy(), tau.cpu().numpy()
        for i, (r, k) in enumerate(cases):
            if k <= 0:
                assert c[i] == -1
                continue
            s64 = rows[r].astype(np.float64)
            finite = np.isfinite(s64)
            got = idx[i, :c[i]]
            assert np.all(np.diff(got) > 0), "positions must ascend"
            if k >= finite.sum():
                assert np.array_equal(got, np.nonzero(finite)[0])
                continue
            ref = orc.topk_select(np.where(finite, s64, -1e30), k)
            want = np.nonzero(finite & (s64 >= ref["tau"]))[0]      # every tie with the k-th score is kept
            assert np.array_equal(got, want), f"case {i}: {len(got)} vs {len(want)}"
            assert c[i] >= k and set(ref["idx"].tolist()) <= set(got.tolist())
            assert t[i] == np.float32(ref["tau"])


def test_topk_and_block_selectors_at_benchmark_size():
    """Configuration 2's score rows (131072 tokens, 64 planted), the budgets the benchmark compares:
    k = 4096 and the block-64 selector at p = 0.9, every row against the oracle."""
    print("[case] selectors at 131072", flush=True)
    w = wl.c2(DEV, seed=77, batch=2)
    run = DecodeRun(w, fuse_level1=False)
    run.index_score()
    sc = run.scores.cpu().numpy().astype(np.float64)
    run.topk(4096)
    sets, cnt = run.sel_sets()
    for r in range(run.R):
        ref = orc.topk_select(sc[r, :131072], 4096)
        want = np.nonzero(sc[r, :131072] >= ref["tau"])[0]
        assert np.array_equal(sets[r], want) and cnt[r] >= 4096
    run.block_topp()
    sets, cnt = run.sel_sets()
    thr = run.thr_bin.cpu().numpy()
    for r in range(run.R):
        ref = orc.block_topp_select(sc[r, :131072], float(w.p_rows[r].item()))
        assert np.array_equal(sets[r], ref["idx"]) and thr[r] == ref["threshold_bin"]


# ---------------------------------------------------------------------------------------------------
# block-wise histogram top-p (Sec. 3.4)
# ---------------------------------------------------------------------------------------------------
def test_block_topp_select_matches_oracle():
    print("[case] block_topp_select", flush=True)
    rng = np.random.default_rng(11)
    rows, ps = [], []

    def add(s, p):
        rows.append(np.asarray(s, dtype=np.float32))
        ps.append(p)

    base = rng.standard_normal(10000) * 1.5
    base[rng.integers(0, 10000, size=12)] += 7.0
    for p in (0.3, 0.8, 0.9, 0.95, 0.999, 1.0, 0.0):
        add(base, p)
    add(rng.standard_normal(64) * 2, 0.9)                                # exactly one block
    add(rng.standard_normal(65) * 2, 0.9)                                # a one-token ragged block
    add(rng.standard_normal(4096 + 63), 0.5)                             # chunk boundary + ragged tail
    add(rng.standard_normal(3 * 4096), 0.97)
    add(np.full(1000, 0.1), 0.5)                                         # every block in one bin
    add(np.clip(rng.standard_normal(777) * 8, -31.0, 31.0), 0.9)         # maxima over many bins, inside the binned range
    add([2.0], 0.7)
    planted = rng.standard_normal(131072).astype(np.float32)
    planted[rng.integers(0, 131072, size=64)] += 9.9
    add(planted, 0.9)                                                    # the benchmark's score law
    R = len(rows)
    n_max = max(len(s) for s in rows)
    stride = (n_max + 3) // 4 * 4
    sc = torch.full((R, stride), float("nan"), dtype=torch.float32)
    for r, s in enumerate(rows):
        sc[r, :len(s)] = torch.from_numpy(s)
    sc = sc.to(DEV)
    row_len = i32([len(s) for s in rows])
    p = torch.tensor(ps, dtype=torch.float32, device=DEV)
    sel = torch.full((R, stride), -1, dtype=torch.int32, device=DEV)
    cnt = torch.full((R,), -9, dtype=torch.int32, device=DEV)
    thr = torch.full((R,), -9, dtype=torch.int32, device=DEV)
    mass = torch.zeros(R, device=DEV)
    nbk = (n_max + 63) // 64
    mask = torch.full((R, nbk), 9, dtype=torch.uint8, device=DEV)
    ws = torch.empty(rtp.rtp_block_topp_workspace_bytes(R, n_max), dtype=torch.uint8, device=DEV)
    lo, width = -32.0, 0.25
    for rep in range(2):
        rtp.rtp_block_topp_select(sc, stride, row_len, p, R, n_max, 64, lo, width, sel, stride, cnt, thr, mass, mask, nbk, ws)
        torch.cuda.synchronize()
        c, idx, tb, ms, mk = cnt.cpu().numpy(), sel.cpu().numpy(), thr.cpu().numpy(), mass.cpu().numpy(), mask.cpu().numpy()
        for r, s in enumerate(rows):
            pr = ps[r]
            if not (pr > 0):
                assert c[r] == -1
                continue
            ref = orc.block_topp_select(s.astype(np.float64), float(np.float32(pr)), block=64, n_bins=256, bin_lo=lo, bin_width=width)
            assert c[r] == ref["count"], f"row {r}: {c[r]} vs {ref['count']}"
            assert np.array_equal(idx[r, :c[r]], ref["idx"]), f"row {r}"
            nb = len(ref["block_mask"])
            assert np.array_equal(mk[r, :nb].astype(bool), ref["block_mask"])
            if pr < 1:
                assert tb[r] == ref["threshold_bin"]
            assert abs(ms[r] - ref["mass"]) < 1e-6


def test_block_selector_feeds_sparse_attention():
    """Selection by blocks, then exact attention over the kept tokens: the output must match the oracle's
    attention over the oracle's block selection."""
    print("[case] block selector -> sparse attention", flush=True)
    w = wl.small_decode(DEV, seed=31, ctx=(700, 1531, 64, 2048))
    run = DecodeRun(w, fuse_level1=False)
    L = w.layer
    run.index_score()
    thr = torch.zeros(run.R, dtype=torch.int32, device=DEV)
    ws = ws_alloc(rtp.rtp_block_topp_workspace_bytes(run.R, run.max_ctx))
    rtp.rtp_block_topp_select(run.scores, run.stride, run.row_len, w.p_rows, run.R, run.max_ctx, 64, -32.0, 0.25,
                              run.sel_idx, run.stride, run.sel_count, thr, run.mass, None, 0, ws)
    run.sparse_attn()
    out = run.out_f64()
    sets, cnt = run.sel_sets()
    sc = run.scores.cpu().numpy().astype(np.float64)
    oi = oracle_inputs(w)
    sm = 1.0 / np.sqrt(128.0)
    for r in range(run.R):
        b, j = divmod(r, L.n_ret)
        n, t0 = w.ctx_len[b], w.seq_start[b]
        # staged: the oracle selects from the GPU's own fp32 scores
        ref = orc.block_topp_select(sc[r, :n], float(w.p_rows[r].item()))
        assert np.array_equal(sets[r], ref["idx"])
        h = L.ret_heads[j]
        kvh = orc.kv_head_of(h, L.n_q_heads, L.n_kv_heads)
        o, _ = orc.attend(oi["q_bits"][b, h], oi["K_bits"][kvh, t0:t0 + n], oi["V_bits"][kvh, t0:t0 + n], ref["idx"], sm)
        err = np.abs(out[b, h] - o)
        assert (err <= 2e-2 + 1e-2 * np.abs(o)).all() and (err <= 1e-3 + 2.0 ** -8 * np.abs(o)).all()


# ---------------------------------------------------------------------------------------------------
# sparsity figures (Sec. 3.2 last paragraph, Sec. 4.2 table)
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("ret_heads", [(0, 1, 5), (0, 4), (2,), (0, 1, 2, 3)])
def test_sparsity_stats_match_oracle(ret_heads):
    print(f"[case] sparsity_stats ret={ret_heads}", flush=True)
    w = wl.small_decode(DEV, seed=41, ctx=(700, 1531, 64, 2048), ret_heads=ret_heads)
    run = DecodeRun(w)
    L = w.layer
    run.step()
    lse_sel = run.lse.clone()
    dense_out, lse_full = torch.zeros_like(run.out), torch.zeros_like(run.lse)
    run.dense_attn(dense_out, lse_full)
    stats = torch.zeros((w.B, 4), dtype=torch.float32, device=DEV)
    unions = torch.zeros((w.B, L.n_kv_heads), dtype=torch.int32, device=DEV)
    rtp.rtp_sparsity_stats(run.desc, run.ctx_len, run.sel_idx, run.stride, run.sel_count, lse_sel, lse_full, w.B, stats, unions)
    nolse = torch.zeros((w.B, 4), dtype=torch.float32, device=DEV)
    rtp.rtp_sparsity_stats(run.desc, run.ctx_len, run.sel_idx, run.stride, run.sel_count, None, None, w.B, nolse, None)
    sets, cnt = run.sel_sets()
    st, un, nl = stats.cpu().numpy(), unions.cpu().numpy(), nolse.cpu().numpy()
    oi = oracle_inputs(w)
    sm = 1.0 / np.sqrt(128.0)
    for b in range(w.B):
        n, t0 = w.ctx_len[b], w.seq_start[b]
        attended, masses = [], []
        for h in range(L.n_q_heads):
            if h in L.ret_heads:
                s = sets[b * L.n_ret + L.ret_heads.index(h)]
                attended.append(s)
                kvh = orc.kv_head_of(h, L.n_q_heads, L.n_kv_heads)
                masses.append(orc.attention_mass(oi["q_bits"][b, h], oi["K_bits"][kvh, t0:t0 + n], s, sm))
            else:
                attended.append(orc.local_set(n - 1, L.sink, L.window))
        ref = orc.sparsity_stats(attended, n, L.n_q_heads, L.n_kv_heads, L.ret_heads)
        assert list(un[b]) == ref["union_sizes"]                                  # integers: exact
        assert abs(st[b, 0] - ref["compute_sparsity"]) < 1e-6
        assert abs(st[b, 1] - ref["memory_sparsity"]) < 1e-6
        assert abs(st[b, 2] - ref["active_tokens"]) < 1e-3
        # the mass comes from two fp32 log-sum-exps of bf16-rounded logits: 1e-3 is their rounding budget
        assert abs(st[b, 3] - float(np.mean(masses))) < 2e-3
        assert np.array_equal(nl[b, :3], st[b, :3]) and np.isnan(nl[b, 3])


# ---------------------------------------------------------------------------------------------------
# bounded (sink + window) cache of the all-local KV heads (Sec. 2.1; Sec. 3.2 last paragraph)
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("heads", [dict(n_q_heads=8, n_kv_heads=4, ret_heads=(0, 5)),      # G = 2, bounded heads 1 and 3
                                   dict(n_q_heads=8, n_kv_heads=2, ret_heads=(1,)),        # G = 4, bounded head 1
                                   dict(n_q_heads=4, n_kv_heads=4, ret_heads=(1, 3)),      # G = 1, bounded heads 0 and 2
                                   dict(n_q_heads=16, n_kv_heads=2, ret_heads=(9,)),       # G = 8, bounded head 0
                                   dict(n_q_heads=8, n_kv_heads=2, ret_heads=(1,), kv_dtype="fp16")])   # fp16 rows
def test_bounded_cache_fill_append_and_local_attention(heads):
    """The bounded cache filled after "prefill" and extended token by token holds the oracle's rows bit for
    bit; local attention read from it matches the oracle's local attention over the full cache -- with the
    full cache's rows of the bounded heads overwritten, to show they are never read."""
    print(f"[case] bounded cache {heads}", flush=True)
    sink, window = 4, 96
    cap = sink + window
    w = wl.small_decode(DEV, seed=51, ctx=(700, 1531, 64, 2048, 3, 100, 101), sink=sink, window=window, **heads)
    L = w.layer
    run = DecodeRun(w)
    ring_heads = rtp.rtp_kv_ring_heads(run.desc)
    assert ring_heads == orc.ring_kv_heads(L.n_q_heads, L.n_kv_heads, L.ret_heads) and len(ring_heads) > 0
    n_ring, B = len(ring_heads), w.B
    ring_K = torch.zeros((n_ring, B * cap + 5, 128), dtype=w.K.dtype, device=DEV)
    ring_V = torch.zeros_like(ring_K)
    ring_start = i64([b * cap + 5 for b in range(B)])                  # (an offset: the start array is honoured)
    hs = ring_K.shape[1] * 128
    # "prefill" leaves all but the last two tokens; the last two arrive one decode step at a time
    rtp.rtp_kv_ring_fill(run.desc, w.K, w.V, 128, w.K.shape[1] * 128, run.seq_start, i32([n - 2 for n in w.ctx_len]), B,
                         ring_K, ring_V, 128, hs, ring_start)
    for back in (2, 1):
        pos = [n - back for n in w.ctx_len]
        rows = torch.as_tensor([w.seq_start[b] + pos[b] for b in range(B)], device=DEV)
        k_new = w.K[:, rows].transpose(0, 1).contiguous()             # [B, n_kv_heads, 128]
        v_new = w.V[:, rows].transpose(0, 1).contiguous()
        rtp.rtp_kv_ring_append(run.desc, k_new, v_new, i32(pos), B, ring_K, ring_V, 128, hs, ring_start)
    torch.cuda.synchronize()
    Kb, Vb = wl.bf16_bits(w.K), wl.bf16_bits(w.V)
    rKb, rVb = wl.bf16_bits(ring_K), wl.bf16_bits(ring_V)
    for b in range(B):
        t0, n = w.seq_start[b], w.ctx_len[b]
        for i, kv in enumerate(ring_heads):
            ok, ov, rows_ = orc.ring_fill(Kb[kv, t0:t0 + n], Vb[kv, t0:t0 + n], n, sink, window)
            r0 = b * cap + 5
            assert np.array_equal(rKb[i, r0:r0 + rows_], ok[:rows_]) and np.array_equal(rVb[i, r0:r0 + rows_], ov[:rows_])

    # local attention: reference results first (full cache), then from the bounded cache with the full
    # cache's copies of the bounded heads destroyed
    run.local_attn()
    torch.cuda.synchronize()
    out_full, lse_full = run.out.clone(), run.lse.clone()
    ref = orc.decode_layer(**oracle_inputs(w))
    Kp, Vp = w.K.clone(), w.V.clone()
    Kp[ring_heads] = float("nan")
    Vp[ring_heads] = float("nan")
    out = torch.full_like(run.out, 5.0)
    lse = torch.full_like(run.lse, 5.0)
    ws = ws_alloc(rtp.rtp_local_attn_ring_workspace_bytes(run.desc, B, run.max_ctx))
    for rep in range(2):
        rtp.rtp_local_attn_ring(run.desc, w.q, Kp, Vp, 128, w.K.shape[1] * 128, run.seq_start, ring_K, ring_V, 128, hs,
                                ring_start, run.ctx_len, B, run.max_ctx, out, lse, ws)
    torch.cuda.synchronize()
    got, got_lse = out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy()
    loc = [h for h in range(L.n_q_heads) if h not in L.ret_heads]
    G = L.n_q_heads // L.n_kv_heads
    assert any(h // G in ring_heads for h in loc)
    for b in range(B):
        for h in loc:
            err = np.abs(got[b, h] - ref["out"][b, h])
            assert (err <= 1e-3 + 2.0 ** -8 * np.abs(ref["out"][b, h])).all(), f"b{b} h{h}: {err.max()}"
            assert abs(got_lse[b, h] - ref["lse"][b, h]) < 2e-3
    # retrieval heads' rows are left alone, and the two sources agree up to summation order
    ret = list(L.ret_heads)
    assert torch.all(out[:, ret] == 5.0)
    assert (out[:, loc].float() - out_full[:, loc].float()).abs().max().item() <= 2e-2
    assert (lse[:, loc] - lse_full[:, loc]).abs().max().item() <= 1e-4


# ---------------------------------------------------------------------------------------------------
# retrieval heads' cache in pages
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("page_size,kv_dtype", [(16, "bf16"), (64, "bf16"), (256, "bf16"), (64, "fp16")])
def test_paged_sparse_attention_matches_contiguous_and_oracle(page_size, kv_dtype):
    """The cache scattered into a shuffled page pool: the paged call must reproduce the contiguous call bit for
    bit (same rows, same order of arithmetic) and match the oracle's paged attention."""
    print(f"[case] paged sparse attention, page size {page_size}", flush=True)
    w = wl.small_decode(DEV, seed=61, ctx=(700, 1531, 64, 2048, 5000), kv_dtype=kv_dtype)
    L = w.layer
    run = DecodeRun(w)
    run.index_score()
    run.topp()
    run.sparse_attn()
    torch.cuda.synchronize()
    out_ref, lse_ref = run.out.clone(), run.lse.clone()
    # page tables: every sequence draws its pages from one shuffled pool
    g = torch.Generator().manual_seed(7)
    n_pages = [-(-n // page_size) for n in w.ctx_len]
    pool_pages = sum(n_pages) + 9
    perm = torch.randperm(pool_pages, generator=g)
    pt_stride = max(n_pages) + 2
    table = torch.full((w.B, pt_stride), -1, dtype=torch.int32)
    at = 0
    for b in range(w.B):
        table[b, :n_pages[b]] = perm[at:at + n_pages[b]].to(torch.int32)
        at += n_pages[b]
    K_pool = torch.full((L.n_kv_heads, pool_pages * page_size, 128), float("nan"), dtype=w.K.dtype, device=DEV)
    V_pool = torch.full_like(K_pool, float("nan"))
    for b in range(w.B):
        t0, n = w.seq_start[b], w.ctx_len[b]
        t = torch.arange(n)
        rows = (table[b, t // page_size].long() * page_size + t % page_size).to(DEV)
        K_pool[:, rows] = w.K[:, t0:t0 + n]
        V_pool[:, rows] = w.V[:, t0:t0 + n]
    table_d = table.to(DEV)
    out = torch.full_like(run.out, 2.0)
    lse = torch.full_like(run.lse, 2.0)
    for rep in range(2):
        rtp.rtp_sparse_attn_decode_paged(run.desc, w.q, K_pool, V_pool, 128, K_pool.shape[1] * 128, table_d, pt_stride,
                                         page_size, run.sel_idx, run.stride, run.sel_count, run.max_ctx, w.B, out, lse,
                                         run.ws_sparse)
    torch.cuda.synchronize()
    ret = list(L.ret_heads)
    assert torch.equal(out[:, ret], out_ref[:, ret]) and torch.equal(lse[:, ret], lse_ref[:, ret])
    loc = [h for h in range(L.n_q_heads) if h not in ret]
    assert torch.all(out[:, loc] == 2.0)                          # rows of the other heads are left alone
    # the oracle through the page table
    sets, cnt = run.sel_sets()
    qb, Kb, Vb = wl.bf16_bits(w.q), wl.bf16_bits(K_pool.nan_to_num(0.0)), wl.bf16_bits(V_pool.nan_to_num(0.0))
    got = out.float().cpu().numpy().astype(np.float64)
    G = L.n_q_heads // L.n_kv_heads
    for b in range(w.B):
        for j, h in enumerate(ret):
            o, l = orc.paged_attend(qb[b, h], Kb[h // G], Vb[h // G], table[b].numpy(), page_size, sets[b * L.n_ret + j],
                                    1.0 / np.sqrt(128.0), kv_dtype)
            err = np.abs(got[b, h] - o)
            assert (err <= 1e-3 + 2.0 ** -8 * np.abs(o)).all()
            assert abs(float(lse[b, h]) - l) < 2e-3


@pytest.mark.parametrize("case", ["g4", "g8_f16", "g1", "g2_bigbatch"])
def test_decode_attention_from_a_paged_cache(case):
    """Everything after the score pass with the whole K/V cache in pages (retrieval heads' gather and the local
    heads' sink + window rows through the page table): selections and outputs bit-identical to the contiguous
    call, and every head against the oracle's attention read through the table.  The cases cover the carried
    form (G = 2, 4, 8), the fall-back that runs the parts in turn (G = 1) and fp16 rows."""
    print(f"[case] decode attention from a paged cache, {case}", flush=True)
    kw = {"g4": dict(),
          "g8_f16": dict(n_q_heads=16, n_kv_heads=2, ret_heads=(3, 8), sink=4, window=700, kv_dtype="fp16"),
          "g1": dict(n_q_heads=4, n_kv_heads=4, ret_heads=(1, 3)),
          "g2_bigbatch": dict(n_q_heads=8, n_kv_heads=4, ret_heads=(0, 1, 6))}[case]
    ctx = (700, 1531, 64, 2048, 9000, 13) if case != "g2_bigbatch" else tuple(int(x) for x in
                                                                             np.random.default_rng(3).integers(5, 3000, size=40))
    page_size = 64 if case != "g1" else 16
    w = wl.small_decode(DEV, seed=71, ctx=ctx, **kw)
    L = w.layer
    run = DecodeRun(w)
    run.step_one_stream()
    torch.cuda.synchronize()
    want = (run.out.clone(), run.lse.clone(), run.sel_idx.clone(), run.sel_count.clone(), run.tau.clone(), run.mass.clone())
    # one shuffled pool for all sequences and KV heads
    g = torch.Generator().manual_seed(11)
    n_pages = [-(-n // page_size) for n in w.ctx_len]
    pool_pages = sum(n_pages) + 5
    perm = torch.randperm(pool_pages, generator=g)
    pt_stride = max(n_pages) + 1
    table = torch.full((w.B, pt_stride), -1, dtype=torch.int32)
    at = 0
    for b in range(w.B):
        table[b, :n_pages[b]] = perm[at:at + n_pages[b]].to(torch.int32)
        at += n_pages[b]
    K_pool = torch.full((L.n_kv_heads, pool_pages * page_size, 128), float("nan"), dtype=w.K.dtype, device=DEV)
    V_pool = torch.full_like(K_pool, float("nan"))
    for b in range(w.B):
        t0, n = w.seq_start[b], w.ctx_len[b]
        t = torch.arange(n)
        rows = (table[b, t // page_size].long() * page_size + t % page_size).to(DEV)
        K_pool[:, rows] = w.K[:, t0:t0 + n]
        V_pool[:, rows] = w.V[:, t0:t0 + n]
    table_d = table.to(DEV)
    for rep in range(2):
        run.out.fill_(3.0)
        run.lse.fill_(3.0)
        run.sel_idx.fill_(-1)
        run.sel_count.fill_(-9)
        run.index_score()
        rtp.rtp_decode_attention_paged(run.desc, run.scores, run.stride, run.row_len, w.p_rows, run.ctx_len, w.B, run.max_ctx,
                                       w.q, K_pool, V_pool, 128, K_pool.shape[1] * 128, table_d, pt_stride, page_size,
                                       run.sel_idx, run.stride, run.sel_count, run.tau, run.mass, run.out, run.lse,
                                       run.ws_topp, run.ws_fused, run.ws_local, level1_ready=1)
        run._level1_pending = False
        torch.cuda.synchronize()
        got = (run.out, run.lse, run.sel_idx, run.sel_count, run.tau, run.mass)
        for i, (a, b_) in enumerate(zip(want, got)):
            if i == 2:                                     # index lists: the written part
                cn = want[3].cpu().numpy()
                assert all(torch.equal(a[r, :max(cn[r], 0)], b_[r, :max(cn[r], 0)]) for r in range(run.R))
            else:
                assert torch.equal(a, b_), f"paged call differs from the contiguous one (output {i}, repeat {rep})"
    # and against the oracle reading through the table
    sets, cnt = run.sel_sets()
    qb, Kb, Vb = wl.bf16_bits(w.q), wl.bf16_bits(K_pool.nan_to_num(0.0)), wl.bf16_bits(V_pool.nan_to_num(0.0))
    out = run.out_f64()
    G = L.n_q_heads // L.n_kv_heads
    for b in range(w.B):
        for h in range(L.n_q_heads):
            ids = sets[b * L.n_ret + list(L.ret_heads).index(h)] if h in L.ret_heads else orc.local_set(w.ctx_len[b] - 1, L.sink, L.window)
            o, l = orc.paged_attend(qb[b, h], Kb[h // G], Vb[h // G], table[b].numpy(), page_size, ids, 1.0 / np.sqrt(128.0),
                                    L.kv_dtype)
            err = np.abs(out[b, h] - o)
            assert (err <= 1e-3 + 2.0 ** -8 * np.abs(o)).all(), f"b{b} h{h}: {err.max()}"
            assert abs(float(run.lse[b, h]) - l) < 2e-3
