"""GPU parity of the decode path (index score -> top-p -> sparse attention, local attention, dense
comparison) against the CPU oracle, element by element, through the C-ABI."""
import numpy as np
import pytest
import torch

from oracle import rtp_oracle as orc
from paper_2605_16928_amd import rtp, workloads as wl
from gpu_util import (DEV, DecodeRun, oracle_inputs, check_scores, check_selection, check_selection_valid, check_out,
                      check_layer, attend_reference, i32)

pytestmark = pytest.mark.gpu


def _cases():
    return {
        # ragged batch, two retrieval heads on one KV head, G = 4, contexts below and above sink+window
        "small": lambda: wl.small_decode(DEV),
        # fp32 projections (index query computed by the library), G = 4
        "small_proj": lambda: wl.small_decode(DEV, seed=12, index_mode="proj", ctx=(515, 2300, 129)),
        # G = 1 and G = 2
        "g1": lambda: wl.small_decode(DEV, seed=13, n_q_heads=4, n_kv_heads=4, ret_heads=(1, 3), ctx=(300, 9000)),
        "g2": lambda: wl.small_decode(DEV, seed=14, n_q_heads=8, n_kv_heads=4, ret_heads=(0, 1, 6), ctx=(4100, 77)),
        # configuration 1 at full size
        "c1": lambda: wl.c1(DEV),
        # configuration 2, shrunk: several top-p chunks and a ragged tail
        "c2_small": lambda: wl.c2(DEV, ctx=20000, batch=3, p=0.9),
        # configuration 5, shrunk: G = 8, ragged lengths, per-row p, flat and peaked rows
        "c5_small": lambda: wl.c5(DEV, batch=5, lo=3000, hi=40000),
        # the same head shape with a batch large enough for several local work items per carrying workgroup
        "c5_many": lambda: wl.c5(DEV, seed=6, batch=40, lo=100, hi=2500),
        # fp16 attention tensors (q, K, V, output): G = 4 ragged, G = 1 and 2, G = 8, configuration 2 shrunk
        "small_f16": lambda: wl.small_decode(DEV, seed=15, kv_dtype="fp16"),
        "g1_f16": lambda: wl.small_decode(DEV, seed=16, n_q_heads=4, n_kv_heads=4, ret_heads=(1, 3), ctx=(300, 9000), kv_dtype="fp16"),
        "g2_f16": lambda: wl.small_decode(DEV, seed=17, n_q_heads=8, n_kv_heads=4, ret_heads=(0, 1, 6), ctx=(4100, 77), kv_dtype="fp16"),
        "g8_f16": lambda: wl.small_decode(DEV, seed=18, n_q_heads=16, n_kv_heads=2, ret_heads=(3, 8), ctx=(2500, 130, 9000),
                                          sink=4, window=700, kv_dtype="fp16"),
        "c2_small_f16": lambda: wl.c2(DEV, ctx=20000, batch=3, p=0.9, kv_dtype="fp16"),
    }


@pytest.mark.parametrize("name", list(_cases()))
def test_decode_path_matches_oracle(name):
    print(f"[case] decode {name}", flush=True)
    w = _cases()[name]()
    run = DecodeRun(w)
    L = w.layer
    oi = oracle_inputs(w)
    ref = orc.decode_layer(**oi)

    # ---- stage 1: index query and scores ----
    run.index_score()
    torch.cuda.synchronize()
    qI_gpu = wl.bf16_bits(run.qI_out)
    assert np.array_equal(qI_gpu, ref["qI_bits"]), "index query bits differ"
    s_gpu = run.scores.cpu().numpy()
    row = 0
    for b in range(w.B):
        t0, n = w.seq_start[b], w.ctx_len[b]
        for j in range(L.n_ret):
            check_scores(s_gpu[row, :n], ref["scores"][row], ref["qI_bits"][b, j], oi["kI_bits"][j, t0:t0 + n],
                         f"{name} row {row}")
            row += 1

    # ---- stage 2: top-p on the GPU's own scores (isolates the selector) ----
    run.topp()
    sets, cnt = run.sel_sets()
    raw = run.sel_idx.cpu().numpy()
    for r in range(run.R):
        assert np.array_equal(raw[r, :cnt[r]], sets[r]), "selected positions must come out ascending"
    tau, mass = run.tau.cpu().numpy(), run.mass.cpu().numpy()
    for r in range(run.R):
        n = w.ctx_len[r // L.n_ret]
        p = float(w.p_rows[r])
        s64 = s_gpu[r, :n].astype(np.float64)
        rr = orc.topp_select(s64, p)
        check_selection(sets[r], s64, rr, p, f"{name} row {r} (same scores)")
        assert abs(tau[r] - rr["tau"]) <= 1e-5 * max(1.0, abs(rr["tau"]))
        assert abs(mass[r] - rr["mass"]) <= 1e-4
        # and end to end against the oracle's own scores
        slack = float(np.abs(s64 - ref["scores"][r]).max())
        check_selection_valid(sets[r], ref["scores"][r], p, slack, f"{name} row {r} (end to end)")
        assert abs(cnt[r] - ref["sel"][r]["count"]) <= 2 + int(1e-3 * ref["sel"][r]["count"])

    # ---- stage 3: sparse attention over the GPU's sets vs the oracle over the same sets ----
    run.sparse_attn()
    run.local_attn()
    out = run.out_f64()
    lse = run.lse.cpu().numpy()
    sc = 1.0 / np.sqrt(128.0)
    for b in range(w.B):
        t0, n = w.seq_start[b], w.ctx_len[b]
        for j, h in enumerate(L.ret_heads):
            kvh = h // (L.n_q_heads // L.n_kv_heads)
            o, l = orc.attend(oi["q_bits"][b, h], oi["K_bits"][kvh, t0:t0 + n], oi["V_bits"][kvh, t0:t0 + n],
                              sets[b * L.n_ret + j], sc, L.kv_dtype)
            check_out(out[b, h], o, f"{name} sparse b{b} h{h}")
            assert abs(lse[b, h] - l) < 2e-3

    # ---- stage 4: whole layer (retrieval + local rows) against the oracle end to end ----
    check_layer(out, lse, w, oi, ref, sets, f"{name} layer")

    # ---- dense comparison kernel ----
    dout = torch.zeros_like(run.out)
    dlse = torch.zeros_like(run.lse)
    run.dense_attn(dout, dlse)
    torch.cuda.synchronize()
    dref = orc.decode_layer(**oi, dense=True)
    check_out(dout.float().cpu().numpy().astype(np.float64), dref["out"], f"{name} dense")
    assert np.allclose(dlse.cpu().numpy(), dref["lse"], atol=2e-3, rtol=0)


def test_topp_edge_rows():
    """Hand-made score rows: ties at the threshold, uniform rows, p = 1, invalid p, -inf entries,
    a single element, lengths that are not multiples of 4."""
    print("[case] topp edge rows", flush=True)
    rng = np.random.default_rng(3)
    n_max = 9001
    stride = 9004
    rows, ps = [], []

    def add(s, p):
        rows.append(np.asarray(s, dtype=np.float32))
        ps.append(p)

    add(np.log(np.array([8, 4, 2, 1, 1], dtype=np.float64)), 0.9)       # tie at the threshold: both kept
    add(np.log(np.array([8, 4, 2, 1, 1], dtype=np.float64)), 0.45)
    add(np.log(np.array([8, 4, 2, 1, 1], dtype=np.float64)), 0.7)
    add(np.full(8, 0.25), 0.875)                                        # uniform: every entry ties
    add(np.full(9001, -3.0), 0.3)
    add(rng.standard_normal(9001), 1.0)                                 # keep everything
    add(rng.standard_normal(5000), 0.0)                                 # invalid p
    add(rng.standard_normal(5000), float("nan"))
    add([1.5], 0.9)                                                     # single element
    s = rng.standard_normal(8191) * 2
    s[100:200] = -np.inf                                                # masked entries are never selected
    add(s, 0.999)
    add(rng.standard_normal(8193) * 0.01, 0.5)                          # flat
    add(np.concatenate([[30.0], rng.standard_normal(3000)]), 0.9)       # one spike
    add(-np.arange(40) * np.log(2.0), 0.999)                            # geometric
    add(np.concatenate([rng.standard_normal(4097), [np.float32(-0.0), np.float32(0.0)]]), 0.7)
    R = len(rows)
    sc = torch.full((R, stride), float("nan"), dtype=torch.float32)
    for r, s in enumerate(rows):
        sc[r, :len(s)] = torch.from_numpy(s)
    sc = sc.to(DEV)
    row_len = i32([len(s) for s in rows])
    p = torch.tensor(ps, dtype=torch.float32, device=DEV)
    sel = torch.full((R, stride), -1, dtype=torch.int32, device=DEV)
    cnt = torch.full((R,), -9, dtype=torch.int32, device=DEV)
    tau = torch.zeros(R, device=DEV)
    mass = torch.zeros(R, device=DEV)
    ws = torch.empty(rtp.rtp_topp_workspace_bytes(R, n_max), dtype=torch.uint8, device=DEV)
    for rep in range(2):                      # twice: the workspace is reused dirty
        rtp.rtp_topp_select(sc, stride, row_len, p, R, n_max, sel, stride, cnt, tau, mass, ws)
        torch.cuda.synchronize()
        c = cnt.cpu().numpy()
        idx = sel.cpu().numpy()
        t = tau.cpu().numpy()
        for r, s in enumerate(rows):
            pr = ps[r]
            if not (pr > 0):
                assert c[r] == -1
                continue
            got = np.sort(idx[r, :c[r]])
            s64 = s.astype(np.float64)
            finite = np.isfinite(s64)
            if pr >= 1:
                assert np.array_equal(got, np.nonzero(finite)[0])
                continue
            ref = orc.topp_select(np.where(finite, s64, -1e30), pr)
            # the library keeps ALL ties at the threshold
            want = np.nonzero(finite & (s64 >= ref["tau"]))[0]
            assert np.array_equal(got, want), f"row {r}: {len(got)} vs {len(want)}"
            assert t[r] == np.float32(ref["tau"])
    assert c[0] == 5 and c[1] == 1 and c[2] == 2 and c[3] == 8 and c[8] == 1
    assert c[4] == 9001                        # all-equal row: every entry ties with the threshold


def test_topp_large_score_magnitudes():
    """The indexer equation (Sec. 3.2) has no scale, so scores far from 0 are reachable.  The selector's masses
    are fixed point relative to the edge of a score's quarter binade: rows whose largest score lies inside
    (-128, 128) must match the oracle as any other row (spread-out rows, rows sitting at +-100, a row whose
    tail reaches below -128), rows whose largest score lies outside are reported with sel_count = -2."""
    print("[case] topp large magnitudes", flush=True)
    rng = np.random.default_rng(8)
    n_max = 131072
    stride = n_max
    rows, ps = [], []

    def add(s, p):
        rows.append(np.asarray(s, dtype=np.float32))
        ps.append(p)

    add(rng.standard_normal(50000) * 20.0, 0.9)                      # spread over +-90
    add(rng.standard_normal(50000) * 20.0, 0.999)
    add(100.0 + rng.standard_normal(131072), 0.9)                    # everything in [96, 104]: bins 8 and 16 wide
    add(100.0 + rng.standard_normal(131072) * 0.3, 0.95)
    add(-100.0 + rng.standard_normal(70001), 0.9)
    add(np.concatenate([[127.9], 64.5 + rng.standard_normal(30000) * 3.0]), 0.99)   # maximum just inside
    add(np.concatenate([rng.standard_normal(9000) * 40.0 - 120.0, [5.0]]), 0.9)     # tail far below -128
    add(64.01 + rng.random(131072) * 0.5, 0.5)                       # bottom of a 16-wide bin, flat
    add(np.concatenate([[128.0], rng.standard_normal(5000)]), 0.9)   # unsupported: maximum at +128
    add(rng.standard_normal(5000) * 50.0 + 200.0, 0.9)               # unsupported
    add(-128.0 - rng.random(5000) * 30.0, 0.9)                       # unsupported: maximum <= -128
    n_bad = 3
    R = len(rows)
    sc = torch.full((R, stride), float("nan"), dtype=torch.float32)
    for r, s in enumerate(rows):
        sc[r, :len(s)] = torch.from_numpy(s)
    sc = sc.to(DEV)
    row_len = i32([len(s) for s in rows])
    p = torch.tensor(ps, dtype=torch.float32, device=DEV)
    sel = torch.full((R, stride), -1, dtype=torch.int32, device=DEV)
    cnt = torch.full((R,), -9, dtype=torch.int32, device=DEV)
    tau = torch.zeros(R, device=DEV)
    mass = torch.zeros(R, device=DEV)
    ws = torch.empty(rtp.rtp_topp_workspace_bytes(R, n_max), dtype=torch.uint8, device=DEV)
    rtp.rtp_topp_select(sc, stride, row_len, p, R, n_max, sel, stride, cnt, tau, mass, ws)
    torch.cuda.synchronize()
    c, idx, t, m = cnt.cpu().numpy(), sel.cpu().numpy(), tau.cpu().numpy(), mass.cpu().numpy()
    for r, s in enumerate(rows):
        if r >= R - n_bad:
            assert c[r] == -2, f"row {r}: count {c[r]}, expected the unsupported-magnitude mark"
            continue
        s64 = s.astype(np.float64)
        ref = orc.topp_select(s64, ps[r])
        check_selection(np.sort(idx[r, :c[r]]), s64, ref, ps[r], f"row {r}")
        assert t[r] == np.float32(ref["tau"]) and abs(m[r] - ref["mass"]) <= 1e-4, (r, t[r], ref["tau"], m[r], ref["mass"])


def test_decode_step_with_an_index_scale():
    """index_scale = 8 puts the planted scores of configuration 2's law near 80 and the background over +-35:
    the whole step against the oracle; index_scale = 16 moves the planted scores past 128: every retrieval row
    is reported unsupported (sel_count = -2, zero output rows), the local heads are served as always."""
    print("[case] decode step with an index scale", flush=True)
    w = wl.c2("cpu", ctx=20000, batch=2, p=0.9, seed=9)
    w.layer.index_scale = 8.0
    w = w.to(DEV)
    oi = oracle_inputs(w)
    ref = orc.decode_layer(**oi)
    assert max(float(s.max()) for s in ref["scores"]) > 64.0
    for fuse in (False, True):
        run = DecodeRun(w, fuse_level1=fuse)
        run.step_one_stream()
        sets, cnt = run.sel_sets()
        s_gpu = run.scores.cpu().numpy()
        for r in range(run.R):
            n = w.ctx_len[r // w.layer.n_ret]
            slack = float(np.abs(s_gpu[r, :n] - ref["scores"][r]).max())
            assert slack <= 1e-5 * 80.0
            check_selection_valid(sets[r], ref["scores"][r], float(w.p_rows[r]), slack, f"scale 8 row {r}")
        check_layer(run.out_f64(), run.lse.cpu().numpy(), w, oi, ref, sets, "scale 8")
    w.layer.index_scale = 16.0
    oi = oracle_inputs(w)
    ref = orc.decode_layer(**oi)
    assert min(float(s.max()) for s in ref["scores"]) > 128.0
    L = w.layer
    for form in ("five", "one_call"):
        run = DecodeRun(w)
        run.out.fill_(3.0)
        if form == "five":
            run.step()
        else:
            run.step_one_stream()
        out = run.out_f64()
        assert (run.sel_count == -2).all(), run.sel_count.tolist()
        for h in range(L.n_q_heads):
            if h in L.ret_heads:
                assert np.all(out[:, h] == 0.0)
            else:
                check_out(out[:, h], ref["out"][:, h], f"scale 16 local head {h}")


def test_sparse_attn_degenerate_sets():
    """Empty sets, single-token sets, a set that is the whole context, unsorted index lists."""
    print("[case] sparse degenerate sets", flush=True)
    w = wl.small_decode(DEV, seed=21, ctx=(300, 1000, 50))
    run = DecodeRun(w)
    L = w.layer
    oi = oracle_inputs(w)
    rng = np.random.default_rng(5)
    sets = []
    for r in range(run.R):
        n = w.ctx_len[r // L.n_ret]
        kind = r % 5
        if kind == 0:
            s = np.array([], dtype=np.int64)
        elif kind == 1:
            s = np.array([n - 1])
        elif kind == 2:
            s = rng.permutation(n)                         # everything, shuffled
        elif kind == 3:
            s = rng.choice(n, size=min(n, 129), replace=False)
        else:
            s = np.arange(0, n, 3)
        sets.append(s)
    idx = torch.zeros((run.R, run.stride), dtype=torch.int32)
    for r, s in enumerate(sets):
        idx[r, :len(s)] = torch.from_numpy(s.astype(np.int32))
    cnt = i32([len(s) for s in sets])
    run.out.fill_(7.0)
    run.sparse_attn(idx.to(DEV), cnt)
    out = run.out_f64()
    lse = run.lse.cpu().numpy()
    sc = 1.0 / np.sqrt(128.0)
    for b in range(w.B):
        t0, n = w.seq_start[b], w.ctx_len[b]
        for j, h in enumerate(L.ret_heads):
            r = b * L.n_ret + j
            kvh = h // (L.n_q_heads // L.n_kv_heads)
            if len(sets[r]) == 0:
                assert np.all(out[b, h] == 0) and lse[b, h] == -np.inf
                continue
            o, l = orc.attend(oi["q_bits"][b, h], oi["K_bits"][kvh, t0:t0 + n], oi["V_bits"][kvh, t0:t0 + n], sets[r], sc)
            check_out(out[b, h], o, f"row {r}")
            if len(sets[r]) == 1:
                assert np.array_equal(out[b, h], orc.bf16_to_f64(oi["V_bits"][kvh, t0 + sets[r][0]]))
        for h in range(L.n_q_heads):
            if h not in L.ret_heads:
                assert np.all(out[b, h] == 7.0)            # local rows are not touched by the sparse call


def test_local_attn_short_contexts_and_interleaved_kv():
    """Contexts of 1, below sink, exactly sink+window, and K|V interleaved rows (row stride 256)."""
    print("[case] local short contexts / interleaved KV", flush=True)
    w = wl.small_decode(DEV, seed=31, ctx=(1, 3, 100, 101, 5000), sink=4, window=96, p=(0.9,) * 5, n_planted=0)
    L = w.layer
    oi = oracle_inputs(w)
    ref = orc.decode_layer(**oi)
    run = DecodeRun(w)
    run.step()
    check_out(run.out_f64(), ref["out"], "short contexts")
    # interleave K and V rows: element (kvh, t, :) of K at kv[kvh, t, 0:128], of V at kv[kvh, t, 128:256]
    kv = torch.cat([w.K, w.V], dim=2).contiguous()
    T = w.T_tot
    out2 = torch.zeros_like(run.out)
    Kp, Vp = kv.data_ptr(), kv.data_ptr() + 256
    rtp.rtp_local_attn(run.desc, w.q, Kp, Vp, 256, T * 256, run.seq_start, run.ctx_len, None, w.B, 1, run.max_ctx,
                       out2, None, run.ws_local)
    rtp.rtp_sparse_attn_decode(run.desc, w.q, Kp, Vp, 256, T * 256, run.seq_start, run.sel_idx, run.stride,
                               run.sel_count, run.max_ctx, w.B, out2, None, run.ws_sparse)
    torch.cuda.synchronize()
    assert torch.equal(out2, run.out)


def test_level1_in_score_pass_gives_the_same_selection():
    """The score pass accumulating the selector's first histogram level, and the selector doing it
    itself, must give the same bits -- also on repeated steps (the workspace is handed back initialised)."""
    print("[case] level-1 histogram fused into the score pass", flush=True)
    for w in (wl.c2(DEV, ctx=50000, batch=2, p=0.9), wl.c5(DEV, batch=3, lo=3000, hi=30000),
              wl.small_decode(DEV, seed=12, index_mode="proj", ctx=(515, 2300, 129))):
        res = {}
        for fuse in (False, True):
            run = DecodeRun(w, fuse_level1=fuse)
            for rep in range(3):
                run.sel_idx.fill_(-1)
                run.index_score()
                run.topp()
                torch.cuda.synchronize()
            res[fuse] = (run.scores.clone(), run.sel_idx.clone(), run.sel_count.clone(), run.tau.clone(), run.mass.clone())
        assert int(res[True][2].min()) > 0
        for a, b in zip(res[False], res[True]):
            assert torch.equal(a, b, ) if a.dtype != torch.float32 else torch.equal(a.nan_to_num(), b.nan_to_num())


_attend_reference = attend_reference


@pytest.mark.parametrize("name", ["small", "small_proj", "g1", "g2", "c2_small", "c5_small", "small_f16", "g1_f16", "c2_small_f16"])
@pytest.mark.parametrize("fuse", [False, True])
def test_select_attend_in_one_call_matches_oracle_and_the_two_calls(name, fuse):
    """rtp_select_attend_decode: the selection must be the oracle's top-p set of the same scores, the
    output the oracle's attention over that set, and every selection output bit-identical to
    rtp_topp_select's; twice in a row, the workspaces reused as the call left them."""
    print(f"[case] select+attend {name} level1-in-score-pass={fuse}", flush=True)
    w = _cases()[name]()
    L = w.layer
    oi = oracle_inputs(w)
    two = DecodeRun(w, fuse_level1=fuse)
    two.index_score()
    two.topp()
    two.sparse_attn()
    torch.cuda.synchronize()
    run = DecodeRun(w, fuse_level1=fuse)
    for rep in range(2):
        run.sel_idx.fill_(-1)
        run.sel_count.fill_(-9)
        run.out.zero_()
        run.lse.zero_()
        run.index_score()
        run.select_attend()
        sets, cnt = run.sel_sets()
        assert torch.equal(run.sel_count, two.sel_count)
        for r in range(run.R):
            assert torch.equal(run.sel_idx[r, :cnt[r]], two.sel_idx[r, :cnt[r]])
        assert torch.equal(run.tau, two.tau) and torch.equal(run.mass, two.mass)
        s_gpu = run.scores.cpu().numpy()
        for r in range(run.R):
            n = w.ctx_len[r // L.n_ret]
            s64 = s_gpu[r, :n].astype(np.float64)
            p = float(w.p_rows[r])
            check_selection(sets[r], s64, orc.topp_select(s64, p), p, f"{name} row {r}")
        out, lse = run.out_f64(), run.lse.cpu().numpy()
        ref = _attend_reference(w, oi, sets)
        for (b, h), (o, l) in ref.items():
            check_out(out[b, h], o, f"{name} b{b} h{h}")
            assert abs(lse[b, h] - l) < 2e-3
        ret = list(L.ret_heads)
        assert (run.out[:, ret].float() - two.out[:, ret].float()).abs().max().item() <= 2e-2


def test_select_attend_degenerate_rows():
    """Rows that keep everything (p = 1), invalid rows (p = 0), a row without a finite score and contexts
    shorter than one chunk, next to ordinary rows of the same batch."""
    print("[case] select+attend degenerate rows", flush=True)
    w = wl.small_decode(DEV, seed=21, ctx=(700, 5000, 9, 4097))
    L = w.layer
    oi = oracle_inputs(w)
    p = w.p_rows.clone()
    p[0] = 1.0                       # sequence 0, first retrieval head: keep everything
    p[1] = 0.0                       # invalid
    p[5] = float("nan")              # invalid
    w.p_rows = p
    run = DecodeRun(w, fuse_level1=False)
    dead = 3                         # sequence 1, first retrieval head: no finite score
    for rep in range(2):
        run.out.fill_(7.0)
        run.lse.fill_(7.0)
        run.index_score()
        run.scores[dead, :] = float("-inf")
        if rep == 0:
            run.select_attend()
        else:
            run.decode_attention()             # the same with the local heads on board
        sets, cnt = run.sel_sets()
        assert cnt[0] == w.ctx_len[0] and cnt[1] == -1 and cnt[5] == -1 and cnt[dead] == 0
        out, lse = run.out_f64(), run.lse.cpu().numpy()
        sets = [s if c > 0 else np.zeros(0, dtype=np.int64) for s, c in zip(sets, cnt)]
        ref = _attend_reference(w, oi, sets)
        for r in range(run.R):
            b, h = r // L.n_ret, L.ret_heads[r % L.n_ret]
            if cnt[r] <= 0:
                assert np.all(out[b, h] == 0.0) and lse[b, h] == -np.inf
            else:
                check_out(out[b, h], ref[(b, h)][0], f"row {r}")
                assert abs(lse[b, h] - ref[(b, h)][1]) < 2e-3


@pytest.mark.parametrize("name", ["small", "g1", "g2", "c2_small", "c5_small", "c5_many", "small_f16", "g1_f16", "g2_f16",
                                  "g8_f16", "c2_small_f16"])
def test_decode_attention_in_one_call_matches_oracle(name):
    """rtp_decode_attention: everything after the score pass -- the layer's output (retrieval and local rows)
    against the oracle end to end, the selection bit-identical to rtp_topp_select's, twice in a row.  The cases
    cover the carried form (G = 2, 4, and 8 with a small batch) and the fall-back (G = 1; G = 8 with a large batch)."""
    print(f"[case] decode attention in one call {name}", flush=True)
    w = _cases()[name]()
    L = w.layer
    oi = oracle_inputs(w)
    ref = orc.decode_layer(**oi)
    two = DecodeRun(w)
    two.index_score()
    two.topp()
    torch.cuda.synchronize()
    run = DecodeRun(w)
    for rep in range(2):
        run.sel_idx.fill_(-1)
        run.sel_count.fill_(-9)
        run.out.fill_(3.0)
        run.lse.fill_(3.0)
        run.step_one_stream()
        sets, cnt = run.sel_sets()
        assert torch.equal(run.sel_count, two.sel_count) and torch.equal(run.tau, two.tau)
        for r in range(run.R):
            assert torch.equal(run.sel_idx[r, :cnt[r]], two.sel_idx[r, :cnt[r]])
        out, lse = run.out_f64(), run.lse.cpu().numpy()
        # retrieval rows: the oracle's attention over the GPU's sets; local rows: the oracle's layer
        att = _attend_reference(w, oi, sets)
        for b in range(w.B):
            for h in range(L.n_q_heads):
                if h in L.ret_heads:
                    o, l = att[(b, h)]
                else:
                    o, l = ref["out"][b, h], ref["lse"][b, h]
                check_out(out[b, h], o, f"{name} b{b} h{h}")
                assert abs(lse[b, h] - l) < 2e-3
        check_layer(out, lse, w, oi, ref, sets, f"{name} layer")


def test_decode_step_replays_from_a_hip_graph():
    """The step (score pass + rtp_decode_attention) captured once and replayed: every replay, with eager steps
    of another copy and synchronisations in between, must reproduce the eager result bit for bit (the library
    records kernel launches only: no memset nodes, no allocation, no host synchronisation)."""
    print("[case] decode step in a HIP graph", flush=True)
    w = wl.c2(DEV, ctx=20000, batch=3, p=0.9)
    run, other = DecodeRun(w), DecodeRun(wl.c2(DEV, seed=5, ctx=9000, batch=2, p=0.8))
    run.step_one_stream()
    torch.cuda.synchronize()
    want = (run.out.clone(), run.lse.clone(), run.sel_idx.clone(), run.sel_count.clone(), run.tau.clone())
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        run.step_one_stream()
    for rep in range(3):
        run.out.zero_()
        run.sel_count.zero_()
        other.step_one_stream()                      # eager work of the same library between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = (run.out, run.lse, run.sel_idx, run.sel_count, run.tau)
        for a, b in zip(want, got):
            assert torch.equal(a, b), f"replay {rep} differs from the eager step"


def test_select_attend_with_clustered_kept_tokens():
    """Rows whose kept tokens sit mostly in one 8192-score chunk (recent tokens, or a run in the middle of the
    context): the one-call forms then hand every workgroup of the row an equal share of the row's ranks, taken
    from other chunks than its own.  Selection outputs must stay bit-identical to rtp_topp_select's, the
    attention must be the oracle's over that set; rtp_decode_attention must agree with the two separate
    calls on every head.  Rows of the same batch that stay spread out take the ordinary path."""
    print("[case] select+attend clustered", flush=True)
    w = wl.small_decode(DEV, seed=29, ctx=(40000, 70000, 9000, 33000))
    L = w.layer
    oi = oracle_inputs(w)

    def boost(run):
        s = run.scores
        for r in range(run.R):
            n = w.ctx_len[r // L.n_ret]
            if r % 4 == 0:
                s[r, max(0, n - 6000):n] += 4.0          # recency: the last chunk(s) hold nearly all of the set
            elif r % 4 == 1:
                s[r, 9000:15000] += 3.0                   # a run inside the second chunk
            elif r % 4 == 2:
                s[r, 100:300] += 8.0                      # a short run: few tokens, all in the first chunk
            # r % 4 == 3: left as generated

    two = DecodeRun(w, fuse_level1=False)
    two.index_score()
    boost(two)
    two.topp()
    two.sparse_attn()
    two.local_attn()
    torch.cuda.synchronize()
    cnt2 = two.sel_count.cpu().numpy()
    clustered_rows = 0
    for r in range(two.R):
        n = w.ctx_len[r // L.n_ret]
        n_chunks = (n + 8191) // 8192
        per_chunk = np.bincount(two.sel_idx[r, :cnt2[r]].cpu().numpy() // 8192, minlength=n_chunks)
        clustered_rows += int(n_chunks > 1 and per_chunk.max() > 5 * (cnt2[r] // n_chunks) // 4 + 400)
    assert clustered_rows >= 3, "the test's score laws no longer cluster the kept tokens"

    for form in ("select_attend", "decode_attention"):
        run = DecodeRun(w, fuse_level1=False)
        for rep in range(2):
            run.sel_idx.fill_(-1)
            run.sel_count.fill_(-9)
            run.out.zero_()
            run.lse.zero_()
            run.index_score()
            boost(run)
            getattr(run, form)()
            sets, cnt = run.sel_sets()
            assert torch.equal(run.sel_count, two.sel_count), form
            for r in range(run.R):
                assert torch.equal(run.sel_idx[r, :cnt[r]], two.sel_idx[r, :cnt[r]]), (form, r)
            assert torch.equal(run.tau, two.tau) and torch.equal(run.mass, two.mass)
            out, lse = run.out_f64(), run.lse.cpu().numpy()
            ref = _attend_reference(w, oi, sets)
            for (b, h), (o, l) in ref.items():
                check_out(out[b, h], o, f"clustered {form} b{b} h{h}")
                assert abs(lse[b, h] - l) < 2e-3
            heads = list(L.ret_heads) if form == "select_attend" else list(range(L.n_q_heads))
            assert (run.out[:, heads].float() - two.out[:, heads].float()).abs().max().item() <= 2e-2
    s_gpu = two.scores.cpu().numpy()
    sets, _ = two.sel_sets()
    for r in range(two.R):
        n = w.ctx_len[r // L.n_ret]
        s64 = s_gpu[r, :n].astype(np.float64)
        p = float(w.p_rows[r])
        check_selection(sets[r], s64, orc.topp_select(s64, p), p, f"clustered row {r}")
