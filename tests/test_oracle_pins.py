"""Pins for the CPU oracle: every check here compares the oracle with something
that is NOT the oracle -- exact rational arithmetic, pure-Python brute force,
closed forms, hand-worked cases, or invariants of the definition -- so that a
dropped term, a wrong sign or index, or a transposed operand fails a test.

Citations are to the paper's Section 3.2 (indexer equation, sparse-attention
equation, Top-P active set), Section 3.4 (mass "reaches p") and Section 4.2
(sink + window rule for local heads).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import rtp_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- helpers (independent of the oracle)
def f32_to_bf16_bits_by_torch(x_f32: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.asarray(x_f32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bf16_fraction(bits: int) -> Fraction:
    """Exact rational value of one bf16 bit pattern (normal numbers and zero)."""
    sign = -1 if bits & 0x8000 else 1
    e = (bits >> 7) & 0xFF
    man = bits & 0x7F
    if e == 0:
        return Fraction(sign * man, 1 << 133)          # subnormal: man * 2^-7 * 2^-126
    return sign * Fraction(128 + man, 128) * (Fraction(2) ** (e - 127))


def rand_bf16(rng, shape, std=1.0):
    return f32_to_bf16_bits_by_torch(rng.standard_normal(shape).astype(np.float32) * std)


def brute_attention(q, K, V, ids, scale):
    """Textbook two-pass softmax attention in pure Python floats."""
    logits = [scale * sum(q[c] * K[n][c] for c in range(len(q))) for n in ids]
    mx = max(logits)
    ex = [math.exp(l - mx) for l in logits]
    den = sum(ex)
    out = [sum(ex[i] * V[n][c] for i, n in enumerate(ids)) / den for c in range(len(q))]
    return out, mx + math.log(den)


def online_attention(q, K, V, ids, scale):
    """The same quantity a second way: one pass with a running max (online softmax)."""
    m, l, acc = -math.inf, 0.0, [0.0] * len(q)
    for n in ids:
        s = scale * sum(q[c] * K[n][c] for c in range(len(q)))
        m_new = max(m, s)
        corr = math.exp(m - m_new) if m != -math.inf else 0.0
        pw = math.exp(s - m_new)
        l = l * corr + pw
        acc = [a * corr + pw * V[n][c] for c, a in enumerate(acc)]
        m = m_new
    return [a / l for a in acc], m + math.log(l)


# ---------------------------------------------------------------- number formats
def test_bf16_widening_known_patterns():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3F00, 0x0000, 0x4049, 0x3F81], dtype=np.uint16)
    want = [1.0, -1.0, 2.0, 0.5, 0.0, 3.140625, 1.0078125]
    assert orc.bf16_to_f64(bits).tolist() == want


def test_bf16_widening_matches_exact_rationals():
    rng = np.random.default_rng(0)
    bits = rand_bf16(rng, (200,), 3.0)
    got = orc.bf16_to_f64(bits)
    for b, g in zip(bits.tolist(), got.tolist()):
        assert Fraction(g) == bf16_fraction(b)


def test_bf16_rounding_ties_to_even_and_single_rounding():
    x = np.array([1.0,
                  1.0 + 2.0 ** -8,               # tie between 0x3F80 and 0x3F81 -> even
                  1.0 + 3 * 2.0 ** -8,           # tie between 0x3F81 and 0x3F82 -> even
                  1.0 + 2.0 ** -8 + 2.0 ** -40,  # just above the tie: must round UP (a detour
                                                 # through float32 would drop 2^-40 and tie down)
                  -(1.0 + 2.0 ** -8 + 2.0 ** -40),
                  0.0, 255.5, 1e-3])
    got = orc.f64_to_bf16_bits(x)
    assert got[0] == 0x3F80 and got[1] == 0x3F80 and got[2] == 0x3F82
    assert got[3] == 0x3F81 and got[4] == 0xBF81 and got[5] == 0
    assert got[6] == 0x4380            # 255.5 -> 256 (tie to even mantissa, carries into the exponent)
    # float32-representable inputs: one rounding == torch's RNE conversion
    rng = np.random.default_rng(1)
    y = (rng.standard_normal(5000) * np.exp(rng.uniform(-6, 6, 5000))).astype(np.float32)
    assert np.array_equal(orc.f64_to_bf16_bits(y.astype(np.float64)), f32_to_bf16_bits_by_torch(y))


# ---------------------------------------------------------------- indexer (Sec. 3.2, indexer equation)
def test_index_score_exact_against_rationals():
    rng = np.random.default_rng(2)
    q = rand_bf16(rng, (16,))
    k = rand_bf16(rng, (37, 16))
    got = orc.index_score(q, k, 1.0)
    for n in range(37):
        exact = sum(bf16_fraction(int(q[i])) * bf16_fraction(int(k[n, i])) for i in range(16))
        assert abs(Fraction(float(got[n])) - exact) <= abs(exact) * Fraction(1, 10 ** 14) + Fraction(1, 10 ** 18)


def test_index_score_unit_query_returns_key_column_and_scale():
    rng = np.random.default_rng(3)
    k = rand_bf16(rng, (50, 16))
    for i in (0, 7, 15):
        e = np.zeros(16, dtype=np.uint16)
        e[i] = 0x3F80
        assert np.array_equal(orc.index_score(e, k, 1.0), orc.bf16_to_f64(k[:, i]))
        assert np.array_equal(orc.index_score(e, k, 0.5), 0.5 * orc.bf16_to_f64(k[:, i]))


def test_index_project_exact_against_rationals():
    rng = np.random.default_rng(4)
    W = (rng.standard_normal((16, 128)) / math.sqrt(128)).astype(np.float32)
    x = rand_bf16(rng, (3, 128))
    got = orc.index_project(W, x)
    assert got.shape == (3, 16) and got.dtype == np.uint16
    for b in range(3):
        for i in range(16):
            exact = sum(Fraction(float(W[i, c])) * bf16_fraction(int(x[b, c])) for c in range(128))
            g = bf16_fraction(int(got[b, i]))
            ulp = Fraction(2) ** (math.floor(math.log2(abs(float(exact)))) - 7)
            assert abs(g - exact) <= ulp / 2          # correctly rounded to 8 significant bits


def test_index_project_is_not_transposed():
    W = np.zeros((16, 128), dtype=np.float32)
    W[3, 100] = 2.0
    x = np.zeros((128,), dtype=np.uint16)
    x[100] = 0x3FC0                                    # 1.5
    got = orc.bf16_to_f64(orc.index_project(W, x))
    want = np.zeros(16)
    want[3] = 3.0
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- top-p (Sec. 3.2 Top-P, Sec. 3.4)
def _read_hand_cases():
    cases = []
    with open(os.path.join(GOLD, "topp_hand_cases.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w, p, ids = [x.strip() for x in line.split(";")]
            cases.append(([float(v) for v in w.split()], float(p), [int(v) for v in ids.split()]))
    return cases


@pytest.mark.parametrize("w,p,want", _read_hand_cases())
def test_topp_hand_worked_cases(w, p, want):
    sel, _, _, Z = orc.topp_from_weights(np.array(w), p)
    assert sel.tolist() == want
    assert Z == sum(w)
    # the same cases through the score interface: s = log2-exact weights are powers of two
    if all(v > 0 and math.log2(v).is_integer() for v in w):
        s = np.array([math.log(v) for v in w])
        r = orc.topp_select(s, p)
        assert sorted(r["idx"].tolist()) == sorted(want)


def brute_topp(scores, p):
    """O(N^2)-free but independent reference: python sort + python accumulation."""
    n = len(scores)
    mx = max(scores)
    w = [math.exp(s - mx) for s in scores]
    Z = math.fsum(w)
    order = sorted(range(n), key=lambda i: (-scores[i], i))
    if p >= 1.0:
        return order
    acc, out = 0.0, []
    for i in order:
        out.append(i)
        acc += w[i]
        if acc >= p * Z:
            break
    return out


@pytest.mark.parametrize("seed", range(6))
def test_topp_matches_python_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(5, 400))
    s = rng.standard_normal(n) * rng.uniform(0.2, 4.0)
    p = float(rng.uniform(0.3, 0.99))
    got = orc.topp_select(s, p)
    want = brute_topp(s.tolist(), p)
    # python's sequential accumulation and numpy's cumsum agree to rounding; allow the
    # one-token difference only if the boundary is within rounding of p*Z
    if got["idx"].tolist() != want:
        assert abs(len(want) - got["count"]) == 1
        assert abs(got["mass"] - p) < 1e-12
    else:
        assert got["count"] == len(want)


def test_topp_closed_form_all_equal():
    for n, p in [(8, 0.875), (8, 0.5), (64, 0.75), (1000, 0.9), (1000, 0.901), (7, 1.0), (1, 0.3)]:
        r = orc.topp_select(np.full(n, 1.2345), p)
        # n*p is computed exactly enough for these pairs (0.9*1000 = 900.0000000000001 > 900 though:
        # the definition is cum_k >= p*Z with cum_k = k exactly, so k = ceil(p*n) in floating point)
        assert r["count"] == math.ceil(p * n)
        assert r["idx"].tolist() == list(range(r["count"]))          # ties: lowest index first


def test_topp_closed_form_one_spike():
    # one token with gap g over N-1 equal others: alone iff 1/(1+(N-1)e^-g) >= p
    for n, g, p in [(1000, 12.0, 0.9), (1000, 5.0, 0.9), (50, 3.0, 0.25), (50, 3.0, 0.3)]:
        s = np.zeros(n)
        s[n // 3] = g
        r = orc.topp_select(s, p)
        alone = 1.0 / (1.0 + (n - 1) * math.exp(-g)) >= p
        assert (r["count"] == 1) == alone
        assert r["idx"][0] == n // 3
        if not alone:
            share0 = 1.0 / (1.0 + (n - 1) * math.exp(-g))
            each = math.exp(-g) / (1.0 + (n - 1) * math.exp(-g))
            k = 1 + math.ceil((p - share0) / each - 1e-9)
            assert abs(r["count"] - k) <= 1 and r["mass"] >= p


def test_topp_closed_form_geometric():
    # s_n = -n ln 2  ->  weights 2^-n (exact); mass of the first k = (1-2^-k)/(1-2^-N)
    n = 40
    s = -np.arange(n) * math.log(2.0)
    for p in (0.5, 0.75, 0.9, 0.99, 0.999999):
        r = orc.topp_select(s, p)
        k = next(k for k in range(1, n + 1) if (1 - 2.0 ** -k) / (1 - 2.0 ** -n) >= p)
        assert r["count"] == k and r["idx"].tolist() == list(range(k))


@pytest.mark.parametrize("seed", range(8))
def test_topp_invariants(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(50, 3000))
    s = rng.standard_normal(n) * rng.uniform(0.3, 3.0)
    s[rng.integers(0, n, 5)] += rng.uniform(3, 9)
    p1, p2 = sorted(rng.uniform(0.2, 0.995, 2).tolist())
    a, b = orc.topp_select(s, p1), orc.topp_select(s, p2)
    w = np.exp(s - s.max())
    Z = w.sum()
    for r, p in ((a, p1), (b, p2)):
        ids = r["idx"]
        assert w[ids].sum() / Z >= p - 1e-15                       # mass reaches p ...
        assert w[ids[:-1]].sum() / Z < p                            # ... and not without the last (smallest) token
        assert s[ids].min() == r["tau"] == s[ids[-1]]
        rest = np.setdiff1d(np.arange(n), ids)
        assert rest.size == 0 or s[rest].max() <= r["tau"]          # upward closed in score
        assert abs(r["mass"] - w[ids].sum() / Z) < 1e-12
    assert set(a["idx"].tolist()) <= set(b["idx"].tolist())         # monotone in p
    c = orc.topp_select(s + 3.75, p1)                               # shift invariance (3.75 keeps sums close)
    assert abs(c["count"] - a["count"]) <= 1
    perm = rng.permutation(n)                                       # permutation equivariance
    d = orc.topp_select(s[perm], p1)
    assert set(perm[d["idx"]].tolist()) == set(a["idx"].tolist())
    assert orc.topp_select(s, 1.0)["count"] == n


def test_topp_rejects_bad_p_and_empty():
    with pytest.raises(ValueError):
        orc.topp_select(np.zeros(4), 0.0)
    with pytest.raises(ValueError):
        orc.topp_select(np.zeros(4), float("nan"))
    with pytest.raises(ValueError):
        orc.topp_from_weights(np.zeros(0), 0.5)


# ---------------------------------------------------------------- attention (Sec. 3.2) and local rule (Sec. 4.2)
def test_local_set_cases():
    assert orc.local_set(0, 4, 8).tolist() == [0]
    assert orc.local_set(2, 4, 8).tolist() == [0, 1, 2]
    assert orc.local_set(11, 4, 8).tolist() == list(range(12))            # m+1 == sink+window: dense
    assert orc.local_set(12, 4, 8).tolist() == [0, 1, 2, 3] + list(range(5, 13))
    s = orc.local_set(1000, 4, 512)
    assert len(s) == 516 and s[-1] == 1000 and s[4] == 489 and 488 not in s
    assert orc.local_set(5, 0, 3).tolist() == [3, 4, 5]
    for m in range(0, 40):
        ids = orc.local_set(m, 3, 7)
        assert len(set(ids.tolist())) == len(ids) and ids.max() == m
        assert len(ids) == min(m + 1, 3 + 7) if m + 1 <= 10 else len(ids) == 10


def _tiny(seed, n=23, d=128):
    rng = np.random.default_rng(seed)
    return rand_bf16(rng, (d,)), rand_bf16(rng, (n, d)), rand_bf16(rng, (n, d)), rng


@pytest.mark.parametrize("seed", range(3))
def test_attend_matches_brute_force_two_ways(seed):
    qb, Kb, Vb, rng = _tiny(seed)
    ids = sorted(rng.choice(23, size=9, replace=False).tolist())
    q = orc.bf16_to_f64(qb).tolist()
    K = orc.bf16_to_f64(Kb).tolist()
    V = orc.bf16_to_f64(Vb).tolist()
    sc = 1.0 / math.sqrt(128)
    o, lse = orc.attend(qb, Kb, Vb, ids, sc)
    o1, l1 = brute_attention(q, K, V, ids, sc)
    o2, l2 = online_attention(q, K, V, ids, sc)
    assert np.allclose(o, o1, rtol=0, atol=1e-13) and np.allclose(o, o2, rtol=0, atol=1e-13)
    assert abs(lse - l1) < 1e-13 and abs(lse - l2) < 1e-13
    # order of the set does not matter; K and V are not interchangeable
    o3, _ = orc.attend(qb, Kb, Vb, ids[::-1], sc)
    assert np.allclose(o, o3, rtol=0, atol=1e-13)
    o4, _ = orc.attend(qb, Vb, Kb, ids, sc)
    assert not np.allclose(o, o4, atol=1e-3)


def test_attend_single_token_and_convex_hull():
    qb, Kb, Vb, rng = _tiny(7)
    o, _ = orc.attend(qb, Kb, Vb, [5], 0.3)
    assert np.array_equal(o, orc.bf16_to_f64(Vb[5]))
    ids = [1, 4, 9, 20]
    o, _ = orc.attend(qb, Kb, Vb, ids, 0.3)
    v = orc.bf16_to_f64(Vb[ids])
    assert np.all(o <= v.max(0) + 1e-15) and np.all(o >= v.min(0) - 1e-15)


def _tiny_layer(seed, ctx=(40, 17), Hq=4, Hkv=2, d=128, r=16):
    rng = np.random.default_rng(seed)
    T = sum(ctx)
    return dict(q_bits=rand_bf16(rng, (len(ctx), Hq, d)), K_bits=rand_bf16(rng, (Hkv, T, d)),
                V_bits=rand_bf16(rng, (Hkv, T, d)), kI_bits=rand_bf16(rng, (2, T, r)),
                qI_bits=rand_bf16(rng, (len(ctx), 2, r)),
                seq_start=[0, ctx[0]], ctx_len=list(ctx), n_q_heads=Hq, n_kv_heads=Hkv)


def test_decode_layer_p1_and_wide_window_reproduce_dense():
    """p = 1 and sink + window >= N must collapse every head to dense attention,
    which is checked against the pure-Python brute force (not against the oracle)."""
    L = _tiny_layer(5)
    r = orc.decode_layer(**L, ret_heads=[1, 2], sink=4, window=64, p_rows=np.ones(4))
    dn = orc.decode_layer(**L, ret_heads=[1, 2], sink=4, window=64, p_rows=np.ones(4), dense=True)
    assert np.array_equal(r["out"][:, [0, 3]], dn["out"][:, [0, 3]])          # local == dense, same op order
    assert np.allclose(r["out"], dn["out"], rtol=0, atol=1e-14)               # retrieval: same set, other order
    sc = 1.0 / math.sqrt(128)
    for b in range(2):
        t0, n = L["seq_start"][b], L["ctx_len"][b]
        for h in range(4):
            kvh = h // 2
            K = orc.bf16_to_f64(L["K_bits"][kvh, t0:t0 + n]).tolist()
            V = orc.bf16_to_f64(L["V_bits"][kvh, t0:t0 + n]).tolist()
            q = orc.bf16_to_f64(L["q_bits"][b, h]).tolist()
            o, lse = brute_attention(q, K, V, list(range(n)), sc)
            assert np.allclose(r["out"][b, h], o, rtol=0, atol=1e-13)
            assert abs(r["lse"][b, h] - lse) < 1e-13


def test_decode_layer_routes_heads_and_sequences():
    """Small p and a narrow window: each head must use ITS set, KV head and sequence."""
    L = _tiny_layer(6)
    r = orc.decode_layer(**L, ret_heads=[1, 2], sink=2, window=5, p_rows=np.array([0.5, 0.6, 0.7, 0.8]))
    sc = 1.0 / math.sqrt(128)
    row = 0
    for b in range(2):
        t0, n = L["seq_start"][b], L["ctx_len"][b]
        for h in range(4):
            kvh = h // 2
            K = orc.bf16_to_f64(L["K_bits"][kvh, t0:t0 + n]).tolist()
            V = orc.bf16_to_f64(L["V_bits"][kvh, t0:t0 + n]).tolist()
            q = orc.bf16_to_f64(L["q_bits"][b, h]).tolist()
            if h in (1, 2):
                j = (1, 2).index(h)
                qi = orc.bf16_to_f64(L["qI_bits"][b, j]).tolist()
                ki = orc.bf16_to_f64(L["kI_bits"][j, t0:t0 + n]).tolist()
                s = [sum(a * c for a, c in zip(qi, kn)) for kn in ki]
                ids = brute_topp(s, [0.5, 0.6, 0.7, 0.8][b * 2 + j])
                assert sorted(ids) == sorted(r["sel"][row]["idx"].tolist())
                row += 1
            else:
                ids = [i for i in range(n) if i < 2 or i >= max(2, n - 5)]
            o, _ = brute_attention(q, K, V, ids, sc)
            assert np.allclose(r["out"][b, h], o, rtol=0, atol=1e-13)


def test_prefill_rows_causal_and_dense_limit():
    rng = np.random.default_rng(9)
    T, Hq, Hkv, d, N0 = 6, 4, 2, 128, 30
    q = rand_bf16(rng, (T, Hq, d))
    K, V = rand_bf16(rng, (Hkv, N0 + T, d)), rand_bf16(rng, (Hkv, N0 + T, d))
    kI, qI = rand_bf16(rng, (1, N0 + T, 16)), rand_bf16(rng, (1, T, 16))
    rows = [(t, h) for t in range(T) for h in range(Hq)]
    common = dict(rows=rows, q_bits=q, K_bits=K, V_bits=V, chunk_start=N0, n_q_heads=Hq, n_kv_heads=Hkv)
    full = orc.prefill_rows(**common, kI_bits=kI, qI_bits=qI, ret_heads=[2], sink=4, window=64, p=1.0)
    dn = orc.dense_rows(**common)
    sc = 1.0 / math.sqrt(d)
    for a, b in zip(full, dn):
        assert np.allclose(a["out"], b["out"], rtol=0, atol=1e-14)
        m = N0 + a["t"]
        kvh = a["h"] // 2
        o, _ = brute_attention(orc.bf16_to_f64(q[a["t"], a["h"]]).tolist(),
                               orc.bf16_to_f64(K[kvh, :m + 1]).tolist(),
                               orc.bf16_to_f64(V[kvh, :m + 1]).tolist(), list(range(m + 1)), sc)
        assert np.allclose(a["out"], o, rtol=0, atol=1e-13)          # causal: never sees n > m
    sp = orc.prefill_rows(**common, kI_bits=kI, qI_bits=qI, ret_heads=[2], sink=1, window=3, p=0.5)
    for a in sp:
        m = N0 + a["t"]
        if a["h"] == 2:
            assert a["sel"]["idx"].max() <= m and a["sel"]["mass"] >= 0.5
            s = [sum(x * y for x, y in zip(orc.bf16_to_f64(qI[0, a["t"]]).tolist(), kn))
                 for kn in orc.bf16_to_f64(kI[0, :m + 1]).tolist()]
            assert sorted(brute_topp(s, 0.5)) == sorted(a["sel"]["idx"].tolist())


# =====================================================================================================
# widened rows: index-key build, static top-k, block-wise histogram selector, sparsity statistics
# =====================================================================================================
def test_build_index_keys_routes_kv_heads_and_is_exact():
    """Key side of the indexer equation (Sec. 3.2): the projection belongs to the QUERY head, the key row
    to the KV head that query head reads.  One-hot projections must copy key columns bit for bit, and a
    dense projection must agree with exact rational arithmetic."""
    rng = np.random.default_rng(5)
    T, Hq, Hkv, d, r = 9, 8, 2, 128, 16
    ret = [1, 6]                                         # KV heads 0 and 1
    k_pre = rand_bf16(rng, (T, Hkv, d))
    cols = rng.integers(0, d, size=(2, r))
    W = np.zeros((2, r, d), dtype=np.float32)
    for j in range(2):
        W[j, np.arange(r), cols[j]] = 1.0
    kI = orc.build_index_keys(W, k_pre, ret, Hq, Hkv)
    assert kI.shape == (2, T, r) and kI.dtype == np.uint16
    for j, kvh in enumerate((0, 1)):
        assert np.array_equal(kI[j], k_pre[:, kvh][:, cols[j]])
    # dense projection, one output against Fractions
    W = (rng.standard_normal((2, r, d)) / 8).astype(np.float32)
    kI = orc.build_index_keys(W, k_pre, ret, Hq, Hkv)
    j, n, i = 1, 4, 7
    exact = sum(Fraction(float(W[j, i, c])) * bf16_fraction(int(k_pre[n, 1, c])) for c in range(d))
    got = bf16_fraction(int(kI[j, n, i]))
    ulp = Fraction(2) ** (math.floor(math.log2(abs(float(exact)))) - 7)
    assert abs(got - exact) <= ulp / 2


def test_topk_hand_cases_with_ties():
    """Static top-k (Sec. 4.1 'Baselines'): the k best scores, ties to the lower index, never more than exist."""
    s = np.array([3.0, 1.0, 2.0, 5.0, 0.0, 4.0, 4.0, -1.0])
    want = {1: [3], 2: [3, 5], 3: [3, 5, 6], 4: [3, 5, 6, 0], 8: [3, 5, 6, 0, 2, 1, 4, 7], 100: [3, 5, 6, 0, 2, 1, 4, 7]}
    for k, ids in want.items():
        r = orc.topk_select(s, k)
        assert list(r["idx"]) == ids and r["count"] == len(ids)
        assert r["tau"] == s[ids[-1]]
    # masses on exactly representable weights: scores ln(8,4,2,1,1) -> top-2 holds 12/16
    r = orc.topk_select(np.log(np.array([8.0, 4.0, 2.0, 1.0, 1.0])), 2)
    assert list(r["idx"]) == [0, 1] and abs(r["mass"] - 0.75) < 1e-12
    with pytest.raises(ValueError):
        orc.topk_select(s, 0)
    with pytest.raises(ValueError):
        orc.topk_select(np.zeros(0), 3)


@pytest.mark.parametrize("seed", range(5))
def test_topk_invariants_and_relation_to_topp(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(50, 400))
    s = rng.standard_normal(n) * 2.0                      # continuous: no ties
    prev = set()
    for k in (1, 2, 7, n // 3, n - 1, n, n + 5):
        r = orc.topk_select(s, k)
        sel = set(r["idx"].tolist())
        assert len(sel) == min(k, n) == r["count"]
        rest = np.setdiff1d(np.arange(n), r["idx"])
        if rest.size:
            assert s[r["idx"]].min() > s[rest].max()      # nothing left out beats anything kept
        assert prev <= sel                                # monotone in k
        prev = sel
        # the same set by a library partition (independent of the oracle's sort)
        part = set(np.argpartition(-s, min(k, n) - 1)[:min(k, n)].tolist())
        assert part == sel
    # a top-k with the budget top-p arrived at is the top-p set
    tp = orc.topp_select(s, 0.9)
    tk = orc.topk_select(s, tp["count"])
    assert set(tk["idx"].tolist()) == set(tp["idx"].tolist())
    assert abs(tk["mass"] - tp["mass"]) < 1e-12 and tk["tau"] == tp["tau"]


def _read_block_cases():
    cases = []
    with open(os.path.join(GOLD, "block_topp_hand_cases.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            w, p, thr, blocks = [x.strip() for x in line.split(";")]
            cases.append(([float(x) for x in w.split()], float(p), int(thr), [int(x) for x in blocks.split()]))
    return cases


@pytest.mark.parametrize("w,p,thr,blocks", _read_block_cases())
def test_block_topp_hand_worked_cases(w, p, thr, blocks):
    """Sec. 3.4 selector on hand-worked inputs (tests/golden/block_topp_hand_cases.txt)."""
    ln2 = math.log(2.0)
    r = orc.block_topp_select(np.log(np.array(w)), p, block=2, n_bins=8, bin_lo=-0.5 * ln2, bin_width=ln2)
    assert r["threshold_bin"] == thr
    assert list(np.nonzero(r["block_mask"])[0]) == blocks
    want_idx = [n for b in blocks for n in (2 * b, 2 * b + 1) if n < len(w)]
    assert list(r["idx"]) == want_idx and r["count"] == len(want_idx)
    tot = sum(w)
    assert abs(r["mass"] - sum(w[n] for n in want_idx) / tot) < 1e-12


def test_block_topp_bins_clamp_and_block_pairs():
    # block maxima outside the binned range fall into the first / last bin
    s = np.array([-100.0, -101.0, 0.1, 0.0, 50.0, 49.0])
    r = orc.block_topp_select(s, 0.5, block=2, n_bins=16, bin_lo=-4.0, bin_width=0.5)
    assert list(r["bins"]) == [0, 8, 15]
    # the log-sum-exp pair of a block, against math.fsum
    assert abs(r["m_b"][1] - 0.1) < 1e-15
    assert abs(r["l_b"][1] - math.fsum([1.0, math.exp(-0.1)])) < 1e-15


@pytest.mark.parametrize("seed", range(6))
def test_block_topp_invariants(seed):
    """The selector's defining properties: the kept mass reaches p, dropping the threshold bin's blocks
    falls short of p, the mask is upward closed in the block maximum, and with one-token blocks and fine
    bins it contains the exact top-p set plus only tokens within one bin of the threshold."""
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(300, 2000))
    s = rng.standard_normal(n) * 1.5
    s[rng.integers(0, n, size=5)] += 6.0
    for p in (0.3, 0.8, 0.95):
        r = orc.block_topp_select(s, p, block=64)
        w = np.exp(s - s.max())
        Z = w.sum()
        assert r["mass"] >= p - 1e-12 and abs(w[r["idx"]].sum() / Z - r["mass"]) < 1e-12
        blk = np.arange(n) // 64
        below = r["bins"] > r["threshold_bin"]                        # strictly above the threshold bin
        assert w[np.isin(blk, np.nonzero(below)[0])].sum() / Z < p
        kept_max = r["m_b"][r["block_mask"]].min()
        if (~r["block_mask"]).any():
            assert r["m_b"][~r["block_mask"]].max() < kept_max + 0.25  # only a bin's width of overlap
            assert r["bins"][~r["block_mask"]].max() < r["bins"][r["block_mask"]].min()
        # one token per block, fine bins: the exact set is inside, the surplus hugs the threshold
        width = 1e-3
        r1 = orc.block_topp_select(s, p, block=1, n_bins=1 << 15, bin_lo=-16.0, bin_width=width)
        exact = orc.topp_select(s, p)
        extra = set(r1["idx"].tolist()) - set(exact["idx"].tolist())
        assert set(exact["idx"].tolist()) <= set(r1["idx"].tolist())
        assert all(exact["tau"] - width <= s[i] <= exact["tau"] for i in extra)
    assert orc.block_topp_select(s, 1.0)["count"] == n
    with pytest.raises(ValueError):
        orc.block_topp_select(s, 0.0)


def test_attention_mass_closed_forms_and_lse_identity():
    """True attention mass of a token set (Sec. 4.2, sparsity table): uniform logits give |S| / N, a
    two-level logit pattern gives its closed form, and for any set it equals exp(lse_S - lse_all) with
    the log-sum-exps of `attend` (an independently pinned function)."""
    rng = np.random.default_rng(3)
    N, d = 37, 128
    q = rand_bf16(rng, (d,))
    K0 = np.zeros((N, d), dtype=np.uint16)
    ids = np.array([1, 5, 6, 30])
    assert abs(orc.attention_mass(q, K0, ids, 0.125) - 4 / 37) < 1e-15
    # q = e_0, K[n, 0] = 2 for the set, 0 elsewhere: mass = k e^{2c} / (k e^{2c} + (N - k))
    q1 = np.zeros(d, dtype=np.uint16); q1[0] = 0x3F80
    K1 = np.zeros((N, d), dtype=np.uint16); K1[ids, 0] = 0x4000
    c = 0.3
    want = 4 * math.exp(2 * c) / (4 * math.exp(2 * c) + (N - 4))
    assert abs(orc.attention_mass(q1, K1, ids, c) - want) < 1e-14
    K = rand_bf16(rng, (N, d)); V = rand_bf16(rng, (N, d))
    _, lse_s = orc.attend(q, K, V, ids, 0.09)
    _, lse_a = orc.attend(q, K, V, np.arange(N), 0.09)
    assert abs(orc.attention_mass(q, K, ids, 0.09) - math.exp(lse_s - lse_a)) < 1e-13
    assert abs(orc.attention_mass(q, K, np.arange(N), 0.09) - 1.0) < 1e-15


def test_sparsity_stats_hand_case_and_limits():
    """Compute sparsity over query heads, memory sparsity over the per-KV-head unions (Sec. 3.2, last paragraph)."""
    att = [[0, 1, 2], [2, 3], [5], [5, 6, 7, 8]]                     # Hq = 4, Hkv = 2, N = 10
    r = orc.sparsity_stats(att, 10, 4, 2, ret_heads=[0, 3])
    assert abs(r["compute_sparsity"] - 0.75) < 1e-15                 # 1 - mean(3, 2, 1, 4) / 10
    assert r["union_sizes"] == [4, 4] and abs(r["memory_sparsity"] - 0.6) < 1e-15
    assert abs(r["active_tokens"] - 3.5) < 1e-15
    full = [list(range(10))] * 4
    r = orc.sparsity_stats(full, 10, 4, 2, ret_heads=[1])
    assert r["compute_sparsity"] == 0.0 and r["memory_sparsity"] == 0.0 and r["active_tokens"] == 10
    # disjoint sets of k tokens: the union of a group of G heads holds G k tokens
    att = [list(range(h * 3, h * 3 + 3)) for h in range(8)]
    r = orc.sparsity_stats(att, 48, 8, 2, ret_heads=[])
    assert abs(r["compute_sparsity"] - (1 - 3 / 48)) < 1e-15 and abs(r["memory_sparsity"] - (1 - 12 / 48)) < 1e-15
    # the union is never smaller than the mean: memory sparsity <= compute sparsity
    rng = np.random.default_rng(0)
    for _ in range(20):
        att = [rng.choice(64, size=int(rng.integers(1, 40)), replace=False).tolist() for _ in range(8)]
        r = orc.sparsity_stats(att, 64, 8, 4, ret_heads=[0, 2])
        assert r["memory_sparsity"] <= r["compute_sparsity"] + 1e-15


# ---------------------------------------------------------------- bounded cache of all-local KV heads
def test_ring_kv_heads_hand_cases():
    """Sec. 2.1 / Sec. 3.2 last paragraph: a KV head may drop remote tokens only if all its query heads are local."""
    assert orc.ring_kv_heads(32, 8, [0, 8, 16, 24]) == [1, 3, 5, 7]     # the benchmark layer: G = 4
    assert orc.ring_kv_heads(8, 2, [0, 5]) == []                        # both groups hold a retrieval head
    assert orc.ring_kv_heads(8, 8, [1, 3]) == [0, 2, 4, 5, 6, 7]        # G = 1
    assert orc.ring_kv_heads(8, 2, []) == [0, 1]


def test_ring_slots_keep_exactly_the_local_set():
    """Brute force, independent of ring_fill: replay the appends into a dict slot -> token and compare the
    resident tokens with the sink + window set of the newest position, for contexts below the sink count,
    below sink + window, equal to it and far above (several wraps)."""
    for sink, window in ((4, 16), (0, 5), (3, 1), (4, 96)):
        resident = {}
        for t in range(0, 3 * (sink + window) + 7):
            s = orc.ring_slot(t, sink, window)
            assert 0 <= s < sink + window
            assert (s == t) if t < sink else (sink <= s)
            resident[s] = t
            want = set(int(x) for x in orc.local_set(t, sink, window))    # the set a local head at position t sees
            assert set(resident.values()) == want, (sink, window, t)
            # valid rows are a prefix of the buffer
            assert sorted(resident) == list(range(min(t + 1, sink + window)))


def test_ring_fill_and_attention_match_the_full_cache():
    """The bounded cache holds the same (K, V) rows as the full cache restricted to the local set, so a local
    head's attention read from it equals its attention read from the full cache (same terms, other order)."""
    rng = np.random.default_rng(5)
    d, sink, window = 8, 4, 12
    for n in (1, 3, 4, 5, 16, 17, 40, 100):
        K = rng.integers(0x3c00, 0x4100, size=(n, d)).astype(np.uint16)    # bf16 patterns of moderate values
        V = rng.integers(0xbc00, 0xc100, size=(n, d)).astype(np.uint16)
        q = rng.integers(0x3c00, 0x4100, size=d).astype(np.uint16)
        rk, rv, rows = orc.ring_fill(K, V, n, sink, window)
        assert rows == min(n, sink + window)
        ids = orc.local_set(n - 1, sink, window)
        # row contents: token t sits where ring_slot says, bit for bit
        for t in ids:
            s = orc.ring_slot(int(t), sink, window)
            assert np.array_equal(rk[s], K[t]) and np.array_equal(rv[s], V[t])
        o_ring, lse_ring = orc.ring_local_attend(q, rk, rv, rows, 0.35)
        o_full, lse_full = orc.attend(q, K, V, ids, 0.35)
        assert np.allclose(o_ring, o_full, rtol=1e-13, atol=1e-13) and abs(lse_ring - lse_full) < 1e-12


# ---------------------------------------------------------------- paged cache
def test_paged_rows_by_construction_and_attention_is_layout_independent():
    """A pool is filled by explicit loops from a contiguous cache through a shuffled page table; the rows the
    oracle looks up must hold exactly the tokens asked for, and attention through the page table must equal
    attention on the contiguous cache bit for bit (same terms in the same order)."""
    rng = np.random.default_rng(9)
    d = 8
    for page_size, n in ((16, 100), (64, 64), (32, 1), (16, 257)):
        n_pages = -(-n // page_size)
        pool_pages = n_pages + 5
        table = rng.permutation(pool_pages)[:n_pages]
        K = rng.integers(0x3c00, 0x4100, size=(n, d)).astype(np.uint16)
        V = rng.integers(0xbc00, 0xc100, size=(n, d)).astype(np.uint16)
        Kp = np.zeros((pool_pages * page_size, d), dtype=np.uint16)
        Vp = np.zeros_like(Kp)
        for t in range(n):                                   # explicit placement, no oracle code
            page, off = divmod(t, page_size)
            Kp[int(table[page]) * page_size + off] = K[t]
            Vp[int(table[page]) * page_size + off] = V[t]
        ids = np.sort(rng.choice(n, size=max(1, n // 3), replace=False))
        rows = orc.paged_rows(table, page_size, ids)
        assert len(set(rows.tolist())) == len(ids)
        assert np.array_equal(Kp[rows], K[ids]) and np.array_equal(Vp[rows], V[ids])
        q = rng.integers(0x3c00, 0x4100, size=d).astype(np.uint16)
        o_p, l_p = orc.paged_attend(q, Kp, Vp, table, page_size, ids, 0.35)
        o_c, l_c = orc.attend(q, K, V, ids, 0.35)
        assert np.array_equal(o_p, o_c) and l_p == l_c
    # hand case: page size 4, table [2, 0]: token 5 -> page 0 of the pool ... row 0 * 4 + 1
    assert orc.paged_rows([2, 0], 4, [0, 3, 4, 5]).tolist() == [8, 11, 0, 1]


# =====================================================================================================
# the layer drivers' projection branch: which q_pre row meets which W^Q
# =====================================================================================================
def test_layer_drivers_project_the_retrieval_heads_own_pre_rope_query():
    """Query side of the indexer equation (Sec. 3.2): the index query of retrieval head h = ret_heads[j] is
    W^Q_j applied to q_pre of query head h -- not of head j, not of the KV head.  With one-hot projections the
    index query must copy chosen columns of q_pre[., ret_heads[j]] bit for bit (every head's q_pre is different,
    so any other pairing shows), in the decode driver and in the prefill driver; and the scores the drivers go
    on to select from must be the plain dot products of those copied columns with the index keys."""
    rng = np.random.default_rng(17)
    B, Hq, Hkv, d, r = 3, 8, 2, 128, 16
    ret = [1, 6, 7]                                      # none equal to its own position j in the list
    ctx = [5, 9, 7]
    start = [0, 5, 14]
    T_tot = sum(ctx)
    q_pre = rand_bf16(rng, (B, Hq, d))
    cols = np.stack([rng.choice(d, size=r, replace=False) for _ in ret])
    WQ = np.zeros((len(ret), r, d), dtype=np.float32)
    for j in range(len(ret)):
        WQ[j, np.arange(r), cols[j]] = 1.0
    kI = rand_bf16(rng, (len(ret), T_tot, r))
    common = dict(K_bits=rand_bf16(rng, (Hkv, T_tot, d)), V_bits=rand_bf16(rng, (Hkv, T_tot, d)), kI_bits=kI,
                  n_q_heads=Hq, n_kv_heads=Hkv, ret_heads=ret, sink=1, window=3)
    out = orc.decode_layer(q_bits=rand_bf16(rng, (B, Hq, d)), seq_start=start, ctx_len=ctx,
                           p_rows=np.full(B * len(ret), 0.7), WQ=WQ, q_pre_bits=q_pre, **common)
    for b in range(B):
        for j, h in enumerate(ret):
            assert np.array_equal(out["qI_bits"][b, j], q_pre[b, h][cols[j]]), (b, j, h)
            for other in range(Hq):
                if other != h:
                    assert not np.array_equal(out["qI_bits"][b, j], q_pre[b, other][cols[j]])
            # scores by exact rational arithmetic from the copied columns
            row = b * len(ret) + j
            n = 2
            exact = sum(bf16_fraction(int(q_pre[b, h][cols[j][i]])) * bf16_fraction(int(kI[j, start[b] + n, i]))
                        for i in range(r))
            assert abs(Fraction(float(out["scores"][row][n])) - exact) <= abs(exact) * Fraction(1, 2 ** 48)
    # prefill driver: q_pre is [T, Hq, d]; one sequence, queries at chunk_start + t
    T = 4
    q_pre_t = rand_bf16(rng, (T, Hq, d))
    rows = [(t, h) for t in range(T) for h in ret]
    res = orc.prefill_rows(rows=rows, q_bits=rand_bf16(rng, (T, Hq, d)), chunk_start=6, p=0.7, WQ=WQ,
                           q_pre_bits=q_pre_t, **common)
    for a in res:
        j = ret.index(a["h"])
        assert np.array_equal(a["qI_bits"], q_pre_t[a["t"], a["h"]][cols[j]]), (a["t"], a["h"])
        exact = sum(bf16_fraction(int(q_pre_t[a["t"], a["h"]][cols[j][i]])) * bf16_fraction(int(kI[j, 3, i]))
                    for i in range(r))
        assert abs(Fraction(float(a["scores"][3])) - exact) <= abs(exact) * Fraction(1, 2 ** 48)


# =====================================================================================================
# fp16 attention tensors
# =====================================================================================================
def half_fraction(bits: int) -> Fraction:
    """Exact rational value of one finite IEEE binary16 bit pattern, from its fields."""
    sign = -1 if bits & 0x8000 else 1
    e = (bits >> 10) & 0x1F
    man = bits & 0x3FF
    assert e != 31
    if e == 0:
        return Fraction(sign * man, 1 << 24)           # subnormal: man * 2^-10 * 2^-14
    return sign * Fraction(1024 + man, 1024) * (Fraction(2) ** (e - 15))


def test_fp16_widening_is_exact_for_every_finite_pattern():
    """Every finite binary16 pattern against its value spelled out from sign, exponent and mantissa fields."""
    bits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    vals = orc.fp16_to_f64(bits)
    for b in range(1 << 16):
        if (b >> 10) & 0x1F == 31:
            assert not np.isfinite(vals[b])
            continue
        assert Fraction(float(vals[b])) == half_fraction(b), hex(b)
    assert vals[0x3C00] == 1.0 and vals[0xC000] == -2.0 and vals[0x7BFF] == 65504.0 and vals[0x0001] == 2.0 ** -24
    assert np.signbit(vals[0x8000]) and vals[0x8000] == 0.0
    with pytest.raises(TypeError):
        orc.fp16_to_f64(np.zeros(3, dtype=np.int16))
    with pytest.raises(ValueError):
        orc.widen(np.zeros(3, dtype=np.uint16), "fp8")


def test_attend_and_layer_drivers_read_fp16_tensors_as_fp16():
    """The same bit patterns mean different numbers in the two formats: with kv_dtype = "fp16" the attention must
    be the brute-force attention over the binary16 VALUES (q, K and V alike), in attend and through the decode
    and prefill drivers; index keys stay bf16."""
    rng = np.random.default_rng(23)
    N, d, Hq, Hkv = 40, 128, 4, 2
    f16 = lambda shape: rng.standard_normal(shape).astype(np.float16).view(np.uint16)
    q, K, V = f16((1, Hq, d)), f16((Hkv, N, d)), f16((Hkv, N, d))
    val = lambda bits: [[float(half_fraction(int(x))) for x in row] for row in np.atleast_2d(bits)]
    ids = [3, 7, 8, 20, 39]
    o, lse = orc.attend(q[0, 1], K[0], V[0], ids, 0.11, kv_dtype="fp16")
    bo, bl = brute_attention(val(q[0, 1])[0], val(K[0]), val(V[0]), ids, 0.11)
    assert np.allclose(o, bo, rtol=1e-12, atol=1e-14) and abs(lse - bl) < 1e-12
    o_bf, _ = orc.attend(q[0, 1], K[0], V[0], ids, 0.11)          # the same bits read as bf16: other numbers
    assert not np.allclose(o, o_bf, atol=1e-3)
    kI = rand_bf16(rng, (1, N, 16))
    qI = rand_bf16(rng, (1, 1, 16))
    common = dict(K_bits=K, V_bits=V, kI_bits=kI, n_q_heads=Hq, n_kv_heads=Hkv, ret_heads=[2], sink=2, window=5,
                  kv_dtype="fp16")
    dec = orc.decode_layer(q_bits=q, seq_start=[0], ctx_len=[N], p_rows=np.array([0.6]), qI_bits=qI, **common)
    for h in range(Hq):
        ids_h = dec["sel"][0]["idx"].tolist() if h == 2 else orc.local_set(N - 1, 2, 5).tolist()
        bo, _ = brute_attention(val(q[0, h])[0], val(K[h // 2]), val(V[h // 2]), ids_h, 1.0 / math.sqrt(d))
        assert np.allclose(dec["out"][0, h], bo, rtol=1e-12, atol=1e-14), h
    rows = orc.prefill_rows(rows=[(0, 0), (0, 2)], q_bits=q, chunk_start=N - 1, p=0.6, qI_bits=qI.reshape(1, 1, 16), **common)
    assert np.allclose(rows[0]["out"], dec["out"][0, 0], rtol=1e-12) and np.allclose(rows[1]["out"], dec["out"][0, 2], rtol=1e-12)
    dr = orc.dense_rows(rows=[(0, 3)], q_bits=q, K_bits=K, V_bits=V, chunk_start=N - 1, n_q_heads=Hq, n_kv_heads=Hkv,
                        kv_dtype="fp16")
    bo, _ = brute_attention(val(q[0, 3])[0], val(K[1]), val(V[1]), list(range(N)), 1.0 / math.sqrt(d))
    assert np.allclose(dr[0]["out"], bo, rtol=1e-12, atol=1e-14)
