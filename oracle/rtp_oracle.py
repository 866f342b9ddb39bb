"""CPU oracle for the RTPurbo sparse-attention hot path.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the smoke
check and the benchmark's CPU-baseline leg may import it.  It shares no code
with the HIP library and never calls it.

Everything here is plain numpy in float64, written from the definitions in the
paper (Section 3.2 "Adaptive Sparse Attention Mechanism" and Section 4.2
"Sparsity Analysis"), one function per step, with no blocking, fusion or
re-ordering.  bf16 tensors travel as uint16 bit patterns and are widened
exactly to float64 before any arithmetic.

Steps (one attention layer, query position m of a sequence, head h):

  retrieval head  (h in H_ret)
    index_project   qI = bf16( W^Q_h q^pre_{m,h} )                 Sec. 3.2, indexer equation
    index_score     s_n = scale * <qI, kI_{n,h}>  for every candidate n        (same equation)
    topp_select     S = Top-P(s, p): the shortest prefix of the candidates in
                    descending score order whose softmax mass reaches p        Sec. 3.2, sparse-attention equation
    attend          O = sum_{n in S} softmax_S(q.k_n / sqrt(d_h)) v_n          (same equation)
  local head      (h in H_loc)
    local_set       sink tokens + sliding window                               Sec. 3.2 first sentence; Sec. 4.2
    attend          softmax attention over that set
  dense reference   attend over every causal candidate                         Sec. 3.2 (prefill rule)

Readings taken where the paper is silent:
  * the indexer softmax has scale 1 unless the caller passes another scale;
  * ties in score are ordered by ascending token index;
  * "reaches p" means cumulative mass >= p * Z; p >= 1 keeps every candidate;
    at least one token is always kept;
  * the window of a local head is the `window` most recent positions,
    the query's own position included; sinks are positions 0..sink-1;
  * GQA: query head h reads KV head h // (Hq // Hkv);
  * decode candidates are all ctx_len cached tokens; prefill candidates are
    the causal ones, n <= m.

Widened rows (each pinned the same way, see the end of this file):
    build_index_keys   kI = bf16( W^K_h k^pre_{n,kv(h)} ), the key side of the indexer equation
    topk_select        the static top-k rule the paper ablates against (Sec. 4.1 "Baselines")
    block_topp_select  the block-wise histogram selector of Sec. 3.4, with the readings stated there
    attention_mass     true attention probability captured by a token set        Sec. 4.2, sparsity table
    sparsity_stats     compute / memory sparsity, active tokens                  Sec. 3.2 (last paragraph), Sec. 4.2
    ring_kv_heads, ring_slot, ring_append, ring_fill, ring_local_attend
                       the KV cache of a KV head whose query heads are all local keeps only the sink
                       tokens and the last `window` tokens (Sec. 2.1: the full cache is retained for
                       retrieval heads only; Sec. 3.2 last paragraph: memory is counted per KV head)
    paged_rows, paged_attend
                       the same sparse-attention equation with the full cache of the retrieval heads held in
                       fixed-size pages (a storage layout, not in the paper: token t of a sequence lives in row
                       page_table[t // page_size] * page_size + t % page_size of a pool shared by all sequences)

Parity status: every function below is pinned by tests/test_oracle_pins.py
(brute-force dense attention, hand-worked exact-binary top-p cases, closed
forms, invariants).  Agreement with the paper's real-model statistics
(the top-p token counts of its tables) is "parity unpinned": they cannot be
re-derived without the model's activations.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "bf16_to_f64", "fp16_to_f64", "widen", "f64_to_bf16_bits", "index_project", "index_score",
    "topp_from_weights", "topp_select", "attend", "local_set", "kv_head_of",
    "decode_layer", "prefill_rows", "dense_rows",
    "build_index_keys", "topk_select", "block_topp_select", "attention_mass", "sparsity_stats",
    "ring_kv_heads", "ring_slot", "ring_append", "ring_fill", "ring_local_attend",
    "paged_rows", "paged_attend",
]


# --------------------------------------------------------------------------
# number formats
# --------------------------------------------------------------------------
def bf16_to_f64(bits) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float64; exact."""
    b = np.asarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("bf16 tensors are passed as uint16 bit patterns")
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def fp16_to_f64(bits) -> np.ndarray:
    """Widen IEEE binary16 bit patterns (uint16) to float64; exact (subnormals, infinities included).

    The paper's own decode kernel reads its K and V as 16-bit halves (Sec. 3.4, "Bandwidth-optimized sparse
    decoding"); the library accepts either 16-bit format for q, K and V.
    """
    b = np.asarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("fp16 tensors are passed as uint16 bit patterns")
    return b.view(np.float16).astype(np.float64)


def widen(bits, kv_dtype: str = "bf16") -> np.ndarray:
    """Bit patterns of the attention tensors (q, K, V) to float64, by their element type."""
    if kv_dtype == "bf16":
        return bf16_to_f64(bits)
    if kv_dtype == "fp16":
        return fp16_to_f64(bits)
    raise ValueError(f"unknown element type {kv_dtype!r}")


def f64_to_bf16_bits(x) -> np.ndarray:
    """Round float64 to bf16, round-to-nearest-even, in ONE rounding step.

    (Going through float32 first would round twice.)  Only normal-range
    values are supported, which is all the indexer produces.
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(x.shape, dtype=np.float64)
    nz = x != 0.0
    _, e = np.frexp(x[nz])                    # |x| = f * 2**e, f in [0.5, 1)
    ulp = np.ldexp(1.0, e - 8)                # bf16 keeps 8 significant bits
    out[nz] = np.rint(x[nz] / ulp) * ulp      # rint = half-to-even; the scaling is exact
    f32 = out.astype(np.float32)              # exact: 8 significant bits fit
    if not np.all(f32.astype(np.float64) == out):
        raise OverflowError("value outside the bf16 normal range")
    bits32 = f32.view(np.uint32)
    assert np.all((bits32 & np.uint32(0xFFFF)) == 0)
    return (bits32 >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------
# indexer  (Sec. 3.2, indexer equation)
# --------------------------------------------------------------------------
def index_project(W, x_pre_bits) -> np.ndarray:
    """qI = bf16( W x ), W float32 [r, d], x bf16 [..., d]  ->  uint16 [..., r].

    The sum over d runs in float64 (every product bf16*fp32 is exact there)
    and is rounded to bf16 once.
    """
    W64 = np.asarray(W, dtype=np.float32).astype(np.float64)
    x64 = bf16_to_f64(x_pre_bits)
    return f64_to_bf16_bits(x64 @ W64.T)


def index_score(qI_bits, kI_bits, index_scale: float = 1.0) -> np.ndarray:
    """s_n = index_scale * sum_i qI[i] * kI[n, i];  qI [r], kI [N, r] -> float64 [N]."""
    q = bf16_to_f64(qI_bits)
    k = bf16_to_f64(kI_bits)
    return float(index_scale) * (k @ q)


# --------------------------------------------------------------------------
# top-p  (Sec. 3.2: S = Top-P(s, p); Sec. 3.4: threshold where the cumulative softmax mass reaches p)
# --------------------------------------------------------------------------
def topp_from_weights(w, p: float, key=None):
    """Shortest descending prefix whose weight reaches p * sum(w).

    w   : non-negative weights, one per candidate.
    key : what "descending" refers to (defaults to w); ties go to the lower
          candidate index.
    Returns (selected indices in rank order, rank order of all candidates,
             cumulative weights in rank order, Z).
    """
    w = np.asarray(w, dtype=np.float64)
    n = w.shape[0]
    if n == 0:
        raise ValueError("top-p needs at least one candidate")
    if not (p > 0.0):
        raise ValueError("p must be positive")
    key = w if key is None else np.asarray(key, dtype=np.float64)
    order = np.lexsort((np.arange(n), -key))      # key descending, index ascending
    cum = np.cumsum(w[order])
    Z = float(np.sum(w))
    if p >= 1.0:
        k = n
    else:
        reached = np.nonzero(cum >= p * Z)[0]
        k = int(reached[0]) + 1 if reached.size else n
    return order[:k], order, cum, Z


def topp_select(scores, p: float) -> dict:
    """Top-P over the softmax of `scores` (float64 [N]).

    Returns dict(idx=selected token ids in rank order, count, tau=score of the
    last selected token, mass=selected softmax mass, Z=sum exp(s - max)).
    """
    s = np.asarray(scores, dtype=np.float64)
    w = np.exp(s - np.max(s))
    sel, order, cum, Z = topp_from_weights(w, p, key=s)
    k = sel.shape[0]
    return dict(idx=sel, count=k, tau=float(s[sel[-1]]), mass=float(cum[k - 1] / Z),
                Z=Z, smax=float(np.max(s)))


# --------------------------------------------------------------------------
# attention over a token set  (Sec. 3.2, sparse-attention equation)
# --------------------------------------------------------------------------
def attend(q_bits, K_bits, V_bits, token_ids, softmax_scale: float, kv_dtype: str = "bf16"):
    """O = sum_{n in S} softmax_S(scale * q.k_n) v_n  and its log-sum-exp.

    q [d] bit patterns; K, V [N, d] bit patterns (one KV head of one sequence), all of element type
    kv_dtype ("bf16" or "fp16"); token_ids: the set S.  Returns (O float64 [d], lse float64).
    """
    ids = np.asarray(token_ids, dtype=np.int64)
    q = widen(q_bits, kv_dtype)
    k = widen(K_bits[ids], kv_dtype)
    v = widen(V_bits[ids], kv_dtype)
    logits = float(softmax_scale) * (k @ q)
    mx = np.max(logits)
    a = np.exp(logits - mx)
    denom = np.sum(a)
    return (a @ v) / denom, float(mx + np.log(denom))


def local_set(m: int, sink: int, window: int) -> np.ndarray:
    """Tokens a local head at query position m may see: sinks + sliding window."""
    lo = max(sink, m - window + 1)
    head = np.arange(0, min(sink, m + 1), dtype=np.int64)
    tail = np.arange(lo, m + 1, dtype=np.int64)
    return np.concatenate([head, tail])


def kv_head_of(h: int, n_q_heads: int, n_kv_heads: int) -> int:
    return h // (n_q_heads // n_kv_heads)


# --------------------------------------------------------------------------
# layer drivers (loops over sequences / heads / query rows, nothing else)
# --------------------------------------------------------------------------
def _scale(softmax_scale, d):
    return (1.0 / np.sqrt(float(d))) if not softmax_scale else float(softmax_scale)


def decode_layer(*, q_bits, K_bits, V_bits, kI_bits, seq_start, ctx_len,
                 n_q_heads, n_kv_heads, ret_heads, sink, window, p_rows,
                 qI_bits=None, WQ=None, q_pre_bits=None,
                 softmax_scale=0.0, index_scale=0.0, dense=False, kv_dtype="bf16"):
    """One decode step of one layer.

    q_bits [B, Hq, d]; K_bits, V_bits [Hkv, T_tot, d]; kI_bits [n_ret, T_tot, r];
    seq_start/ctx_len [B]; p_rows [B * n_ret] (row = b * n_ret + j).
    Either qI_bits [B, n_ret, r] or (WQ [n_ret, r, d], q_pre_bits [B, Hq, d]).
    Returns dict(out float64 [B, Hq, d], lse [B, Hq], scores (list per row),
    sel (list of dicts per row), qI_bits).  With dense=True every head attends
    to the whole context (the comparison system) and no selection happens.
    """
    B, Hq, d = q_bits.shape
    ret_heads = list(ret_heads)
    n_ret = len(ret_heads)
    sc = _scale(softmax_scale, d)
    isc = 1.0 if not index_scale else float(index_scale)
    out = np.zeros((B, Hq, d))
    lse = np.zeros((B, Hq))
    scores, sels = [], []
    if qI_bits is None and not dense:
        qI_bits = np.stack([np.stack([index_project(WQ[j], q_pre_bits[b, h])
                                      for j, h in enumerate(ret_heads)]) for b in range(B)])
    for b in range(B):
        t0, n = int(seq_start[b]), int(ctx_len[b])
        m = n - 1
        for h in range(Hq):
            kvh = kv_head_of(h, Hq, n_kv_heads)
            Kb, Vb = K_bits[kvh, t0:t0 + n], V_bits[kvh, t0:t0 + n]
            if dense:
                ids = np.arange(n)
            elif h in ret_heads:
                j = ret_heads.index(h)
                s = index_score(qI_bits[b, j], kI_bits[j, t0:t0 + n], isc)
                sel = topp_select(s, float(p_rows[b * n_ret + j]))
                scores.append(s)
                sels.append(sel)
                ids = sel["idx"]
            else:
                ids = local_set(m, sink, window)
            out[b, h], lse[b, h] = attend(q_bits[b, h], Kb, Vb, ids, sc, kv_dtype)
    return dict(out=out, lse=lse, scores=scores, sel=sels, qI_bits=qI_bits)


def prefill_rows(*, rows, q_bits, K_bits, V_bits, kI_bits, chunk_start,
                 n_q_heads, n_kv_heads, ret_heads, sink, window, p,
                 qI_bits=None, WQ=None, q_pre_bits=None,
                 softmax_scale=0.0, index_scale=0.0, kv_dtype="bf16"):
    """Selected (t, h) rows of one causal prefill chunk of ONE sequence.

    q_bits [T, Hq, d] holds the chunk's queries, query t sits at position
    m = chunk_start + t; K_bits, V_bits [Hkv, >= m + 1, d]; kI_bits [n_ret, >=, r];
    qI_bits [n_ret, T, r] or (WQ, q_pre_bits [T, Hq, d]).
    Retrieval heads: causal candidates n <= m, Top-P, attention over the set.
    Local heads: sink + window.  Returns a list of dicts, one per row.
    """
    T, Hq, d = q_bits.shape
    ret_heads = list(ret_heads)
    sc = _scale(softmax_scale, d)
    isc = 1.0 if not index_scale else float(index_scale)
    res = []
    for (t, h) in rows:
        m = int(chunk_start) + int(t)
        kvh = kv_head_of(h, Hq, n_kv_heads)
        Kb, Vb = K_bits[kvh, :m + 1], V_bits[kvh, :m + 1]
        r = dict(t=t, h=h, m=m)
        if h in ret_heads:
            j = ret_heads.index(h)
            qi = qI_bits[j, t] if qI_bits is not None else index_project(WQ[j], q_pre_bits[t, h])
            s = index_score(qi, kI_bits[j, :m + 1], isc)
            sel = topp_select(s, p)
            ids = sel["idx"]
            r.update(scores=s, sel=sel, qI_bits=qi)
        else:
            ids = local_set(m, sink, window)
        r["out"], r["lse"] = attend(q_bits[t, h], Kb, Vb, ids, sc, kv_dtype)
        res.append(r)
    return res


def dense_rows(*, rows, q_bits, K_bits, V_bits, chunk_start, n_q_heads, n_kv_heads,
               softmax_scale=0.0, kv_dtype="bf16"):
    """Dense causal attention for selected (t, h) rows of a prefill chunk."""
    T, Hq, d = q_bits.shape
    sc = _scale(softmax_scale, d)
    res = []
    for (t, h) in rows:
        m = int(chunk_start) + int(t)
        kvh = kv_head_of(h, Hq, n_kv_heads)
        o, l = attend(q_bits[t, h], K_bits[kvh, :m + 1], V_bits[kvh, :m + 1], np.arange(m + 1), sc, kv_dtype)
        res.append(dict(t=t, h=h, m=m, out=o, lse=l))
    return res


# --------------------------------------------------------------------------
# index keys  (Sec. 3.2, indexer equation, key side)
# --------------------------------------------------------------------------
def build_index_keys(WK, k_pre_bits, ret_heads, n_q_heads: int, n_kv_heads: int) -> np.ndarray:
    """kI[j, n, :] = bf16( W^K_{h_j} k^pre_{n, kv(h_j)} ) for every retrieval query head h_j.

    WK float32 [n_ret, r, d]; k_pre_bits bf16 [T, Hkv, d] (keys BEFORE the rotary
    embedding).  The projection is indexed by the QUERY head, the key row it is
    applied to belongs to the KV head that query head reads.  -> uint16 [n_ret, T, r].
    """
    out = []
    for j, h in enumerate(ret_heads):
        kvh = kv_head_of(int(h), n_q_heads, n_kv_heads)
        out.append(index_project(WK[j], k_pre_bits[:, kvh]))
    return np.stack(out)


# --------------------------------------------------------------------------
# static top-k  (Sec. 4.1 "Baselines": the fixed-budget comparison, k = 4096 there)
# --------------------------------------------------------------------------
def topk_select(scores, k: int) -> dict:
    """The k highest-scoring candidates (all of them if there are fewer); ties go to the lower index.

    Returns dict(idx in rank order, count, tau = score of the last selected token,
    mass = selected softmax mass of the scores).
    """
    s = np.asarray(scores, dtype=np.float64)
    n = s.shape[0]
    if n == 0:
        raise ValueError("top-k needs at least one candidate")
    if k < 1:
        raise ValueError("k must be at least 1")
    order = np.lexsort((np.arange(n), -s))
    kk = min(int(k), n)
    sel = order[:kk]
    w = np.exp(s - np.max(s))
    return dict(idx=sel, count=kk, tau=float(s[sel[-1]]), mass=float(np.sum(w[sel]) / np.sum(w)))


# --------------------------------------------------------------------------
# block-wise top-p  (Sec. 3.4 "Sort-free top-p via histogram")
# --------------------------------------------------------------------------
def block_topp_select(scores, p: float, block: int = 64, n_bins: int = 256,
                      bin_lo: float = -32.0, bin_width: float = 0.25) -> dict:
    """Block-level top-p in the order the section gives its steps.

    1. cut the candidates into blocks of `block` consecutive tokens; block b is
       reduced to its log-sum-exp pair  m_b = max s,  l_b = sum exp(s - m_b);
    2. every block deposits its mass  l_b * exp(m_b)  into the histogram bin its
       maximum m_b falls into;
    3. the histogram is scanned from the highest bin down; the threshold bin is
       the first one at which the cumulative mass reaches p * (total mass);
    4. the mask keeps every block whose bin is at or above the threshold bin.

    Readings (the section names neither the bin mapping nor the common scale of
    the deposits): bins are uniform in score, bin(m) = floor((m - bin_lo) /
    bin_width) clamped to [0, n_bins - 1]; masses are compared on one common
    scale (here exp(. - max score), any common scale decides alike); p >= 1
    keeps every block; whole blocks are kept, so the kept mass overshoots p by
    up to the mass of the threshold bin.

    Returns dict(block_mask bool [N_b], bins int [N_b], threshold_bin, idx =
    token ids of the kept blocks ascending, count, mass = kept mass / total,
    m_b, l_b).
    """
    s = np.asarray(scores, dtype=np.float64)
    n = s.shape[0]
    if n == 0:
        raise ValueError("needs at least one candidate")
    if not (p > 0.0):
        raise ValueError("p must be positive")
    nb = (n + block - 1) // block
    m_b = np.empty(nb)
    l_b = np.empty(nb)
    for b in range(nb):
        sb = s[b * block:(b + 1) * block]
        m_b[b] = np.max(sb)
        l_b[b] = np.sum(np.exp(sb - m_b[b]))
    bins = np.clip(np.floor((m_b - bin_lo) / bin_width), 0, n_bins - 1).astype(np.int64)
    ref = np.max(m_b)
    mass_b = l_b * np.exp(m_b - ref)
    hist = np.zeros(n_bins)
    for b in range(nb):
        hist[bins[b]] += mass_b[b]
    total = float(np.sum(mass_b))
    if p >= 1.0:
        thr = 0
    else:
        cum = 0.0
        thr = 0
        for k in range(n_bins - 1, -1, -1):
            cum += hist[k]
            if cum >= p * total:
                thr = k
                break
    mask = bins >= thr
    idx = np.concatenate([np.arange(b * block, min((b + 1) * block, n)) for b in range(nb) if mask[b]])
    return dict(block_mask=mask, bins=bins, threshold_bin=int(thr), idx=idx.astype(np.int64), count=int(idx.shape[0]),
                mass=float(np.sum(mass_b[mask]) / total), m_b=m_b, l_b=l_b)


# --------------------------------------------------------------------------
# sparsity statistics  (Sec. 3.2 last paragraph; Sec. 4.2 "Sparsity Analysis" and its table)
# --------------------------------------------------------------------------
def attention_mass(q_bits, K_bits, token_ids, softmax_scale: float) -> float:
    """Probability the FULL softmax attention of q over all rows of K puts on the set `token_ids`."""
    q = bf16_to_f64(q_bits)
    logits = float(softmax_scale) * (bf16_to_f64(K_bits) @ q)
    a = np.exp(logits - np.max(logits))
    return float(np.sum(a[np.asarray(token_ids, dtype=np.int64)]) / np.sum(a))


def sparsity_stats(attended, n_ctx: int, n_q_heads: int, n_kv_heads: int, ret_heads) -> dict:
    """Sparsity of one decode step of one sequence.

    attended: list over query heads of the token-id sets they attend to.
    compute sparsity = 1 - (mean over query heads of the attended count) / n_ctx;
    memory sparsity  = 1 - (mean over KV heads of the size of the UNION of the
    sets of the query heads mapped to that KV head) / n_ctx;
    active tokens    = mean attended count over the retrieval heads.
    """
    sizes = [len(set(int(x) for x in a)) for a in attended]
    compute = 1.0 - float(np.mean(sizes)) / n_ctx
    unions = []
    for g in range(n_kv_heads):
        u = set()
        for h in range(n_q_heads):
            if kv_head_of(h, n_q_heads, n_kv_heads) == g:
                u |= set(int(x) for x in attended[h])
        unions.append(len(u))
    memory = 1.0 - float(np.mean(unions)) / n_ctx
    ret = list(ret_heads)
    active = float(np.mean([sizes[h] for h in ret])) if ret else 0.0
    return dict(compute_sparsity=compute, memory_sparsity=memory, active_tokens=active, union_sizes=unions)


# ---- bounded cache of the all-local KV heads --------------------------------------------------------
# Sec. 2.1 keeps the full KV cache for retrieval heads only; the other heads may drop remote tokens.
# Under GQA the cache is per KV head (Sec. 3.2, last paragraph), so a KV head can drop them only when
# every query head mapped to it is local.  Such a head then needs `sink + window` rows per sequence.
# Reading (the paper does not give a layout): row i < sink holds token i; token t >= sink lives in row
# sink + (t - sink) mod window, overwriting the token that left the window when t arrived.

def ring_kv_heads(n_q_heads: int, n_kv_heads: int, ret_heads) -> list:
    """KV heads none of whose query heads is a retrieval head, ascending."""
    ret = set(int(h) for h in ret_heads)
    g = n_q_heads // n_kv_heads
    return [kv for kv in range(n_kv_heads) if not any(h in ret for h in range(kv * g, (kv + 1) * g))]


def ring_slot(t: int, sink: int, window: int) -> int:
    """Row of the bounded cache that token position t occupies."""
    return int(t) if t < sink else sink + (int(t) - sink) % window


def ring_append(ring_K_bits, ring_V_bits, k_row_bits, v_row_bits, t: int, sink: int, window: int) -> None:
    """Stores token t's K and V rows (uint16 [d]) into the bounded cache (uint16 [sink + window, d]), in place."""
    s = ring_slot(t, sink, window)
    ring_K_bits[s] = k_row_bits
    ring_V_bits[s] = v_row_bits


def ring_fill(K_bits, V_bits, n: int, sink: int, window: int):
    """The bounded cache after tokens 0..n-1 of one KV head (rows of K_bits, V_bits) have been appended
    in order, written out token by token.  Returns (ring_K, ring_V, rows): rows = how many rows hold a token."""
    d = K_bits.shape[1]
    rk = np.zeros((sink + window, d), dtype=np.uint16)
    rv = np.zeros((sink + window, d), dtype=np.uint16)
    for t in range(int(n)):
        ring_append(rk, rv, K_bits[t], V_bits[t], t, sink, window)
    return rk, rv, min(int(n), sink + window)


def ring_local_attend(q_bits, ring_K_bits, ring_V_bits, rows: int, softmax_scale: float, kv_dtype: str = "bf16"):
    """A local head's attention at decode time read from the bounded cache: softmax attention over its
    first `rows` rows (a softmax over a set does not depend on the order of its members)."""
    return attend(q_bits, ring_K_bits, ring_V_bits, np.arange(int(rows)), softmax_scale, kv_dtype)


# ---- paged cache ------------------------------------------------------------------------------------
def paged_rows(page_table, page_size: int, token_ids) -> np.ndarray:
    """Pool rows of the given token positions of ONE sequence: page_table[i] is the pool page that holds
    tokens i * page_size .. (i + 1) * page_size - 1."""
    t = np.asarray(token_ids, dtype=np.int64)
    pt = np.asarray(page_table, dtype=np.int64)
    return pt[t // int(page_size)] * int(page_size) + t % int(page_size)


def paged_attend(q_bits, K_pool_bits, V_pool_bits, page_table, page_size: int, token_ids, softmax_scale: float,
                 kv_dtype: str = "bf16"):
    """The sparse-attention equation over the set `token_ids` of a sequence whose K/V rows live in a paged
    pool (uint16 [pool_rows, d], one KV head)."""
    return attend(q_bits, K_pool_bits, V_pool_bits, paged_rows(page_table, page_size, token_ids), softmax_scale, kv_dtype)
