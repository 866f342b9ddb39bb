"""Seeded synthetic inputs for the sparse-attention hot path.

This module only draws random tensors and lays them out; it holds none of the
method's arithmetic and is the one piece of code that both the HIP parity
tests and the CPU oracle's callers use.  Tensors are produced with torch on
the requested device ("cpu" here, "cuda" on the GPU machine) from a seeded
torch.Generator, in fp32, and rounded once to bf16.

The recipes stand in for the long-context prompts and model activations the
paper evaluates on (Sec. 4): shapes follow its 32K-1M settings, and the
indexer-score laws are shaped so that top-p keeps between a few dozen and
tens of thousands of tokens, the range its per-head token-count tables show.
Planted tokens get index keys aligned with the index query, which makes the
indexer's softmax mass peaky; everything else is Gaussian background.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch

HEAD_DIM = 128
INDEX_DIM = 16


@dataclass
class Layer:
    n_q_heads: int
    n_kv_heads: int
    ret_heads: List[int]
    sink: int
    window: int
    head_dim: int = HEAD_DIM
    index_dim: int = INDEX_DIM
    kv_dtype: str = "bf16"          # element type of q, K, V and the output: "bf16" or "fp16"
    softmax_scale: float = 0.0      # 0 = the paper's 1/sqrt(head_dim)
    index_scale: float = 0.0        # 0 = 1 (the indexer equation has no scale)

    @property
    def n_ret(self) -> int:
        return len(self.ret_heads)


@dataclass
class DecodeWorkload:
    name: str
    layer: Layer
    ctx_len: List[int]
    seq_start: List[int]
    q: torch.Tensor                 # bf16 [B, Hq, D]      post-RoPE queries
    K: torch.Tensor                 # bf16 [Hkv, T_tot, D]
    V: torch.Tensor                 # bf16 [Hkv, T_tot, D]
    kI: torch.Tensor                # bf16 [n_ret, T_tot, r]
    p_rows: torch.Tensor            # fp32 [B * n_ret]
    qI: Optional[torch.Tensor] = None      # bf16 [B, n_ret, r] (given directly) or None
    WQ: Optional[torch.Tensor] = None      # fp32 [n_ret, r, D]
    q_pre: Optional[torch.Tensor] = None   # bf16 [B, Hq, D]    pre-RoPE queries
    planted: dict = field(default_factory=dict)   # (b, j) -> LongTensor of planted positions

    @property
    def B(self) -> int:
        return len(self.ctx_len)

    @property
    def T_tot(self) -> int:
        return int(self.K.shape[1])

    def to(self, device) -> "DecodeWorkload":
        """The same workload with every tensor on `device` (a workload drawn on the CPU replays
        bit for bit on any machine, which a device-side generator does not promise)."""
        return _moved(self, device)


def _moved(w, device):
    import dataclasses
    kw = {}
    for f in dataclasses.fields(w):
        v = getattr(w, f.name)
        if isinstance(v, torch.Tensor):
            v = v.to(device)
        elif isinstance(v, dict):
            v = {k: (x.to(device) if isinstance(x, torch.Tensor) else x) for k, x in v.items()}
        kw[f.name] = v
    return type(w)(**kw)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn_bf16(shape, g, device, std: float = 1.0, chunk_rows: int = 1 << 20, dtype=torch.bfloat16) -> torch.Tensor:
    """N(0, std^2) in fp32, rounded once to bf16 (or `dtype`); generated in slabs to bound the fp32 temporary."""
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1, shape[-1])
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        x = torch.randn((r1 - r0, shape[-1]), generator=g, device=device, dtype=torch.float32)
        if std != 1.0:
            x *= std
        flat[r0:r1] = x.to(dtype)
    return out


def _kv_torch_dtype(layer) -> torch.dtype:
    return {"bf16": torch.bfloat16, "fp16": torch.float16}[layer.kv_dtype]


def _unit(x: torch.Tensor) -> torch.Tensor:
    return x / x.norm(dim=-1, keepdim=True)


def _planted_positions(n_ctx: int, n_planted: int, g, device, runs_of: int = 0) -> torch.Tensor:
    """Distinct positions; optionally half of them laid out as contiguous runs."""
    if n_planted <= 0:
        return torch.empty(0, dtype=torch.long, device=device)
    if runs_of <= 1 or n_planted < 2 * runs_of or n_ctx < 8 * n_planted:
        perm = torch.randperm(n_ctx, generator=g, device=device)[:n_planted]
        return perm.sort().values
    n_run_tok = (n_planted // 2) // runs_of * runs_of
    n_runs = n_run_tok // runs_of
    # draw from a coarse grid so that runs never overlap each other or the isolated tokens
    slots = torch.randperm(n_ctx // runs_of, generator=g, device=device)
    run_starts = slots[:n_runs] * runs_of
    runs = (run_starts[:, None] + torch.arange(runs_of, device=device)[None, :]).reshape(-1)
    n_iso = n_planted - n_run_tok
    iso_off = torch.randint(0, runs_of, (n_iso,), generator=g, device=device)
    iso = slots[n_runs:n_runs + n_iso] * runs_of + iso_off
    return torch.cat([runs, iso]).sort().values


def planted_alpha(n_ctx: int, n_planted: int, frac: float, bg_std: float = 1.0) -> float:
    """Score level that gives `n_planted` tokens the share `frac` of the softmax
    mass against n_ctx background scores ~ N(0, bg_std^2)."""
    return math.log(frac / (1.0 - frac) * n_ctx * math.exp(0.5 * bg_std * bg_std) / n_planted)


def make_decode(name: str, layer: Layer, ctx_len: List[int], p, seed: int, device="cpu", *,
                index_mode: str = "direct", n_planted: int = 64, planted_frac: float = 0.85,
                planted_jitter: float = 0.25, bg_std=1.0, runs_of: int = 4,
                planted_rows=None) -> DecodeWorkload:
    """Build one decode-step workload.

    index_mode "direct": a unit-norm index query qI is handed over as is, the
        background index keys are N(0, bg_std^2 I) so background scores are
        N(0, bg_std^2), and planted keys are (alpha + N(0, jitter^2)) * qI_hat.
    index_mode "proj": fp32 projections W^Q ~ N(0, 1/D) and pre-RoPE queries are
        handed over; planted keys have cosine ~0.9 with W^Q q_pre.
    p: a float or a list with one value per sequence.
    bg_std / planted_rows: floats, or dicts keyed by (b, j) for per-row laws.
    """
    dev = torch.device(device)
    g = _gen(seed, dev)
    B, Hq, Hkv, D, r = len(ctx_len), layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.index_dim
    n_ret = layer.n_ret
    seq_start = [0]
    for n in ctx_len[:-1]:
        seq_start.append(seq_start[-1] + int(n))
    T_tot = int(sum(ctx_len))

    kvt = _kv_torch_dtype(layer)
    K = _randn_bf16((Hkv, T_tot, D), g, dev, dtype=kvt)
    V = _randn_bf16((Hkv, T_tot, D), g, dev, dtype=kvt)
    q = _randn_bf16((B, Hq, D), g, dev, dtype=kvt)
    kI = torch.empty((n_ret, T_tot, r), dtype=torch.bfloat16, device=dev)

    WQ = q_pre = qI = None
    if index_mode == "proj":
        WQ = torch.randn((n_ret, r, D), generator=g, device=dev, dtype=torch.float32) * (D ** -0.5)
        q_pre = _randn_bf16((B, Hq, D), g, dev)
        # direction of the index query, used ONLY to aim the planted keys
        aim = torch.einsum("jrd,bjd->bjr", WQ.double(),
                           q_pre[:, layer.ret_heads, :].double())
    elif index_mode == "direct":
        qI = _unit(torch.randn((B, n_ret, r), generator=g, device=dev, dtype=torch.float32)).to(torch.bfloat16)
        aim = qI.double()
    else:
        raise ValueError(index_mode)

    planted = {}
    for b in range(B):
        t0, n = seq_start[b], int(ctx_len[b])
        for j in range(n_ret):
            std = bg_std[(b, j)] if isinstance(bg_std, dict) else float(bg_std)
            npl = planted_rows[(b, j)] if isinstance(planted_rows, dict) else n_planted
            npl = min(int(npl), max(n // 8, 0))
            rows = torch.randn((n, r), generator=g, device=dev, dtype=torch.float32) * std
            pos = _planted_positions(n, npl, g, dev, runs_of)
            if npl > 0:
                a = aim[b, j].float()
                a_hat = a / a.norm()
                if index_mode == "proj":
                    u = torch.randn((npl, r), generator=g, device=dev, dtype=torch.float32)
                    u = _unit(u - (u @ a_hat)[:, None] * a_hat[None, :])
                    rows[pos] = a.norm() * (0.9 * a_hat[None, :] + math.sqrt(1.0 - 0.81) * u)
                else:
                    alpha = planted_alpha(n, npl, planted_frac, std)
                    lvl = alpha + planted_jitter * torch.randn((npl,), generator=g, device=dev,
                                                               dtype=torch.float32)
                    rows[pos] = lvl[:, None] * a_hat[None, :] / a.norm()
            kI[j, t0:t0 + n] = rows.to(torch.bfloat16)
            planted[(b, j)] = pos

    if isinstance(p, (list, tuple)):
        assert len(p) == B
        p_rows = torch.tensor([float(p[b]) for b in range(B) for _ in range(n_ret)], dtype=torch.float32)
    else:
        p_rows = torch.full((B * n_ret,), float(p), dtype=torch.float32)
    return DecodeWorkload(name=name, layer=layer, ctx_len=[int(n) for n in ctx_len], seq_start=seq_start,
                          q=q, K=K, V=V, kI=kI, p_rows=p_rows.to(dev), qI=qI, WQ=WQ, q_pre=q_pre,
                          planted=planted)


# ---------------------------------------------------------------------------
# the named decode configurations
# ---------------------------------------------------------------------------
def c1(device="cpu", seed: int = 0, ctx: int = 4096) -> DecodeWorkload:
    """Single decode step, 8 query / 2 KV heads, heads 0 and 4 retrieval, context 4096,
    fp32 projections, 8 planted tokens with cosine ~0.9, p = 0.9, 4 sink + 512 window."""
    layer = Layer(8, 2, [0, 4], sink=4, window=512)
    return make_decode("c1", layer, [ctx], 0.9, seed, device, index_mode="proj", n_planted=8, runs_of=0)


def c2(device="cpu", seed: int = 1, p: float = 0.9, ctx: int = 131072, batch: int = 8, kv_dtype: str = "bf16") -> DecodeWorkload:
    """Decode, 32 query / 8 KV heads, 4 retrieval heads, batch 8 x 131072, 64 planted
    tokens per row holding ~85 % of the indexer mass, background scores ~ N(0,1),
    local heads 4 sink + 2048 window."""
    layer = Layer(32, 8, [0, 8, 16, 24], sink=4, window=2048, kv_dtype=kv_dtype)
    return make_decode("c2", layer, [ctx] * batch, p, seed, device, index_mode="direct",
                       n_planted=64, planted_frac=0.85)


def c4_decode(device="cpu", seed: int = 3, ctx: int = 1 << 20) -> DecodeWorkload:
    """One decode step on the 1M-token layer: batch 1, 4 retrieval heads, p = 0.9,
    local heads 4 sink + 4096 window."""
    layer = Layer(32, 8, [0, 8, 16, 24], sink=4, window=4096)
    return make_decode("c4dec", layer, [ctx], 0.9, seed, device, index_mode="direct",
                       n_planted=64, planted_frac=0.85)


def c5(device="cpu", seed: int = 4, batch: int = 32, lo: int = 16384, hi: int = 262144) -> DecodeWorkload:
    """Ragged decode batch: contexts log-uniform in [lo, hi], 64 query / 8 KV heads,
    8 retrieval heads, per-sequence p ~ U[0.85, 0.98]; each (sequence, head) row
    draws its score law between flat (N(0, 0.3^2), no planted tokens) and peaked
    (N(0,1) background + 16 planted tokens), so the selected-set size spans > 100x."""
    dev = torch.device("cpu")
    g = _gen(seed * 7919 + 17, dev)
    u = torch.rand((batch,), generator=g)
    ctx = [int(math.exp(math.log(lo) + float(x) * (math.log(hi) - math.log(lo)))) for x in u]
    p = [0.85 + 0.13 * float(x) for x in torch.rand((batch,), generator=g)]
    layer = Layer(64, 8, list(range(0, 64, 8)), sink=4, window=2048)
    mix = torch.rand((batch, layer.n_ret), generator=g)
    bg, npl = {}, {}
    for b in range(batch):
        for j in range(layer.n_ret):
            m = float(mix[b, j])
            bg[(b, j)] = 0.3 + 0.7 * m            # flat ... N(0,1)
            npl[(b, j)] = 16 if m > 0.5 else 0    # peaked rows carry planted tokens
    return make_decode("c5", layer, ctx, p, seed, device, index_mode="direct",
                       planted_frac=0.85, bg_std=bg, planted_rows=npl)


def small_decode(device="cpu", seed: int = 11, ctx=(700, 1531, 64, 2048), *, n_q_heads=8, n_kv_heads=2,
                 ret_heads=(0, 1, 5), sink=4, window=96, p=(0.8, 0.9, 0.95, 0.9),
                 index_mode="direct", n_planted=8, kv_dtype="bf16") -> DecodeWorkload:
    """A shrunken ragged batch with every structural feature of the large ones:
    several sequences of unequal length, two retrieval heads sharing a KV head,
    contexts shorter and longer than sink + window."""
    layer = Layer(n_q_heads, n_kv_heads, list(ret_heads), sink=sink, window=window, kv_dtype=kv_dtype)
    p = [p[i % len(p)] for i in range(len(ctx))]          # one p per sequence, cycling the given ones
    return make_decode("small", layer, list(ctx), list(p), seed, device, index_mode=index_mode,
                       n_planted=n_planted, planted_frac=0.6)


# ---------------------------------------------------------------------------
# helpers for handing tensors to numpy consumers
# ---------------------------------------------------------------------------
def bf16_bits(t: torch.Tensor):
    """bf16 (or fp16) tensor -> numpy uint16 array of its bit patterns (a copy on the host)."""
    import numpy as np
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


# ---------------------------------------------------------------------------
# prefill workloads (one sequence, one chunk of queries)
# ---------------------------------------------------------------------------
@dataclass
class PrefillWorkload:
    name: str
    layer: Layer
    N: int                          # cached tokens, the chunk's own tokens included (= chunk_start + T)
    chunk_start: int
    T: int
    p: float
    q: torch.Tensor                 # bf16 [T, Hq, D]      post-RoPE queries of the chunk
    K: torch.Tensor                 # bf16 [Hkv, N, D]
    V: torch.Tensor                 # bf16 [Hkv, N, D]
    kI: torch.Tensor                # bf16 [n_ret, N, r]
    qI: Optional[torch.Tensor] = None      # bf16 [n_ret, T, r]
    WQ: Optional[torch.Tensor] = None      # fp32 [n_ret, r, D]
    q_pre: Optional[torch.Tensor] = None   # bf16 [T, Hq, D]
    cluster_start: Optional[torch.Tensor] = None
    cluster_size: Optional[torch.Tensor] = None

    def to(self, device) -> "PrefillWorkload":
        return _moved(self, device)


def make_prefill(name: str, layer: Layer, chunk_start: int, T: int, p: float, seed: int, device="cpu", *,
                 index_mode: str = "direct", tokens_per_cluster: int = 1024, cluster_len=32,
                 own_frac: float = 0.8, q_noise: float = 0.3, zipf: float = 0.0, max_cluster: int = 4096,
                 pick_run: int = 1) -> PrefillWorkload:
    """One causal prefill chunk: queries at positions chunk_start .. chunk_start+T-1 of a sequence
    whose first chunk_start+T tokens are cached.

    Index side ("direct"): N / tokens_per_cluster planted clusters, each a run of consecutive tokens
    (length cluster_len, or Zipf(zipf)-distributed in [1, max_cluster]) whose index keys are
    a * u_c + N(0, sb^2 I) for a random unit direction u_c; background keys are N(0, sb^2 I).  Query m
    picks one cluster that starts before m (probability proportional to its size; with pick_run > 1 a run of
    that many consecutive queries shares the pick of its first query, the way neighbouring prompt tokens ask for
    the same passage) and gets qI = g * u_c + N(0, q_noise^2 I).  g = a and sb are set so that background scores have unit
    variance and the own cluster holds about own_frac of the indexer mass at the full context; the
    other clusters (random directions, cosine std 1/4) supply the tail.
    "proj": fp32 projections and pre-RoPE queries, index keys plain N(0, I) (no planted structure).
    """
    dev = torch.device(device)
    g = _gen(seed, dev)
    Hq, Hkv, D, r, n_ret = layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.index_dim, layer.n_ret
    N = int(chunk_start) + int(T)
    kvt = _kv_torch_dtype(layer)
    K = _randn_bf16((Hkv, N, D), g, dev, dtype=kvt)
    V = _randn_bf16((Hkv, N, D), g, dev, dtype=kvt)
    q = _randn_bf16((T, Hq, D), g, dev, dtype=kvt)
    WQ = q_pre = qI = cstart = csize = None
    if index_mode == "proj":
        WQ = torch.randn((n_ret, r, D), generator=g, device=dev, dtype=torch.float32) * (D ** -0.5)
        q_pre = _randn_bf16((T, Hq, D), g, dev)
        kI = _randn_bf16((n_ret, N, r), g, dev, std=0.6)
    else:
        n_cl = max(1, N // tokens_per_cluster)
        if zipf > 0.0:
            ranks = torch.arange(1, max_cluster + 1, device=dev, dtype=torch.float64)
            pmf = ranks ** (-zipf)
            csize = torch.multinomial((pmf / pmf.sum()).float(), n_cl, replacement=True, generator=g) + 1
        else:
            csize = torch.full((n_cl,), int(cluster_len), device=dev, dtype=torch.long)
        csize = csize.clamp(max=max(1, N // 2))
        cstart = (torch.rand((n_cl,), generator=g, device=dev) * (N - csize).clamp(min=1).float()).long()
        mean_len = float(csize.float().mean())
        ga = math.log(own_frac / (1.0 - own_frac) * N * math.exp(0.5) / max(mean_len, 1.0))
        a_lvl = math.sqrt(max(ga, 1.0))
        sb = 1.0 / math.sqrt(a_lvl * a_lvl + r * q_noise * q_noise)
        kI = torch.empty((n_ret, N, r), dtype=torch.bfloat16, device=dev)
        qI = torch.empty((n_ret, T, r), dtype=torch.bfloat16, device=dev)
        pos = chunk_start + torch.arange(T, device=dev)
        for j in range(n_ret):
            u = _unit(torch.randn((n_cl, r), generator=g, device=dev, dtype=torch.float32))
            rows = torch.randn((N, r), generator=g, device=dev, dtype=torch.float32) * sb
            # cluster membership: later clusters overwrite earlier ones where runs overlap
            owner = torch.full((N,), -1, device=dev, dtype=torch.long)
            for cidx in range(n_cl):
                s0, ln = int(cstart[cidx]), int(csize[cidx])
                owner[s0:s0 + ln] = cidx
            member = owner >= 0
            rows[member] += a_lvl * u[owner[member]]
            kI[j] = rows.to(torch.bfloat16)
            # each query picks a cluster that starts before it (weight = size); none -> cluster 0
            w = csize.float()[None, :] * (cstart[None, :] < pos[:, None]).float()
            w[:, 0] += 1e-6
            pick = torch.multinomial(w, 1, generator=g).squeeze(1)
            if pick_run > 1:
                pick = pick[(torch.arange(T, device=dev) // pick_run) * pick_run]
            qq = a_lvl * u[pick] + q_noise * torch.randn((T, r), generator=g, device=dev, dtype=torch.float32)
            qI[j] = qq.to(torch.bfloat16)
    return PrefillWorkload(name=name, layer=layer, N=N, chunk_start=int(chunk_start), T=int(T), p=float(p),
                           q=q, K=K, V=V, kI=kI, qI=qI, WQ=WQ, q_pre=q_pre, cluster_start=cstart,
                           cluster_size=csize)


def c3_chunk(device="cpu", seed: int = 2, chunk: int = 31, N_total: int = 131072, T: int = 4096,
             p: float = 0.9) -> PrefillWorkload:
    """Chunked prefill, configuration 3: one 4096-query chunk of a 131072-token sequence (chunk index
    0..31; the last one sees the whole context), 32 query / 8 KV heads, 4 retrieval heads, clusters of
    32 relevant tokens, top-p 0.9, local heads 4 sink + 2048 window."""
    layer = Layer(32, 8, [0, 8, 16, 24], sink=4, window=2048)
    return make_prefill("c3", layer, chunk * T, T, p, seed, device, cluster_len=32)


def c4_chunk(device="cpu", seed: int = 3, chunk: int = 127, T: int = 8192, p: float = 0.9, law: str = "broad") -> PrefillWorkload:
    """Configuration 4: one 8192-query chunk of a 1,048,576-token prefill (chunk index 0..127),
    4 retrieval heads over the full cache, local heads 4 sink + 4096 window.
    law "broad": cluster sizes Zipf(1.1) in [1, 4096], the own cluster holds about 0.8 of the indexer mass, every
    query picks its own cluster: p = 0.9 reaches into the tail and keeps thousands of tokens per query.
    law "peaked": one cluster of 32 tokens per 32768 (few enough that the other clusters' tails stay small) that
    holds about 0.97 of its queries' mass, runs of 64 queries share a cluster, little query noise: p = 0.9 is
    reached inside the cluster for every query, about 20 kept tokens.
    law "peaked_hard": the same with the cluster at 0.995 of the mass and the query noise of the broad law: a
    median of about 20 kept tokens, and one or two queries in a thousand with a weak cluster and up to hundreds
    of thousands of kept tokens (a query tile with such a query has to visit every key tile)."""
    layer = Layer(32, 8, [0, 8, 16, 24], sink=4, window=4096)
    if law == "peaked":
        return make_prefill("c4_peaked", layer, chunk * T, T, p, seed, device, cluster_len=32, own_frac=0.97, pick_run=64,
                            tokens_per_cluster=32768, q_noise=0.1)
    if law == "peaked_hard":
        return make_prefill("c4_peaked_hard", layer, chunk * T, T, p, seed, device, cluster_len=32, own_frac=0.995,
                            pick_run=64, tokens_per_cluster=32768)
    if law != "broad":
        raise ValueError("law must be 'broad', 'peaked' or 'peaked_hard'")
    return make_prefill("c4", layer, chunk * T, T, p, seed, device, zipf=1.1)


def small_prefill(device="cpu", seed: int = 41, chunk_start: int = 700, T: int = 200, p: float = 0.9, *,
                  n_q_heads=8, n_kv_heads=2, ret_heads=(0, 5), sink=4, window=160, index_mode="direct",
                  tokens_per_cluster=128, cluster_len=8, zipf=0.0, kv_dtype="bf16", own_frac=0.8, pick_run=1) -> PrefillWorkload:
    layer = Layer(n_q_heads, n_kv_heads, list(ret_heads), sink=sink, window=window, kv_dtype=kv_dtype)
    return make_prefill("small_prefill", layer, chunk_start, T, p, seed, device, index_mode=index_mode,
                        tokens_per_cluster=tokens_per_cluster, cluster_len=cluster_len, zipf=zipf, max_cluster=64,
                        own_frac=own_frac, pick_run=pick_run)
