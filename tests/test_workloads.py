"""The seeded input generators: determinism, layout, and that the recipes give the
indexer-mass structure they promise (checked with the oracle on small sizes)."""
import numpy as np
import pytest
import torch

from oracle import rtp_oracle as orc
from paper_2605_16928_amd import workloads as wl


def test_deterministic_and_shapes():
    a, b = wl.small_decode(seed=5), wl.small_decode(seed=5)
    c = wl.small_decode(seed=6)
    for name in ("q", "K", "V", "kI", "qI", "p_rows"):
        assert torch.equal(getattr(a, name), getattr(b, name))
    assert not torch.equal(a.K, c.K)
    L = a.layer
    assert a.K.shape == (L.n_kv_heads, sum(a.ctx_len), 128) and a.K.dtype == torch.bfloat16
    assert a.kI.shape == (L.n_ret, sum(a.ctx_len), 16)
    assert a.q.shape == (a.B, L.n_q_heads, 128) and a.qI.shape == (a.B, L.n_ret, 16)
    assert a.seq_start == [0, 700, 2231, 2295] and a.p_rows.shape == (a.B * L.n_ret,)


def test_c1_recipe():
    w = wl.c1()
    assert w.layer.ret_heads == [0, 4] and w.ctx_len == [4096] and (w.layer.sink, w.layer.window) == (4, 512)
    assert w.WQ.shape == (2, 16, 128) and w.WQ.dtype == torch.float32 and w.qI is None
    kI = wl.bf16_bits(w.kI)
    for j, h in enumerate(w.layer.ret_heads):
        qI = orc.bf16_to_f64(orc.index_project(w.WQ[j].numpy(), wl.bf16_bits(w.q_pre)[0, h]))
        pos = w.planted[(0, j)].numpy()
        assert len(pos) == 8
        k = orc.bf16_to_f64(kI[j, pos])
        cos = (k @ qI) / (np.linalg.norm(k, axis=1) * np.linalg.norm(qI))
        assert np.all(np.abs(cos - 0.9) < 0.02)


def test_c2_recipe_small_ctx_mass_is_peaky():
    w = wl.c2(ctx=8192, batch=2)
    kI, qI = wl.bf16_bits(w.kI), wl.bf16_bits(w.qI)
    for b in range(2):
        for j in range(4):
            t0 = w.seq_start[b]
            s = orc.index_score(qI[b, j], kI[j, t0:t0 + 8192])
            wgt = np.exp(s - s.max())
            share = wgt[w.planted[(b, j)].numpy()].sum() / wgt.sum()
            assert 0.7 < share < 0.95
            assert orc.topp_select(s, 0.8)["count"] <= 64
            assert orc.topp_select(s, 0.95)["count"] > 500


def test_c5_recipe_spans_flat_to_peaked():
    w = wl.c5(batch=6, lo=4096, hi=16384)
    assert all(4096 <= n <= 16384 for n in w.ctx_len) and len(set(w.ctx_len)) > 1
    assert float(w.p_rows.min()) >= 0.85 and float(w.p_rows.max()) <= 0.98
    kI, qI = wl.bf16_bits(w.kI), wl.bf16_bits(w.qI)
    fr = []
    for b in range(w.B):
        for j in range(w.layer.n_ret):
            t0, n = w.seq_start[b], w.ctx_len[b]
            s = orc.index_score(qI[b, j], kI[j, t0:t0 + n])
            fr.append(orc.topp_select(s, float(w.p_rows[b * w.layer.n_ret + j]))["count"] / n)
    assert max(fr) > 0.6 and min(fr) < 0.1


def test_prefill_laws_broad_and_peaked():
    """The prefill recipes at a size the oracle handles: with the own cluster at 99 % of the mass and runs of
    queries sharing a cluster, top-p 0.9 stays inside the cluster (a handful of tokens, the same for the queries of
    a run); with the broad law (own cluster 80 %) it reaches into the tail."""
    kept = {}
    for name, kw in (("peaked", dict(own_frac=0.99, pick_run=32)), ("broad", dict())):
        w = wl.small_prefill("cpu", seed=70, chunk_start=6000, T=96, p=0.9, **kw)
        kI, qI = wl.bf16_bits(w.kI), wl.bf16_bits(w.qI)
        kept[name] = np.array([orc.topp_select(orc.index_score(qI[0, t], kI[0, :6000 + t + 1]), 0.9)["count"]
                               for t in range(0, 96, 4)])
    assert np.median(kept["peaked"]) <= 10 < np.median(kept["broad"])
    # pick_run: the index queries of a run aim at one cluster
    w = wl.small_prefill("cpu", seed=70, chunk_start=6000, T=96, p=0.9, own_frac=0.99, pick_run=32)
    q = w.qI[0].float()
    cos = torch.nn.functional.cosine_similarity(q[:32].mean(0, keepdim=True), q[:32]).min()
    assert cos > 0.8
    with pytest.raises(ValueError):
        wl.c4_chunk("cpu", law="sharp", T=8, chunk=0)
