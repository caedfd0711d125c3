"""Pins for the oracle's scoring, compaction, attention and block step (CPU only)."""
import math

import numpy as np
import pytest
import torch

from oracle import sdllm_oracle as orc
from paper_2508_02558_amd import workloads as wl


def _brute_attention(q, k, v, scale):
    """Triple-loop softmax attention, one scalar at a time (GQA: head h reads KV head h // G)."""
    hq, n, d = q.shape
    hkv, m, dv = v.shape
    grp = hq // hkv
    out = np.zeros((hq, n, dv))
    for h in range(hq):
        for i in range(n):
            logits = [sum(q[h, i, t] * k[h // grp, j, t] for t in range(d)) * scale for j in range(m)]
            mx = max(logits)
            w = [math.exp(x - mx) for x in logits]
            z = sum(w)
            for j in range(m):
                for t in range(dv):
                    out[h, i, t] += w[j] / z * v[h // grp, j, t]
    return out


def test_attention_brute_force_and_torch_sdpa():
    rng = np.random.default_rng(0)
    for hq, hkv in ((2, 2), (4, 2), (6, 1)):
        q = rng.standard_normal((hq, 3, 8))
        k = rng.standard_normal((hkv, 5, 8))
        v = rng.standard_normal((hkv, 5, 8))
        ours = orc.attention(q, k, v)
        np.testing.assert_allclose(ours, _brute_attention(q, k, v, 1 / math.sqrt(8)), rtol=1e-12, atol=1e-13)
        grp = hq // hkv
        lib = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q)[None], torch.from_numpy(k).repeat_interleave(grp, 0)[None],
            torch.from_numpy(v).repeat_interleave(grp, 0)[None])[0].numpy()
        np.testing.assert_allclose(ours, lib, rtol=1e-12, atol=1e-13)
    # explicit scale is honoured
    np.testing.assert_allclose(orc.attention(q, k, v, 0.3), _brute_attention(q, k, v, 0.3), rtol=1e-12)


def test_attention_closed_forms():
    rng = np.random.default_rng(1)
    k = rng.standard_normal((2, 9, 16))
    v = rng.standard_normal((2, 9, 16))
    # zero queries -> uniform weights -> mean of V
    out = orc.attention(np.zeros((2, 4, 16)), k, v)
    np.testing.assert_allclose(out, np.broadcast_to(v.mean(axis=1, keepdims=True), out.shape), rtol=1e-13)
    # one key dominates (logit +40 above the rest) and carries a one-hot value
    q = np.zeros((1, 1, 4)); q[0, 0, 0] = 1.0
    kk = np.zeros((1, 6, 4)); kk[0, 2, 0] = 40.0 * 2.0      # scale 1/sqrt(4) = 0.5 -> logit 40
    vv = rng.standard_normal((1, 6, 4)); vv[0, 2] = [0, 0, 1, 0]
    out = orc.attention(q, kk, vv)
    np.testing.assert_allclose(out[0, 0], [0, 0, 1, 0], atol=1e-15)
    # permuting the keys (with their values) changes nothing
    q = rng.standard_normal((2, 4, 16))
    perm = rng.permutation(9)
    np.testing.assert_allclose(orc.attention(q, k, v), orc.attention(q, k[:, perm], v[:, perm]), rtol=1e-12, atol=1e-14)


def test_sparse_attention_special_cases():
    rng = np.random.default_rng(2)
    hq, hkv, b, d, L, o = 4, 2, 4, 8, 20, 8
    q = rng.standard_normal((hq, b, d))
    k = rng.standard_normal((hkv, L, d))
    v = rng.standard_normal((hkv, L, d))
    kn, vn = k[:, o:o + b], v[:, o:o + b]
    # Concat order is cache first, block last (Alg. 3)
    kc, vc = rng.standard_normal((hkv, 5, d)), rng.standard_normal((hkv, 5, d))
    ref = orc.attention(q, np.concatenate([kc, kn], 1), np.concatenate([vc, vn], 1))
    np.testing.assert_array_equal(orc.sparse_attention(q, kc, vc, kn, vn), ref)
    # empty cache -> plain b x b attention over the block
    empty = np.zeros((hkv, 0, d))
    np.testing.assert_allclose(orc.sparse_attention(q, empty, empty, kn, vn), orc.attention(q, kn, vn), rtol=1e-14)
    # r = 1: every candidate is retained, so the sparse step reproduces dense attention
    idx, _, _ = orc.score_select(q, k, o, b, 1.0, 3)
    assert idx.shape == (hkv, L - b)
    for g in range(hkv):
        assert idx[g].tolist() == orc.candidate_positions(L, o, b).tolist()
    kc, vc = orc.compact_kv(k, v, idx)
    np.testing.assert_allclose(orc.sparse_attention(q, kc, vc, kn, vn), orc.dense_block_attention(q, k, v),
                               rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ scoring
def _brute_score(q, k, o, b, mode, scale):
    hq, nb, d = q.shape
    hkv, L, _ = k.shape
    grp = hq // hkv
    cand = [c for c in range(L) if not (o <= c < o + b)]
    out = np.zeros((hkv, len(cand)))
    for h in range(hq):
        for i in range(nb):
            logits = [sum(q[h, i, t] * k[h // grp, c, t] for t in range(d)) * scale for c in cand]
            if mode == orc.SOFTMAX_MEAN:
                mx = max(logits)
                w = [math.exp(x - mx) for x in logits]
                z = sum(w)
                w = [x / z for x in w]
            else:
                w = logits
            for j in range(len(cand)):
                out[h // grp, j] += w[j] / (grp * nb)
    return out


@pytest.mark.parametrize("mode", [orc.SOFTMAX_MEAN, orc.LOGIT_MEAN])
def test_score_brute_force(mode):
    rng = np.random.default_rng(3)
    for hq, hkv, o in ((2, 2, 4), (6, 2, 0), (3, 1, 9)):
        q = rng.standard_normal((hq, 3, 8))
        k = rng.standard_normal((hkv, 12, 8))
        got = orc.saliency_score(q, k, o, 3, mode)
        np.testing.assert_allclose(got, _brute_score(q, k, o, 3, mode, 1 / math.sqrt(8)), rtol=1e-12, atol=1e-14)
        assert got.shape == (hkv, 9)


def test_logits_are_the_scaled_products_of_the_candidates():
    rng = np.random.default_rng(4)
    q = rng.standard_normal((2, 3, 16)); k = rng.standard_normal((2, 10, 16))
    a = orc.saliency_logits(q, k, 4, 3)
    kf = np.concatenate([k[:, :4], k[:, 7:]], axis=1)
    np.testing.assert_allclose(a, np.einsum("hid,hcd->hic", q, kf) / 4.0, rtol=1e-13)


def test_logit_mean_is_mean_query_times_keys():
    """Alg. 1 steps 5-6 (mean query, then MatMul) equal the column mean of the main-text logits."""
    rng = np.random.default_rng(5)
    q = rng.standard_normal((4, 32, 16)); k = rng.standard_normal((4, 50, 16))
    score = orc.saliency_score(q, k, 10, 32, orc.LOGIT_MEAN, scale=1.0)
    kf = np.concatenate([k[:, :10], k[:, 42:]], axis=1)
    qbar = q.mean(axis=1)
    np.testing.assert_allclose(score, np.einsum("hd,hcd->hc", qbar, kf), rtol=1e-12, atol=1e-13)


def test_softmax_mean_is_a_distribution_and_zero_queries_give_uniform():
    rng = np.random.default_rng(6)
    q = rng.standard_normal((6, 8, 16)); k = rng.standard_normal((2, 40, 16))
    score = orc.saliency_score(q, k, 16, 8)
    np.testing.assert_allclose(score.sum(axis=-1), 1.0, rtol=1e-13)
    assert (score >= 0).all()
    # Q = 0 -> every candidate scores 1/N -> all ties -> the lowest positions of each segment win
    idx, pooled, score = orc.score_select(np.zeros((6, 8, 16)), k, 16, 8, 0.5, 3)
    np.testing.assert_allclose(score, 1.0 / 32, rtol=1e-15)
    for g in range(2):
        assert idx[g].tolist() == list(range(8)) + list(range(24, 32))


def test_planted_salient_keys_are_retained():
    w = wl.WORKLOADS["tiny"]
    inp = wl.make_block_inputs(w)
    o, b = inp["block_off"], w.block
    q = wl.to_f64(inp["q"][1, 0]); k = wl.to_f64(inp["k_full"][0])
    for mode in (orc.SOFTMAX_MEAN, orc.LOGIT_MEAN):
        idx, _, _ = orc.score_select(q, k, o, b, w.retention, w.pool_kernel, mode)
        for g in range(w.n_kv_heads):
            kept = set(idx[g].tolist())
            for p in inp["salient"].tolist():
                assert {p - 1, p, p + 1} <= kept, (mode, g, p)      # the peak and its pooled neighbours
    w1 = wl.WORKLOADS["llada8b_layer"].scaled(n_q_heads=2, n_kv_heads=2, prompt=256, gen=64)
    inp = wl.make_block_inputs(w1, n_steps=2)
    idx, _, _ = orc.score_select(wl.to_f64(inp["q"][1, 0]), wl.to_f64(inp["k_full"][0]), inp["block_off"],
                                 w1.block, w1.retention, w1.pool_kernel)
    sal = inp["salient"].tolist()
    assert len(sal) > 0
    for g in range(2):
        assert set(sal) <= set(idx[g].tolist())


def test_compaction_is_a_row_gather():
    rng = np.random.default_rng(7)
    k = rng.standard_normal((2, 12, 4)); v = rng.standard_normal((2, 12, 4))
    idx = np.array([[0, 3, 11], [1, 2, 7]])
    kc, vc = orc.compact_kv(k, v, idx)
    for g in range(2):
        for j in range(3):
            assert (kc[g, j] == k[g, idx[g, j]]).all() and (vc[g, j] == v[g, idx[g, j]]).all()


def test_block_step_schedule_and_outputs():
    w = wl.WORKLOADS["tiny"]
    inp = wl.make_block_inputs(w)
    o, b = inp["block_off"], w.block
    cache = {}
    k_full, v_full = inp["k_full"][0].clone(), inp["v_full"][0].clone()
    states = []
    for t in range(4):
        q = wl.to_f64(inp["q"][t, 0])
        if orc.cache_state(t, 1) < 2:
            k_full[:, o:o + b] = inp["k_blk"][t, 0]; v_full[:, o:o + b] = inp["v_blk"][t, 0]
            out, st = orc.block_step(t, 1, q, wl.to_f64(k_full), wl.to_f64(v_full), cache, block_off=o,
                                     block_len=b, r=w.retention, s=w.pool_kernel)
            np.testing.assert_array_equal(out, orc.dense_block_attention(q, wl.to_f64(k_full), wl.to_f64(v_full)))
        else:
            kn, vn = wl.to_f64(inp["k_blk"][t, 0]), wl.to_f64(inp["v_blk"][t, 0])
            out, st = orc.block_step(t, 1, q, kn, vn, cache, block_off=o, block_len=b, r=w.retention,
                                     s=w.pool_kernel)
            np.testing.assert_array_equal(out, orc.sparse_attention(q, cache["k"], cache["v"], kn, vn))
        states.append(st)
        if t == 0:
            assert cache == {}
    assert states == [0, 1, 2, 2]
    assert cache["idx"].shape == (2, 64) and cache["k"].shape == (2, 64, 64)


def test_workload_shapes_and_determinism():
    w = wl.WORKLOADS["tiny"]
    a, b_ = wl.make_block_inputs(w), wl.make_block_inputs(w)
    assert w.seq_len == 160 and a["block_off"] == 64
    for key in ("k_full", "v_full", "q", "k_blk", "v_blk"):
        assert torch.equal(a[key], b_[key])
    assert a["q"].shape == (4, 1, 2, 32, 64) and a["k_full"].shape == (1, 2, 160, 64)
    sal = a["salient"].tolist()
    assert len(sal) == 4 and all(0 < p < 63 for p in sal) and min(np.diff(sal)) >= 3
    names = [x.name for x in wl.WORKLOAD_LIST]
    assert names[:5] == ["tiny", "llada8b_layer", "dream7b_gqa", "llada8b_sweep", "dream_long"]
    assert wl.WORKLOADS["llada8b_gen512"].n_blocks == 16
    w4 = wl.WORKLOADS["dream_long"]
    assert w4.seq_len - w4.block == 33248
