"""Pins for the oracle's pooling, counting, selection and schedule (CPU only)."""
import itertools

import numpy as np
import pytest
import torch
from scipy.ndimage import maximum_filter1d

from oracle import sdllm_oracle as orc


def _floats(s):
    return np.array([float(x) for x in s.split()], dtype=np.float64)


def _ints(s):
    return [int(x) for x in s.split()]


# ------------------------------------------------------------------ golden: hand-worked examples
def test_hand_worked_8_token_examples(golden):
    rows = golden("select_8token.txt")
    assert len(rows) == 6
    for name, mode, s, r_or_k, layout, scores, pooled_exp, kept_exp in rows:
        scores, pooled_exp, kept_exp = _floats(scores), _floats(pooled_exp), _ints(kept_exp)
        s = int(s)
        if mode == orc.PREFIX_ONLY:
            # Alg. 4 through the oracle's only entry that implements it.  One head, head_dim 1, both block
            # queries equal to 1 and scale 1: in "logit_mean" mode the score of a key IS its value, so the
            # hand-worked scores go in as keys (the block's own two keys are arbitrary).
            o, b, L = (int(kv.split("=")[1]) for kv in layout.split(","))
            keys = np.concatenate([scores[:o], [7.0, -3.0], scores[o:]])
            idx, pooled, score = orc.score_select(np.ones((1, b, 1)), keys.reshape(1, L, 1), o, b, float(r_or_k), s,
                                                  orc.LOGIT_MEAN, scale=1.0, evict_scope=orc.PREFIX_ONLY)
            np.testing.assert_allclose(score[0], scores[:o], rtol=0, atol=1e-15, err_msg=name)
            np.testing.assert_allclose(pooled[0], pooled_exp, rtol=0, atol=1e-15, err_msg=name)
            assert idx[0].tolist() == kept_exp, name
        elif layout.startswith("seg:"):
            pooled = orc.pool_1d(scores, s)
            np.testing.assert_allclose(pooled, pooled_exp, rtol=0, atol=0, err_msg=name)
            kept = orc.top_k_lowest_position(pooled, int(r_or_k))
            assert kept.tolist() == kept_exp, name
        else:
            o, b, L = (int(kv.split("=")[1]) for kv in layout.split(","))
            rounding = orc.FLOOR if mode == orc.JOINT else orc.CEIL
            pooled = orc.pool_scores(scores, o, s, mode)
            np.testing.assert_allclose(pooled, pooled_exp, rtol=0, atol=0, err_msg=name)
            idx, k_pre = orc.select_indices(pooled, L, o, b, float(r_or_k), mode, rounding)
            assert idx.tolist() == kept_exp, name
            assert k_pre == sum(1 for p in kept_exp if p < o)


def test_cache_state_table(golden):
    rows = golden("cache_state_table.txt")
    assert [int(r[0]) for r in rows] == [0, 1, 2, 3, 4, 5]
    for delay, states in rows:
        for i, st in enumerate(_ints(states)):
            assert orc.cache_state(i, int(delay)) == st
    # Alg. 2 is the delay-1 special case: state = i for i <= 1, else 2
    assert [orc.cache_state(i) for i in range(5)] == [0, 1, 2, 2, 2]


def test_retained_count_table(golden):
    for r, n, ceil_k, floor_k in golden("retained_count_table.txt"):
        assert orc.retained_count(int(n), float(r), orc.CEIL) == int(ceil_k), (r, n)
        assert orc.retained_count(int(n), float(r), orc.FLOOR) == int(floor_k), (r, n)


# ------------------------------------------------------------------ pooling
@pytest.mark.parametrize("s", [1, 3, 5, 7, 9])
def test_max_pool_matches_library_routines(s):
    rng = np.random.default_rng(s)
    for n in (1, 2, 3, 8, 31, 200):
        x = rng.standard_normal(n)
        ours = orc.pool_1d(x, s)
        # the op Alg. 1 names: MaxPool1D(kernel_size=s, padding=s/2), stride 1
        lib = torch.nn.functional.max_pool1d(torch.from_numpy(x)[None, None], kernel_size=s,
                                             stride=1, padding=s // 2)[0, 0].numpy()
        np.testing.assert_array_equal(ours, lib)
        lib2 = maximum_filter1d(x, size=s, mode="constant", cval=-np.inf)
        np.testing.assert_array_equal(ours, lib2)
        assert (ours >= x).all()
    x = rng.standard_normal(17)
    np.testing.assert_array_equal(orc.pool_1d(x, 1), x)


def test_avg_pool_matches_library_routine():
    rng = np.random.default_rng(5)
    for s in (1, 3, 5):
        x = rng.standard_normal(40)
        lib = torch.nn.functional.avg_pool1d(torch.from_numpy(x)[None, None], kernel_size=s, stride=1,
                                             padding=s // 2, count_include_pad=True)[0, 0].numpy()
        np.testing.assert_allclose(orc.pool_1d(x, s, orc.AVG_POOL), lib, rtol=1e-14, atol=1e-15)


def test_even_pool_kernel_rejected():
    with pytest.raises(ValueError):
        orc.pool_1d(np.zeros(4), 2)


def test_pool_seam_handling():
    # a spike on the last prefix candidate leaks into the suffix only in joint mode
    score = np.zeros(10)
    score[3] = 1.0
    per = orc.pool_scores(score, 4, 3, orc.PER_SEGMENT)
    joint = orc.pool_scores(score, 4, 3, orc.JOINT)
    assert per.tolist() == [0, 0, 1, 1, 0, 0, 0, 0, 0, 0]
    assert joint.tolist() == [0, 0, 1, 1, 1, 0, 0, 0, 0, 0]


# ------------------------------------------------------------------ selection
def _brute_force_topk(values, k):
    """Among all k-subsets: maximal sum of values, then lexicographically smallest positions."""
    best, best_key = None, None
    for comb in itertools.combinations(range(len(values)), k):
        key = (-sum(values[c] for c in comb), comb)
        if best_key is None or key < best_key:
            best, best_key = comb, key
    return list(best) if best is not None else []


def test_topk_brute_force_with_ties():
    rng = np.random.default_rng(11)
    for trial in range(60):
        n = int(rng.integers(1, 12))
        # few distinct dyadic values -> many exact ties, exact sums
        vals = rng.integers(0, 4, size=n).astype(np.float64) / 4.0
        for k in range(0, n + 1):
            got = orc.top_k_lowest_position(vals, k).tolist()
            assert got == _brute_force_topk(vals, k), (vals, k)


def test_topk_matches_torch_topk_without_ties():
    rng = np.random.default_rng(12)
    for n, k in ((50, 10), (257, 128), (1000, 1)):
        v = rng.standard_normal(n)
        lib = sorted(torch.topk(torch.from_numpy(v), k).indices.tolist())
        assert orc.top_k_lowest_position(v, k).tolist() == lib
        # s = 1: selection is the stable argsort prefix
        assert lib == sorted(np.argsort(-v, kind="stable")[:k].tolist())


@pytest.mark.parametrize("mode,rounding", [(orc.PER_SEGMENT, orc.CEIL), (orc.JOINT, orc.FLOOR),
                                           (orc.PER_SEGMENT, orc.FLOOR), (orc.JOINT, orc.CEIL)])
def test_selection_invariants(mode, rounding):
    rng = np.random.default_rng(13)
    for (L, o, b, r, s) in [(160, 64, 32, 0.5, 3), (100, 0, 32, 0.3, 5), (96, 64, 32, 0.7, 3),
                            (77, 20, 7, 0.25, 1), (64, 16, 32, 1.0, 3), (64, 16, 32, 0.0, 3)]:
        n_pre, n_suf = o, L - o - b
        score = rng.random(n_pre + n_suf)
        pooled = orc.pool_scores(score, n_pre, s, mode)
        idx, k_pre = orc.select_indices(pooled, L, o, b, r, mode, rounding)
        assert (np.diff(idx) > 0).all()                         # sorted, no duplicates
        assert not ((idx >= o) & (idx < o + b)).any()           # never the current block
        assert ((idx >= 0) & (idx < L)).all()
        if mode == orc.PER_SEGMENT:
            assert k_pre == orc.retained_count(n_pre, r, rounding)
            assert idx.size - k_pre == orc.retained_count(n_suf, r, rounding)
            segs = [(0, n_pre), (n_pre, n_pre + n_suf)]
        else:
            assert idx.size == orc.retained_count(n_pre + n_suf, r, rounding)
            segs = [(0, n_pre + n_suf)]
        cand = orc.candidate_positions(L, o, b)
        kept = np.isin(cand, idx)
        for lo, hi in segs:
            kv, ev = pooled[lo:hi][kept[lo:hi]], pooled[lo:hi][~kept[lo:hi]]
            if kv.size and ev.size:
                thr = kv.min()
                assert thr >= ev.max()
                # among values equal to the threshold the kept ones are the lowest positions
                eq = np.nonzero(pooled[lo:hi] == thr)[0]
                kept_eq = kept[lo:hi][eq]
                assert not (np.diff(kept_eq.astype(int)) > 0).any()


def test_r_one_keeps_everything_and_r_zero_nothing():
    pooled = np.random.default_rng(3).random(128)
    idx, k_pre = orc.select_indices(pooled, 160, 64, 32, 1.0)
    assert idx.tolist() == orc.candidate_positions(160, 64, 32).tolist() and k_pre == 64
    idx, k_pre = orc.select_indices(pooled, 160, 64, 32, 0.0)
    assert idx.size == 0 and k_pre == 0


def test_candidate_positions():
    assert orc.candidate_positions(10, 4, 2).tolist() == [0, 1, 2, 3, 6, 7, 8, 9]
    assert orc.candidate_positions(6, 0, 2).tolist() == [2, 3, 4, 5]
    assert orc.candidate_positions(6, 4, 2).tolist() == [0, 1, 2, 3]


def test_prefix_only_eviction_keeps_the_whole_suffix():
    """Alg. 4: the prefix is ranked exactly as a sequence that ends with the block would be, and every
    suffix position is appended.  (The hand-worked row `alg4_prefix_only` of the golden file pins the
    same branch without going through the oracle's own bidirectional path.)"""
    rng = np.random.default_rng(21)
    hq, hkv, b, d, L, o = 4, 2, 4, 8, 30, 12
    q = rng.standard_normal((hq, b, d)); k = rng.standard_normal((hkv, L, d))
    idx, pooled, score = orc.score_select(q, k, o, b, 0.5, 3, evict_scope=orc.PREFIX_ONLY)
    ref, pooled_ref, _ = orc.score_select(q, k[:, :o + b], o, b, 0.5, 3)
    assert pooled.shape == (hkv, o)
    np.testing.assert_array_equal(pooled, pooled_ref)
    for g in range(hkv):
        assert idx[g].tolist() == ref[g].tolist() + list(range(o + b, L))
        # the softmax is normalised over the prefix alone
        np.testing.assert_allclose(score[g].sum(), 1.0, rtol=1e-13)
