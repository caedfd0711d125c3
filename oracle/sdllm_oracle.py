"""CPU oracle for the Sparse-dLLM per-layer hot path (float64, NumPy).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
hot path computes.  It is imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product path, and it shares no code
with the HIP kernels.  Everything is float64; inputs are the same fp32 / bf16
values the GPU sees, widened exactly.

What follows the paper, in its notation (b block length, o block offset, L
sequence length, r retention ratio, s pool kernel size):

  candidates   K_f = Concat[K_{:o}, K_{o+b:}]                   Sec. 3.3, first equation; Alg. 1 steps 2-3
  logits       A = Q_b K_f^T / sqrt(d_k)                        Sec. 3.3, second equation
  aggregation  mean over the block's queries                    Alg. 1 steps 5-6 and the sentence introducing Alg. 1
  smoothing    MaxPool1D(kernel s, padding s/2, stride 1)       Sec. 3.3 third equation; Alg. 1 step 8
  selection    top-k of the pooled scores                       Sec. 3.3 third equation; Alg. 1 steps 9-10
  cache        K_c = K_f[I], V_c = V_f[I]                       Sec. 3.3 fourth equation; Alg. 1 steps 12-14
  reuse        attention over Concat(K_c, K_n), Concat(V_c, V_n) Alg. 3, cache_state == 2
  schedule     cache_state(i) = 2 if i > x, 1 if i == x, else 0 Alg. 2 (x = 1) and Alg. 5

Readings taken where the paper leaves a choice (each is a parameter, the
default is listed first):

  score_mode   "softmax_mean": the logits of each query row are softmax-normalised jointly
               over all candidates, then averaged over the block's queries and the query
               heads of the KV group ("average attention scores").  "logit_mean": the raw
               scaled logits are averaged (Alg. 1 read literally: mean query times K_f^T).
  select_mode  "per_segment": prefix and suffix are pooled and ranked separately, each
               keeping its own quota.  "joint": the concatenated candidate array is pooled
               (the window crosses the prefix/suffix seam) and ranked as one (Alg. 1 literal).
  k_rounding   "ceil" (quota ceil(r*n)) or "floor" (Alg. 1 step 9).
  ties         the lower position wins; retained positions are reported ascending.
  GQA          query head h reads KV head h // G; one index set per (batch, KV head).
  evict_scope  "bidirectional" (Alg. 1) or "prefix_only" (Alg. 4, the prefix-sparse ablation:
               only K_{:o} is scored and ranked, every suffix entry is kept).

Parity pins (tests/test_oracle_*.py): brute-force loops on tiny inputs, r = 1
reproducing dense attention, closed forms (zero queries, one-hot values),
library routines on special cases (torch max_pool1d / topk / SDPA,
scipy maximum_filter1d), hand-worked 8-token selections under tests/golden/.
Parity unpinned: nothing in the paper prints a numerical example of its own,
so agreement with the authors' implementation on real model activations
(accuracy / throughput tables) cannot be checked here.
"""
from __future__ import annotations

import math
from typing import Tuple

import numpy as np

SOFTMAX_MEAN = "softmax_mean"
LOGIT_MEAN = "logit_mean"
PER_SEGMENT = "per_segment"
JOINT = "joint"
CEIL = "ceil"
FLOOR = "floor"
MAX_POOL = "max"
AVG_POOL = "avg"
BIDIRECTIONAL = "bidirectional"
PREFIX_ONLY = "prefix_only"


# ----------------------------------------------------------------------------- schedule
def cache_state(step_in_block: int, delay: int = 1) -> int:
    """Alg. 5 (Alg. 2 is delay == 1): 0 = full attention, 1 = update cache, 2 = reuse cache."""
    if step_in_block > delay:
        return 2
    if step_in_block == delay:
        return 1
    return 0


# ----------------------------------------------------------------------------- candidates
def candidate_positions(seq_len: int, block_off: int, block_len: int) -> np.ndarray:
    """Absolute positions of K_f's rows: [0, o) followed by [o+b, L)  (Sec. 3.3, first equation)."""
    return np.concatenate([np.arange(0, block_off), np.arange(block_off + block_len, seq_len)])


def retained_count(n: int, r: float, k_rounding: str = CEIL) -> int:
    """Number of entries kept out of n at retention ratio r (Alg. 1 step 9 for "floor").

    r*n is evaluated in double precision with a 1e-9 guard so that 0.7*10 gives 7 on both
    roundings instead of falling to the wrong side of the integer.
    """
    x = float(r) * n
    k = math.ceil(x - 1e-9) if k_rounding == CEIL else math.floor(x + 1e-9)
    return max(0, min(n, int(k)))


# ----------------------------------------------------------------------------- scoring
def saliency_logits(q_blk: np.ndarray, k_full: np.ndarray, block_off: int, block_len: int,
                    scale: float | None = None) -> np.ndarray:
    """A[h, i, c] = <Q_b[h, i], K_f[g(h), c]> * scale for every candidate c  (Sec. 3.3, second equation).

    q_blk [Hq, b, d], k_full [Hkv, L, d] -> [Hq, b, N].
    """
    hq, b, d = q_blk.shape
    hkv, L, _ = k_full.shape
    grp = hq // hkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    cand = candidate_positions(L, block_off, block_len)
    out = np.empty((hq, b, cand.size), dtype=np.float64)
    for h in range(hq):
        k_f = k_full[h // grp][cand]                      # [N, d]
        out[h] = (q_blk[h] @ k_f.T) * scale
    return out


def saliency_score(q_blk: np.ndarray, k_full: np.ndarray, block_off: int, block_len: int,
                   score_mode: str = SOFTMAX_MEAN, scale: float | None = None) -> np.ndarray:
    """Per-candidate importance before pooling, one row per KV head: [Hkv, N]."""
    hq = q_blk.shape[0]
    hkv = k_full.shape[0]
    grp = hq // hkv
    a = saliency_logits(q_blk, k_full, block_off, block_len, scale)     # [Hq, b, N]
    if score_mode == SOFTMAX_MEAN:
        if a.shape[-1] == 0:
            w = a
        else:
            a = a - a.max(axis=-1, keepdims=True)
            e = np.exp(a)
            w = e / e.sum(axis=-1, keepdims=True)
    elif score_mode == LOGIT_MEAN:
        w = a
    else:
        raise ValueError(score_mode)
    per_head = w.mean(axis=1)                                           # mean over block queries
    return per_head.reshape(hkv, grp, -1).mean(axis=1)                  # mean over the group's heads


# ----------------------------------------------------------------------------- pooling
def pool_1d(x: np.ndarray, s: int, kind: str = MAX_POOL) -> np.ndarray:
    """Stride-1 pooling of a 1-D array with window s (odd), same length as the input.

    Max pooling pads with -inf (Alg. 1 step 8).  Average pooling (the paper's AvgPool
    ablation) pads with zeros and divides by s, the usual AvgPool1D convention.
    """
    if s < 1 or s % 2 == 0:
        raise ValueError("pool kernel must be odd and >= 1")
    n = x.shape[0]
    half = (s - 1) // 2
    out = np.empty(n, dtype=np.float64)
    for c in range(n):
        lo, hi = max(0, c - half), min(n, c + half + 1)
        if kind == MAX_POOL:
            out[c] = x[lo:hi].max()
        else:
            out[c] = x[lo:hi].sum() / s
    return out


def pool_scores(score: np.ndarray, n_pre: int, s: int, select_mode: str = PER_SEGMENT,
                kind: str = MAX_POOL) -> np.ndarray:
    """Pool one candidate-indexed score row [N]; the window stops at the prefix/suffix seam
    in "per_segment" mode and runs across it in "joint" mode."""
    if select_mode == JOINT:
        return pool_1d(score, s, kind)
    return np.concatenate([pool_1d(score[:n_pre], s, kind), pool_1d(score[n_pre:], s, kind)])


# ----------------------------------------------------------------------------- selection
def top_k_lowest_position(values: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest values, ties going to the lower index; returned ascending."""
    n = values.shape[0]
    order = sorted(range(n), key=lambda c: (-values[c], c))
    return np.array(sorted(order[:k]), dtype=np.int64)


def select_indices(pooled: np.ndarray, seq_len: int, block_off: int, block_len: int, r: float,
                   select_mode: str = PER_SEGMENT, k_rounding: str = CEIL) -> Tuple[np.ndarray, int]:
    """Retained absolute positions (ascending) for one pooled row [N] and the number of
    them that lie in the prefix."""
    n_pre = block_off
    n_suf = seq_len - block_off - block_len
    cand = candidate_positions(seq_len, block_off, block_len)
    if select_mode == PER_SEGMENT:
        k_pre = retained_count(n_pre, r, k_rounding)
        k_suf = retained_count(n_suf, r, k_rounding)
        keep_pre = top_k_lowest_position(pooled[:n_pre], k_pre)
        keep_suf = top_k_lowest_position(pooled[n_pre:], k_suf) + n_pre
        keep = np.concatenate([keep_pre, keep_suf])
    elif select_mode == JOINT:
        keep = top_k_lowest_position(pooled, retained_count(n_pre + n_suf, r, k_rounding))
    else:
        raise ValueError(select_mode)
    keep = keep.astype(np.int64)
    return cand[keep], int((keep < n_pre).sum())


def score_select(q_blk: np.ndarray, k_full: np.ndarray, block_off: int, block_len: int, r: float,
                 s: int, score_mode: str = SOFTMAX_MEAN, select_mode: str = PER_SEGMENT,
                 k_rounding: str = CEIL, scale: float | None = None, pool_kind: str = MAX_POOL,
                 evict_scope: str = BIDIRECTIONAL):
    """Alg. 1 (or Alg. 4 for evict_scope == "prefix_only") up to the index set.
    q_blk [Hq,b,d], k_full [Hkv,L,d].

    Returns (idx [Hkv, k] int64 ascending absolute positions, pooled [Hkv, N'], score [Hkv, N'])
    where N' is the number of scored candidates (N, or N_pre for prefix-only eviction).
    """
    hkv, L, _ = k_full.shape
    if evict_scope == PREFIX_ONLY:
        # Alg. 4: K_f = K_{:o} is scored and ranked; K_r = K_{o+b:} is appended whole
        k_prefix_and_block = k_full[:, :block_off + block_len]
        idx, pooled, score = score_select(q_blk, k_prefix_and_block, block_off, block_len, r, s, score_mode,
                                          PER_SEGMENT, k_rounding, scale, pool_kind)
        suffix = np.arange(block_off + block_len, L, dtype=np.int64)
        idx = np.concatenate([idx, np.broadcast_to(suffix, (hkv, suffix.size))], axis=1)
        return idx, pooled, score
    score = saliency_score(q_blk, k_full, block_off, block_len, score_mode, scale)
    pooled = np.stack([pool_scores(score[g], block_off, s, select_mode, pool_kind) for g in range(hkv)])
    idx = np.stack([select_indices(pooled[g], L, block_off, block_len, r, select_mode, k_rounding)[0]
                    for g in range(hkv)])
    return idx, pooled, score


# ----------------------------------------------------------------------------- cache
def compact_kv(k_full: np.ndarray, v_full: np.ndarray, idx: np.ndarray):
    """K_c = K[idx], V_c = V[idx] per KV head (Sec. 3.3, fourth equation).  idx [Hkv, k]."""
    hkv = k_full.shape[0]
    k_c = np.stack([k_full[g][idx[g]] for g in range(hkv)])
    v_c = np.stack([v_full[g][idx[g]] for g in range(hkv)])
    return k_c, v_c


# ----------------------------------------------------------------------------- attention
def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Unmasked softmax attention.  q [Hq, n, d], k/v [Hkv, m, d] -> [Hq, n, d]."""
    hq, n, d = q.shape
    hkv = k.shape[0]
    grp = hq // hkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    out = np.empty((hq, n, v.shape[-1]), dtype=np.float64)
    for h in range(hq):
        g = h // grp
        a = (q[h] @ k[g].T) * scale
        a = a - a.max(axis=-1, keepdims=True)
        p = np.exp(a)
        p = p / p.sum(axis=-1, keepdims=True)
        out[h] = p @ v[g]
    return out


def sparse_attention(q_blk, k_cache, v_cache, k_blk, v_blk, scale=None) -> np.ndarray:
    """Alg. 3, cache_state == 2: keys/values are Concat(K_c, K_n) / Concat(V_c, V_n), no mask."""
    k = np.concatenate([k_cache, k_blk], axis=1)
    v = np.concatenate([v_cache, v_blk], axis=1)
    return attention(q_blk, k, v, scale)


def dense_block_attention(q_blk, k_full, v_full, scale=None) -> np.ndarray:
    """The block's rows of full bidirectional attention (cache_state 0 and 1)."""
    return attention(q_blk, k_full, v_full, scale)


# ----------------------------------------------------------------------------- one block
def block_step(step_in_block: int, delay: int, q_blk, k_in, v_in, cache, *, block_off: int,
               block_len: int, r: float, s: int, score_mode=SOFTMAX_MEAN, select_mode=PER_SEGMENT,
               k_rounding=CEIL, scale=None, pool_kind=MAX_POOL, evict_scope=BIDIRECTIONAL):
    """One denoising step of one layer for one batch element (Alg. 2/5 -> Alg. 3 -> Alg. 1).

    States 0/1: k_in, v_in are the full-sequence K, V [Hkv, L, d]; the output is the block's
    rows of dense attention; state 1 also rebuilds `cache` (a dict) from this step's tensors.
    State 2: k_in, v_in are the block's K_n, V_n [Hkv, b, d]; attention runs over the cache
    plus the block.  Returns (out, state).
    """
    state = cache_state(step_in_block, delay)
    if state in (0, 1):
        out = dense_block_attention(q_blk, k_in, v_in, scale)
        if state == 1:
            idx, pooled, score = score_select(q_blk, k_in, block_off, block_len, r, s, score_mode,
                                              select_mode, k_rounding, scale, pool_kind, evict_scope)
            k_c, v_c = compact_kv(k_in, v_in, idx)
            cache.clear()
            cache.update(k=k_c, v=v_c, idx=idx, pooled=pooled, score=score)
    else:
        out = sparse_attention(q_blk, cache["k"], cache["v"], k_in, v_in, scale)
    return out, state
