"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI on seeded
workloads and compare with the float64 oracle under the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

from oracle import sdllm_oracle as orc
from paper_2508_02558_amd import binding as B
from paper_2508_02558_amd import workloads as wl

# tolerances of the attention output against the float64 oracle
TOL = {"bf16": dict(max_abs=2e-2, mean_abs=2e-3),     # bf16 tensors, fp32 accumulation
       "f32": dict(max_abs=1e-5, mean_abs=1e-6)}
TIE_BAND = 1e-4   # relative half-width of the band around the k-th pooled value counted as ties

DT = {"bf16": B.SDLLM_BF16, "f32": B.SDLLM_F32}
SCORE_MODES = {B.SDLLM_SOFTMAX_MEAN: orc.SOFTMAX_MEAN, B.SDLLM_LOGIT_MEAN: orc.LOGIT_MEAN}
SELECT_MODES = {B.SDLLM_PER_SEGMENT: orc.PER_SEGMENT, B.SDLLM_JOINT: orc.JOINT}
ROUNDINGS = {B.SDLLM_CEIL: orc.CEIL, B.SDLLM_FLOOR: orc.FLOOR}
POOLS = {B.SDLLM_MAX_POOL: orc.MAX_POOL, B.SDLLM_AVG_POOL: orc.AVG_POOL}


def shape_for(w: wl.Workload, block_index: int = 0, **modes):
    return B.make_shape(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                        seq_len=w.seq_len, block_off=w.block_off(block_index), block_len=w.block,
                        dtype=DT[w.dtype], retention=w.retention, pool_kernel=w.pool_kernel, **modes)


def assert_close(out_gpu: torch.Tensor, ref: np.ndarray, dtype: str, what: str = ""):
    got = out_gpu.detach().to("cpu").to(torch.float64).numpy()
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), what
    err = np.abs(got - ref)
    tol = TOL[dtype]
    assert err.max() <= tol["max_abs"], f"{what}: max-abs {err.max():.3e} > {tol['max_abs']}"
    assert err.mean() <= tol["mean_abs"], f"{what}: mean-abs {err.mean():.3e} > {tol['mean_abs']}"
    return float(err.max()), float(err.mean())


def compare_index_rows(idx_gpu: np.ndarray, idx_orc: np.ndarray, pooled_orc: np.ndarray, seq_len: int,
                       block_off: int, block_len: int, segments) -> int:
    """One (batch, KV head) row.  `segments` lists (cand_begin, cand_len, k) of every ranked segment;
    k < 0 marks candidates kept unconditionally.  Outside the tie band the two index sets must be
    identical; inside it the GPU may pick any band member.  Returns the number of band members."""
    cand = orc.candidate_positions(seq_len, block_off, block_len)
    assert idx_gpu.shape == idx_orc.shape
    assert (np.diff(idx_gpu) > 0).all(), "GPU indices not strictly ascending"
    assert np.isin(idx_gpu, cand).all(), "GPU index outside the candidate set"
    ties = 0
    for begin, length, k in segments:
        pos = cand[begin:begin + length]
        g = idx_gpu[np.isin(idx_gpu, pos)]
        o = idx_orc[np.isin(idx_orc, pos)]
        assert g.size == o.size == (length if k < 0 else k), (g.size, o.size, k)
        if k <= 0 or k >= length:
            assert (g == o).all()
            continue
        vals = pooled_orc[begin:begin + length]
        tau = np.sort(vals)[::-1][k - 1]
        band = pos[np.abs(vals - tau) <= TIE_BAND * abs(tau)]
        ties += band.size
        g_out, o_out = g[~np.isin(g, band)], o[~np.isin(o, band)]
        assert g_out.size == o_out.size and (g_out == o_out).all(), "index sets differ outside the tie band"
    return ties


def ranked_segments(shape) -> list:
    n_pre = shape.block_off
    n_suf = shape.seq_len - shape.block_off - shape.block_len
    kt, kp, ks = B.sdllm_retained_count(shape)
    if shape.evict_scope == B.SDLLM_EVICT_PREFIX_ONLY:
        return [(0, n_pre, kp), (n_pre, n_suf, -1)]
    if shape.select_mode == B.SDLLM_PER_SEGMENT:
        return [(0, n_pre, kp), (n_pre, n_suf, ks)]
    return [(0, n_pre + n_suf, kt)]


def oracle_score_select(shape, q_blk: torch.Tensor, k_full: torch.Tensor, heads=None):
    """Oracle index sets for every batch element (optionally only some KV heads).
    q_blk [B,Hq,b,d], k_full [B,Hkv,L,d] -> idx [B,Hkv',k], pooled [B,Hkv',N], score [B,Hkv',N]."""
    G = shape.n_q_heads // shape.n_kv_heads
    idx, pooled, score = [], [], []
    for b in range(q_blk.shape[0]):
        q = wl.to_f64(q_blk[b]); k = wl.to_f64(k_full[b])
        if heads is not None:
            k = k[heads]
            q = np.concatenate([q[g * G:(g + 1) * G] for g in heads])
        scale = shape.softmax_scale if shape.softmax_scale > 0 else None
        scope = orc.PREFIX_ONLY if shape.evict_scope == B.SDLLM_EVICT_PREFIX_ONLY else orc.BIDIRECTIONAL
        i, p, s = orc.score_select(q, k, shape.block_off, shape.block_len, shape.retention, shape.pool_kernel,
                                   SCORE_MODES[shape.score_mode], SELECT_MODES[shape.select_mode],
                                   ROUNDINGS[shape.k_rounding], scale, POOLS[shape.pool_mode], scope)
        idx.append(i); pooled.append(p); score.append(s)
    return np.stack(idx), np.stack(pooled), np.stack(score)


class GpuLayer:
    """Device buffers of one layer and thin calls into the binding."""

    def __init__(self, shape, device="cuda"):
        self.shape = shape
        self.dev = device
        s = shape
        self.tdtype = torch.bfloat16 if s.dtype == B.SDLLM_BF16 else torch.float32
        self.k_total, self.k_pre, self.k_suf = B.sdllm_retained_count(s)
        self.n_cand = s.seq_len - s.block_len
        cache_rows = s.cache_stride[1] // s.head_dim if s.cache_stride[1] else max(1, self.k_total)
        self.k_cache = torch.zeros(s.batch, s.n_kv_heads, cache_rows, s.head_dim, dtype=self.tdtype, device=device)
        self.v_cache = torch.zeros_like(self.k_cache)
        self.idx = torch.full((s.batch, s.n_kv_heads, max(1, self.k_total)), -1, dtype=torch.int32, device=device)
        self.out = torch.zeros(s.batch, s.n_q_heads, s.block_len, s.head_dim, dtype=self.tdtype, device=device)
        nbytes = max(B.sdllm_workspace_bytes(s, B.SDLLM_OP_BLOCK_STEP),
                     B.sdllm_workspace_bytes(s, B.SDLLM_OP_SPARSE_ATTN, self.n_cand))
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)

    def score_select(self, q, k_full, want_scores=True):
        s = self.shape
        pooled = score = None
        if want_scores:
            pooled = torch.full((s.batch, s.n_kv_heads, max(1, self.n_cand)), float("nan"), device=self.dev)
            score = torch.full_like(pooled, float("nan"))
        B.sdllm_score_select(s, q, k_full, self.idx, pooled, score, self.ws)
        torch.cuda.synchronize()
        return self.idx[:, :, :self.k_total].cpu().numpy().astype(np.int64), pooled, score

    def compact(self, k_full, v_full, idx=None):
        B.sdllm_compact_kv(self.shape, k_full, v_full, self.idx if idx is None else idx, self.k_cache, self.v_cache)

    def sparse_attn(self, q, k_blk, v_blk, n_cached=None, k_cache=None, v_cache=None):
        n = self.k_total if n_cached is None else n_cached
        B.sdllm_sparse_attn(self.shape, q, self.k_cache if k_cache is None else k_cache,
                            self.v_cache if v_cache is None else v_cache, n, k_blk, v_blk, self.out, self.ws)
        torch.cuda.synchronize()
        return self.out

    def block_step(self, step, delay, q, k_in, v_in):
        st = B.sdllm_block_step(self.shape, step, delay, q, k_in, v_in, self.idx, self.k_cache, self.v_cache,
                                self.out, self.ws)
        torch.cuda.synchronize()
        return st


def oracle_attention_batch(q, k, v, scale=None):
    """q [B,Hq,n,d], k/v [B,Hkv,m,d] torch tensors -> float64 [B,Hq,n,d]."""
    return np.stack([orc.attention(wl.to_f64(q[b]), wl.to_f64(k[b]), wl.to_f64(v[b]), scale)
                     for b in range(q.shape[0])])
