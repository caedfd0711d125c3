"""Seeded synthetic inputs shaped like the paper's decoding workloads.

This module only draws random tensors and plants structure in them (salient
key directions, step-to-step correlation).  It holds none of the method's
arithmetic: no scoring, pooling, selection or attention.  Both the CPU oracle's
tests and the HIP path's tests/benchmark take their inputs from here, so the
two sides always see identical values.

Shapes follow the paper's experimental settings (block length 32, 32 denoising
steps per block of a 256-token generation, retention ratio 0.5, pool kernel 3,
seed 2025; Experiment/Setup and the benchmark-configuration table in the
appendix).  Head counts and head dimensions are those of LLaDA-8B (32 MHA
heads, d=128) and Dream-7B (28 query / 4 KV heads, d=128).  The "vertical"
attention pattern the paper observes (a few pivotal keys that stay salient for
every query and every step; Observations section) is imitated by scaling a
small fraction of key rows along a direction all queries are biased towards.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import torch

PAPER_SEED = 2025  # Experiment/Setup: fixed random seed 2025


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the benchmark's configuration list
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" | "bf16"
    prompt: int
    gen: int
    block: int
    steps_per_block: int
    retention: float
    pool_kernel: int
    n_layers: int
    salient_frac: float   # fraction of positions carrying a salient key
    salient_gain: float   # salient key = gain * ||k|| * direction
    sink: int             # leading positions that are all salient
    query_bias: float     # queries = N(0,1) + query_bias * direction
    ar_rho: float         # AR(1) correlation of per-step tensors

    @property
    def seq_len(self) -> int:
        return self.prompt + self.gen

    @property
    def n_blocks(self) -> int:
        return self.gen // self.block

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def block_off(self, block_index: int) -> int:
        return self.prompt + block_index * self.block

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def scaled(self, **kw) -> "Workload":
        """A copy with some fields changed (reduced sizes for quick tests)."""
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    # prefix 64 + block 32 + suffix 64; four planted salient prefix keys
    "tiny": Workload("tiny", 0, 1, 2, 2, 64, "f32", 64, 96, 32, 4, 0.5, 3, 1,
                     0.0, 4.0, 0, 0.0, 0.9),
    "llada8b_layer": Workload("llada8b_layer", 1, 1, 32, 32, 128, "bf16", 1024, 256, 32, 32,
                              0.5, 3, 1, 0.02, 3.0, 0, 0.5, 0.9),
    "dream7b_gqa": Workload("dream7b_gqa", 2, 1, 28, 4, 128, "bf16", 4096, 256, 32, 32,
                            0.5, 3, 1, 0.02, 3.0, 0, 0.5, 0.9),
    "llada8b_sweep": Workload("llada8b_sweep", 3, 8, 32, 32, 128, "bf16", 4096, 256, 32, 32,
                              0.5, 3, 32, 0.02, 3.0, 0, 0.5, 0.9),
    "dream_long": Workload("dream_long", 4, 1, 28, 4, 128, "bf16", 32768, 512, 32, 32,
                           0.25, 3, 1, 0.01, 3.0, 64, 0.5, 0.9),
    # second shape family of the paper's runs: 512 denoising steps for a 512-token generation
    # (16 blocks of 32, still 32 steps per block) after a 4k input (HumanEval / LongBench settings)
    "llada8b_gen512": Workload("llada8b_gen512", 5, 8, 32, 32, 128, "bf16", 4096, 512, 32, 32,
                               0.5, 3, 32, 0.02, 3.0, 0, 0.5, 0.9),
    "dream7b_gen512": Workload("dream7b_gen512", 6, 8, 28, 4, 128, "bf16", 4096, 512, 32, 32,
                               0.5, 3, 28, 0.02, 3.0, 0, 0.5, 0.9),
}
WORKLOAD_LIST: List[Workload] = sorted(WORKLOADS.values(), key=lambda w: w.index)


def _generator(w: Workload, layer: int, block_index: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(PAPER_SEED + 1000 * w.index + layer + 100_003 * block_index + 7_000_003 * stream)
    return g


def _randn(shape, g: torch.Generator, device) -> torch.Tensor:
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def salient_positions(w: Workload, layer: int, block_index: int) -> torch.Tensor:
    """Positions (outside the current block) that carry a salient key; always on the host."""
    g = _generator(w, layer, block_index, 1, "cpu")
    L, o, b = w.seq_len, w.block_off(block_index), w.block
    if w.name == "tiny":
        # four prefix positions, pairwise at least 3 apart, away from the edges
        slots = torch.randperm((o - 2) // 3, generator=g)[:4]
        return (slots * 3 + 1).sort().values
    mask = torch.rand(L, generator=g) < w.salient_frac
    mask[:w.sink] = True
    mask[o:o + b] = False
    return mask.nonzero().flatten()


def make_block_inputs(w: Workload, layer: int = 0, block_index: int = 0, n_steps: int | None = None,
                      device="cpu") -> dict:
    """All tensors one (layer, block) of the decode loop consumes.

    Returns a dict with
      k_full, v_full : [B, Hkv, L, d]  candidate K/V, fixed within the block; the rows of
                       the current block hold the step-0 block K/V (callers overwrite them
                       with k_blk[t] / v_blk[t] for the full-sequence steps t)
      q       : [T, B, Hq, b, d]   block queries per denoising step
      k_blk, v_blk : [T, B, Hkv, b, d] block K/V per denoising step
      direction : [B, Hkv, d] unit vector the salient keys and the queries share (fp32)
      salient : 1-D int64 host tensor of salient positions
    All of q/k/v are in the workload's dtype (values already rounded to it).
    """
    T = w.steps_per_block if n_steps is None else n_steps
    B, Hq, Hkv, d, L, b = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.seq_len, w.block
    o = w.block_off(block_index)
    G = w.group
    g_static = _generator(w, layer, block_index, 2, device)
    g_steps = _generator(w, layer, block_index, 3, device)

    k_full = _randn((B, Hkv, L, d), g_static, device)
    v_full = _randn((B, Hkv, L, d), g_static, device)
    direction = _randn((B, Hkv, d), g_static, device)
    direction = direction / direction.norm(dim=-1, keepdim=True)

    rho = w.ar_rho
    innov = (1.0 - rho * rho) ** 0.5

    def ar1(shape):
        out = torch.empty((T,) + shape, device=device, dtype=torch.float32)
        z = _randn(shape, g_steps, device)
        out[0] = z
        for t in range(1, T):
            z = rho * z + innov * _randn(shape, g_steps, device)
            out[t] = z
        return out

    q = ar1((B, Hq, b, d))
    k_blk = ar1((B, Hkv, b, d))
    v_blk = ar1((B, Hkv, b, d))
    # every query head of a KV group leans towards that group's direction
    q = q + w.query_bias * direction.repeat_interleave(G, dim=1)[None, :, :, None, :]

    sal = salient_positions(w, layer, block_index)
    sal_dev = sal.to(device)
    if sal.numel():
        if w.name == "tiny":
            # align with the normalised mean block query of the update step (step 1), per head
            t_upd = min(1, T - 1)
            m = q[t_upd].mean(dim=2)                       # [B, Hq, d]  (MHA: Hq == Hkv)
            m = m / m.norm(dim=-1, keepdim=True)
            dirs = m
        else:
            dirs = direction
        norms = k_full[:, :, sal_dev, :].norm(dim=-1, keepdim=True)       # [B,Hkv,S,1]
        k_full[:, :, sal_dev, :] = w.salient_gain * norms * dirs[:, :, None, :]

    dt = w.torch_dtype
    k_full = k_full.to(dt)
    v_full = v_full.to(dt)
    q, k_blk, v_blk = q.to(dt), k_blk.to(dt), v_blk.to(dt)
    k_full[:, :, o:o + b, :] = k_blk[0]
    v_full[:, :, o:o + b, :] = v_blk[0]
    return dict(k_full=k_full, v_full=v_full, q=q, k_blk=k_blk, v_blk=v_blk,
                direction=direction, salient=sal, block_off=o)


def to_f64(t: torch.Tensor):
    """Exact widening of fp32/bf16 values to a float64 NumPy array (for the CPU oracle)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
