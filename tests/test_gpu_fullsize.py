"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

Every (batch, head) row of a layer is recomputed by the oracle: the dense steps, the index sets (tie band
reported) and the sparse step, at the first block and at a mid-generation block.  Two protocols are used
for the sparse step: the oracle attending to the rows the GPU gathered (so that an in-band swap does not
pollute the numeric check), and end to end, each side with its own index set."""
import numpy as np
import pytest
import torch

from oracle import sdllm_oracle as orc
from paper_2508_02558_amd import binding as B
from paper_2508_02558_amd import workloads as wl
from tests import parity_util as U

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _full_block(w, samples=None, n_steps=3, block_index=0):
    """samples: (batch, KV head) rows the oracle recomputes; None = every row of the layer."""
    if samples is None:
        samples = [(bi, g) for bi in range(w.batch) for g in range(w.n_kv_heads)]
    print(f"[case] full-size {w.name}: B={w.batch} Hq={w.n_q_heads} Hkv={w.n_kv_heads} L={w.seq_len} "
          f"block {block_index}, {len(samples)} of {w.batch * w.n_kv_heads} rows against the oracle", flush=True)
    inp = wl.make_block_inputs(w, 0, block_index, n_steps, device=DEV)
    o, b = inp["block_off"], w.block
    G = w.group
    shape = U.shape_for(w, block_index)
    k_total, k_pre, k_suf = B.sdllm_retained_count(shape)
    shape = B.make_shape(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                         seq_len=w.seq_len, block_off=o, block_len=b, dtype=U.DT[w.dtype], retention=w.retention,
                         pool_kernel=w.pool_kernel, cache_rows=k_total)   # bench.py's cache layout
    gl = U.GpuLayer(shape, DEV)
    k_full, v_full = inp["k_full"], inp["v_full"]
    total_ties = 0
    worst = 0.0
    for t in range(n_steps):
        state = orc.cache_state(t, 1)
        q = inp["q"][t]
        if state < 2:
            k_full[:, :, o:o + b] = inp["k_blk"][t]
            v_full[:, :, o:o + b] = inp["v_blk"][t]
            assert gl.block_step(t, 1, q, k_full, v_full) == state
            out_host = gl.out.cpu()
            for (bi, g) in samples:
                hs = slice(g * G, (g + 1) * G)
                ref = orc.attention(wl.to_f64(q[bi, hs]), wl.to_f64(k_full[bi, g:g + 1]), wl.to_f64(v_full[bi, g:g + 1]))
                worst = max(worst, U.assert_close(out_host[bi, hs], ref, w.dtype, f"dense step {t} row {(bi, g)}")[0])
            if state == 1:
                idx = gl.idx[:, :, :k_total]
                # properties that hold for every row, whatever the size
                idx64 = idx.long()
                assert bool((idx64[..., 1:] > idx64[..., :-1]).all()), "indices not strictly ascending"
                assert bool(((idx64 >= 0) & (idx64 < w.seq_len)).all())
                assert not bool(((idx64 >= o) & (idx64 < o + b)).any()), "a block position was retained"
                assert bool(((idx64 < o).sum(-1) == k_pre).all()) and bool(((idx64 >= o + b).sum(-1) == k_suf).all())
                ex = idx64[..., None].expand(-1, -1, -1, w.head_dim)
                assert torch.equal(gl.k_cache[:, :, :k_total], torch.gather(k_full, 2, ex))
                assert torch.equal(gl.v_cache[:, :, :k_total], torch.gather(v_full, 2, ex))
                idx_host = idx.cpu().numpy().astype(np.int64)
                for (bi, g) in samples:
                    i_orc, pooled_orc, _ = orc.score_select(wl.to_f64(q[bi, g * G:(g + 1) * G]), wl.to_f64(k_full[bi, g:g + 1]),
                                                            o, b, w.retention, w.pool_kernel)
                    total_ties += U.compare_index_rows(idx_host[bi, g], i_orc[0], pooled_orc[0], w.seq_len, o, b,
                                                       U.ranked_segments(shape))
        else:
            kb, vb = inp["k_blk"][t], inp["v_blk"][t]
            assert gl.block_step(t, 1, q, kb, vb) == 2
            out_host = gl.out.cpu()
            kc_host, vc_host = gl.k_cache[:, :, :k_total].cpu(), gl.v_cache[:, :, :k_total].cpu()
            kb_host, vb_host = kb.cpu(), vb.cpu()
            for (bi, g) in samples:
                hs = slice(g * G, (g + 1) * G)
                kc = torch.cat([kc_host[bi, g:g + 1], kb_host[bi, g:g + 1]], 1)
                vc = torch.cat([vc_host[bi, g:g + 1], vb_host[bi, g:g + 1]], 1)
                ref = orc.attention(wl.to_f64(q[bi, hs]), wl.to_f64(kc), wl.to_f64(vc))
                worst = max(worst, U.assert_close(out_host[bi, hs], ref, w.dtype, f"sparse step {t} row {(bi, g)}")[0])
    print(f"[done] ties in band over the compared rows: {total_ties}; worst max-abs error {worst:.2e}", flush=True)


def test_llada8b_sweep_layer_full_size():
    # the benchmark workload: B=8, 32 MHA heads, prompt 4096 (one layer of it), all 256 rows
    _full_block(wl.WORKLOADS["llada8b_sweep"])


def test_llada8b_sweep_mid_generation_block_full_size():
    # block 5 of 8: prefix 4256, suffix 64 (different tile counts and quotas from block 0), all 256 rows
    _full_block(wl.WORKLOADS["llada8b_sweep"], block_index=5)


def test_llada8b_sweep_block_off_the_tile_grid():
    # a prompt that is not a multiple of the 32-key tile: the block straddles two tiles of the dense step,
    # prefix and suffix tiles are ragged, quotas are odd; batch 2 of the benchmark shape, all 64 rows
    _full_block(wl.WORKLOADS["llada8b_sweep"].scaled(batch=2, prompt=4077), block_index=2)


def test_dream_long_full_size():
    # 28 query / 4 KV heads, prompt 32768, r = 0.25: top-k over 33 248 candidates per row, all 4 rows
    _full_block(wl.WORKLOADS["dream_long"])


def test_dream7b_gen512_full_size():
    # the grouped-query bench workload: B=8, 28 query / 4 KV heads, prompt 4096, 512-token generation
    # (dense step through the shared-tile kernel with key splits, sparse step one workgroup per head), all 32 rows
    _full_block(wl.WORKLOADS["dream7b_gen512"])


@pytest.mark.parametrize("name,block_index", [("llada8b_layer", 0), ("llada8b_layer", 4), ("dream7b_gqa", 0), ("dream7b_gqa", 6)])
def test_end_to_end_with_each_side_using_its_own_index_set(name, block_index):
    # The oracle runs the whole block on its own: its own scores, its own index set, its own cache.  The
    # GPU does the same through sdllm_block_step.  Outputs of every step are compared; the index sets may
    # differ inside the tie band only, and such a swap moves the sparse output by far less than the tolerance.
    w = wl.WORKLOADS[name]
    n_steps = 5
    print(f"[case] own-index end to end {name} block {block_index}", flush=True)
    inp = wl.make_block_inputs(w, 0, block_index, n_steps, device=DEV)
    o, b = inp["block_off"], w.block
    shape = U.shape_for(w, block_index)
    gl = U.GpuLayer(shape, DEV)
    k_full, v_full = inp["k_full"], inp["v_full"]
    caches = [dict() for _ in range(w.batch)]
    ties = differing = 0
    for t in range(n_steps):
        state = orc.cache_state(t, 1)
        q = inp["q"][t]
        if state < 2:
            k_full[:, :, o:o + b] = inp["k_blk"][t]
            v_full[:, :, o:o + b] = inp["v_blk"][t]
            k_in, v_in = k_full, v_full
        else:
            k_in, v_in = inp["k_blk"][t], inp["v_blk"][t]
        assert gl.block_step(t, 1, q, k_in, v_in) == state
        for bi in range(w.batch):
            ref, st = orc.block_step(t, 1, wl.to_f64(q[bi]), wl.to_f64(k_in[bi]), wl.to_f64(v_in[bi]), caches[bi], block_off=o,
                                     block_len=b, r=w.retention, s=w.pool_kernel)
            assert st == state
            U.assert_close(gl.out[bi], ref, w.dtype, f"step {t} (state {state}) batch {bi}")
            if state == 1:
                idx_gpu = gl.idx[bi, :, :gl.k_total].cpu().numpy().astype(np.int64)
                for g in range(w.n_kv_heads):
                    ties += U.compare_index_rows(idx_gpu[g], caches[bi]["idx"][g], caches[bi]["pooled"][g], w.seq_len, o, b,
                                                 U.ranked_segments(shape))
                    differing += int((idx_gpu[g] != caches[bi]["idx"][g]).sum())
                # the oracle's own gather against the GPU's cache wherever the two index sets agree
                same = idx_gpu == caches[bi]["idx"]
                kc = gl.k_cache[bi, :, :gl.k_total].cpu().double().numpy()
                vc = gl.v_cache[bi, :, :gl.k_total].cpu().double().numpy()
                assert (kc[same] == caches[bi]["k"][same]).all() and (vc[same] == caches[bi]["v"][same]).all()
    print(f"[done] ties in band: {ties}; index entries that differ between the two sides: {differing}", flush=True)


def test_gen512_late_block_full_size():
    # 512-token generation after a 4k input: block 13 of 16 has a 4512-token prefix and a 64-token suffix
    w = wl.WORKLOADS["llada8b_gen512"].scaled(batch=2)
    print(f"[case] {w.name} block 13", flush=True)
    inp = wl.make_block_inputs(w, 0, 13, 3, device=DEV)
    o, b = inp["block_off"], w.block
    assert o == 4096 + 13 * 32
    shape = U.shape_for(w, 13)
    gl = U.GpuLayer(shape, DEV)
    q1 = inp["q"][1]
    assert gl.block_step(1, 1, q1, inp["k_full"], inp["v_full"]) == 1
    kt = gl.k_total
    assert kt == (o + 1) // 2 + 32
    for (bi, g) in [(0, 0), (1, 31)]:
        i_orc, pooled_orc, _ = orc.score_select(wl.to_f64(q1[bi, g:g + 1]), wl.to_f64(inp["k_full"][bi, g:g + 1]), o, b,
                                                w.retention, w.pool_kernel)
        U.compare_index_rows(gl.idx[bi, g, :kt].cpu().numpy().astype(np.int64), i_orc[0], pooled_orc[0], w.seq_len, o, b,
                             U.ranked_segments(shape))
    q2, kb, vb = inp["q"][2], inp["k_blk"][2], inp["v_blk"][2]
    assert gl.block_step(2, 1, q2, kb, vb) == 2
    for (bi, g) in [(0, 5), (1, 30)]:
        kc = torch.cat([gl.k_cache[bi, g:g + 1, :kt], kb[bi, g:g + 1]], 1)
        vc = torch.cat([gl.v_cache[bi, g:g + 1, :kt], vb[bi, g:g + 1]], 1)
        U.assert_close(gl.out[bi, g:g + 1], orc.attention(wl.to_f64(q2[bi, g:g + 1]), wl.to_f64(kc), wl.to_f64(vc)), "bf16",
                       f"sparse sample {(bi, g)}")
