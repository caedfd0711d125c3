#!/usr/bin/env python3
"""Benchmark of the Sparse-dLLM hot path on one MI355X.

A "step" is one decoding block of the whole workload: every layer runs the 32 denoising steps of
one block through sdllm_block_step (1 dense step, 1 dense + score/select/compact step, 30 sparse
steps at the paper's settings), in model order (for each denoising step, every layer).  All inputs
are synthetic, generated on the device before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llada8b_sweep] [--layers N]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E


def attn_bytes(batch, hq, hkv, d, n_keys, nq, esize):
    """Algorithmic bytes of one block-attention launch: K and V rows read once, Q in, O out."""
    return 2 * batch * hkv * n_keys * d * esize + 2 * batch * hq * nq * d * esize


def measured_traffic(workload: str, default_config: bool):
    """HBM bytes per sparse-attention launch as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE runs scaled
    by a plain copy).  Hardware counters cannot be read from inside this process, so the figure is the
    one stored in the committed counter summary of the same command line; it is only reported when this
    run uses the workload's own batch size and block index (what the summary was taken on)."""
    rel = os.path.join("profiles", f"hbm_traffic_{workload}.txt")
    if default_config:
        try:
            for line in open(os.path.join(ROOT, rel)):
                if line.startswith("traffic_bytes_per_launch[attn_mfma_bf16_kernel<2>]"):
                    return float(line.split("=")[1]), f"stored rocprofv3 --pmc summary {rel} (not measured in this run)"
        except OSError:
            pass
    return None, None


def cpu_baseline(w, inp0, n_batch):
    """The float64 oracle on one layer's block (all denoising steps) for `n_batch` batch elements, once
    with the BLAS thread pool as the box gives it and once pinned to one thread; the faster of the two is
    the reported baseline (the 32-row GEMMs of this path do not always gain from more threads)."""
    from threadpoolctl import threadpool_info, threadpool_limits

    from oracle import sdllm_oracle as orc
    from paper_2508_02558_amd import workloads as wl

    o, b = inp0["block_off"], w.block

    def run(batch_elems):
        t0 = time.perf_counter()
        for bi in range(batch_elems):
            k_full = wl.to_f64(inp0["k_full"][bi])
            v_full = wl.to_f64(inp0["v_full"][bi])
            cache = {}
            for t in range(w.steps_per_block):
                q = wl.to_f64(inp0["q"][t, bi])
                if orc.cache_state(t, 1) < 2:
                    orc.block_step(t, 1, q, k_full, v_full, cache, block_off=o, block_len=b, r=w.retention, s=w.pool_kernel)
                else:
                    orc.block_step(t, 1, q, wl.to_f64(inp0["k_blk"][t, bi]), wl.to_f64(inp0["v_blk"][t, bi]), cache,
                                   block_off=o, block_len=b, r=w.retention, s=w.pool_kernel)
        return time.perf_counter() - t0

    blas = [p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"]
    pool = max(blas) if blas else 1
    dt_all = run(n_batch)
    with threadpool_limits(limits=1, user_api="blas"):
        dt_one = run(n_batch)
    # one sdllm_block_step call covers the whole batch of one layer for one denoising step
    calls_equiv = w.steps_per_block * n_batch / w.batch
    runs = {"all_blas_threads": {"value": calls_equiv / dt_all, "cores": pool, "seconds": dt_all},
            "one_thread": {"value": calls_equiv / dt_one, "cores": 1, "seconds": dt_one}}
    best = max(runs.values(), key=lambda r: r["value"])
    return {
        "value": best["value"], "unit": "block-steps/s per layer", "cores": best["cores"], "kind": "oracle",
        "host_cores": os.cpu_count(),
        "sample": f"one layer, {n_batch} of {w.batch} batch elements, all {w.steps_per_block} denoising steps of one block, "
                  f"scaled to the full batch; run twice ({dt_all:.1f} s with {pool} BLAS threads, {dt_one:.1f} s with one), "
                  f"the faster one reported",
        "runs": runs,
    }


def quick_workload(name: str, dev: str, n_sets: int = 32, reps: int = 3):
    """Short event-timed sweeps of another configuration of the workload list: one layer call per buffer
    set, rotated over n_sets distinct sets so that the last-level cache cannot serve re-reads."""
    import torch

    from paper_2508_02558_amd import binding as B
    from paper_2508_02558_amd import workloads as wl

    w = wl.WORKLOADS[name]
    o, b = w.block_off(0), w.block
    esize = 2 if w.dtype == "bf16" else 4
    kw = dict(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, seq_len=w.seq_len,
              block_off=o, block_len=b, dtype=B.SDLLM_BF16 if w.dtype == "bf16" else B.SDLLM_F32, retention=w.retention,
              pool_kernel=w.pool_kernel)
    k_total, _, _ = B.sdllm_retained_count(B.make_shape(**kw))
    shape = B.make_shape(cache_rows=max(1, k_total), **kw)
    ws = torch.empty(B.sdllm_workspace_bytes(shape, B.SDLLM_OP_BLOCK_STEP), dtype=torch.uint8, device=dev)
    sets = []
    for i in range(n_sets):
        inp = wl.make_block_inputs(w, i, 0, 3, device=dev)
        td = w.torch_dtype
        sets.append(dict(inp, k_cache=torch.zeros(w.batch, w.n_kv_heads, max(1, k_total), w.head_dim, dtype=td, device=dev),
                         v_cache=torch.zeros(w.batch, w.n_kv_heads, max(1, k_total), w.head_dim, dtype=td, device=dev),
                         idx=torch.zeros(w.batch, w.n_kv_heads, max(1, k_total), dtype=torch.int32, device=dev),
                         out=torch.zeros(w.batch, w.n_q_heads, b, w.head_dim, dtype=td, device=dev)))

    def sweep(step):
        for st in sets:
            k_in, v_in = (st["k_blk"][step], st["v_blk"][step]) if step >= 2 else (st["k_full"], st["v_full"])
            B.sdllm_block_step(shape, step, 1, st["q"][step], k_in, v_in, st["idx"], st["k_cache"], st["v_cache"], st["out"], ws)

    def timed(step):
        """(eager, graph): microseconds per layer call with eager launches and as a replayed HIP graph.  The
        calls of these shapes take 10-40 us of GPU time, which two or three kernel launches through Python do
        not always keep ahead of; the replayed graph shows the GPU time, the eager figure what this harness gets."""
        sweep(step)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            sweep(step)
        e1.record()
        torch.cuda.synchronize()
        eager = 1e3 * e0.elapsed_time(e1) / (reps * n_sets)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            sweep(step)
        graph.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        return eager, 1e3 * e0.elapsed_time(e1) / (reps * n_sets)

    (upd_e, upd), (dense_e, dense), (sparse_e, sparse) = timed(1), timed(0), timed(2)   # the update step first: it fills the caches
    bytes_sparse = attn_bytes(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, k_total + b, b, esize)
    T = w.steps_per_block
    return {"shape": f"B={w.batch}, Hq={w.n_q_heads}, Hkv={w.n_kv_heads}, d={w.head_dim}, prompt {w.prompt}, gen {w.gen}, "
                     f"r={w.retention}, retained {k_total}",
            "launch_mode": "hip graph replay (eager figures alongside)",
            "sparse_attn_us": sparse, "dense_block_attn_us": dense, "cache_update_step_us": upd,
            "eager_launches": {"sparse_attn_us": sparse_e, "dense_block_attn_us": dense_e, "cache_update_step_us": upd_e},
            "sparse_attn_algorithmic_bytes": bytes_sparse,
            "sparse_attn_hbm_frac": bytes_sparse / (sparse * 1e-6) / 1e9 / HBM_PEAK_GBS,
            "block_steps_per_s_per_layer": T / ((dense + upd + (T - 2) * sparse) * 1e-6),
            "buffer_sets": n_sets, "timed_sweeps": reps}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llada8b_sweep")
    ap.add_argument("--layers", type=int, default=0, help="override the workload's layer count")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (batch sweep)")
    ap.add_argument("--block-index", type=int, default=0, help="which decoding block of the generation to run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="replay the block as a captured HIP graph (removes host launch cost; matters for batch-1 shapes)")
    ap.add_argument("--cpu-batch", type=int, default=3, help="batch elements the oracle baseline runs")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the short sweeps of the other configurations")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (no sharding, no collectives); run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    from paper_2508_02558_amd import binding as B
    from paper_2508_02558_amd import workloads as wl

    B.load()   # fails loudly when the HIP library has not been built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)

    w = wl.WORKLOADS[args.workload]
    if args.batch > 0:
        w = w.scaled(batch=args.batch)
    n_layers = args.layers if args.layers > 0 else w.n_layers
    # one-layer workloads are rotated over 32 distinct buffer sets so that re-reads cannot be
    # served by the 256 MB last-level cache
    if n_layers == 1 and args.layers == 0:
        n_layers = 32
    T = w.steps_per_block
    o, b = w.block_off(args.block_index), w.block
    esize = 2 if w.dtype == "bf16" else 4
    shape = B.make_shape(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                         seq_len=w.seq_len, block_off=o, block_len=b,
                         dtype=B.SDLLM_BF16 if w.dtype == "bf16" else B.SDLLM_F32, retention=w.retention,
                         pool_kernel=w.pool_kernel)
    k_total, _, _ = B.sdllm_retained_count(shape)
    shape = B.make_shape(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                         seq_len=w.seq_len, block_off=o, block_len=b,
                         dtype=B.SDLLM_BF16 if w.dtype == "bf16" else B.SDLLM_F32, retention=w.retention,
                         pool_kernel=w.pool_kernel, cache_rows=max(1, k_total))
    ws = torch.empty(B.sdllm_workspace_bytes(shape, B.SDLLM_OP_BLOCK_STEP), dtype=torch.uint8, device=dev)

    layers = []
    inp0_host = None
    for layer in range(n_layers):
        inp = wl.make_block_inputs(w, layer, args.block_index, T, device=dev)
        td = w.torch_dtype
        st = dict(k_full=inp["k_full"], v_full=inp["v_full"], q=inp["q"], k_blk=inp["k_blk"], v_blk=inp["v_blk"],
                  k_cache=torch.zeros(w.batch, w.n_kv_heads, max(1, k_total), w.head_dim, dtype=td, device=dev),
                  v_cache=torch.zeros(w.batch, w.n_kv_heads, max(1, k_total), w.head_dim, dtype=td, device=dev),
                  idx=torch.zeros(w.batch, w.n_kv_heads, max(1, k_total), dtype=torch.int32, device=dev),
                  out=torch.zeros(w.batch, w.n_q_heads, b, w.head_dim, dtype=td, device=dev))
        layers.append(st)
        if layer == 0 and not args.no_cpu_baseline:
            nb = min(args.cpu_batch, w.batch)
            inp0_host = {k: (v[:nb].cpu() if k in ("k_full", "v_full") else v[:, :nb].cpu())
                         for k, v in inp.items() if k in ("k_full", "v_full", "q", "k_blk", "v_blk")}
            inp0_host["block_off"] = o
    torch.cuda.synchronize()

    states = [B.sdllm_cache_state(t, 1) for t in range(T)]
    sparse_events = []   # (start, stop) around every all-layer sweep of sparse (state-2) calls

    def run_block(record: bool):
        for t in range(T):
            reuse = states[t] == B.SDLLM_STATE_REUSE
            if record and reuse:
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
            for st in layers:
                if reuse:
                    B.sdllm_block_step(shape, t, 1, st["q"][t], st["k_blk"][t], st["v_blk"][t], st["idx"], st["k_cache"],
                                       st["v_cache"], st["out"], ws)
                else:
                    # a model produces fresh full-sequence K/V at these steps; the synthetic driver
                    # reuses the resident tensors (same bytes read)
                    B.sdllm_block_step(shape, t, 1, st["q"][t], st["k_full"], st["v_full"], st["idx"], st["k_cache"],
                                       st["v_cache"], st["out"], ws)
            if record and reuse:
                e1.record()
                sparse_events.append((e0, e1))

    for _ in range(max(1, args.warmup) if args.graph else args.warmup):
        run_block(False)
    torch.cuda.synchronize()
    if args.graph:
        # the library only enqueues kernels on the given stream (no allocation, no memset, no sync),
        # so a whole block records into one graph; the sparse sweep is captured separately to time it
        side = torch.cuda.Stream()
        g_block, g_sparse = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_block, stream=side):
            run_block(False)
        t_sparse = next(t for t in range(T) if states[t] == B.SDLLM_STATE_REUSE)
        with torch.cuda.graph(g_sparse, stream=side):
            for st in layers:
                B.sdllm_block_step(shape, t_sparse, 1, st["q"][t_sparse], st["k_blk"][t_sparse], st["v_blk"][t_sparse],
                                   st["idx"], st["k_cache"], st["v_cache"], st["out"], ws)
        g_block.replay()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if args.graph:
            g_block.replay()
        else:
            run_block(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if args.graph:
        reps = 10
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g_sparse.replay()
        e1.record()
        torch.cuda.synchronize()
        sparse_events = None
        sparse_ms = [e0.elapsed_time(e1) / reps]
    else:
        sparse_ms = [a.elapsed_time(bb) for a, bb in sparse_events]

    elapsed = t1 - t0
    calls = args.steps * T * n_layers
    sparse_launch_us = 1e3 * sum(sparse_ms) / (len(sparse_ms) * n_layers) if sparse_ms else float("nan")
    # spread over the timed all-layer sweeps (each sample = one sweep's HIP-event time / layers)
    per_sweep = sorted(1e3 * m / n_layers for m in sparse_ms)
    pct = lambda q: per_sweep[min(len(per_sweep) - 1, int(q * len(per_sweep)))] if per_sweep else float("nan")
    sparse_spread = {"samples": len(per_sweep), "p10_us": pct(0.10), "p50_us": pct(0.50), "p90_us": pct(0.90)}
    bytes_sparse = attn_bytes(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, k_total + b, b, esize)
    achieved = bytes_sparse / (sparse_launch_us * 1e-6) / 1e9 if sparse_ms else float("nan")

    # per-stage launch times outside the headline region (same buffers, event-timed sweeps over all layers)
    def sweep_us(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1) / (reps * n_layers)

    def dense_sweep():
        for st in layers:
            B.sdllm_block_step(shape, 0, 1, st["q"][0], st["k_full"], st["v_full"], st["idx"], st["k_cache"], st["v_cache"],
                               st["out"], ws)

    def score_sweep():
        for st in layers:
            B.sdllm_score_select(shape, st["q"][1], st["k_full"], st["idx"], None, None, ws)

    def compact_sweep():
        for st in layers:
            B.sdllm_compact_kv(shape, st["k_full"], st["v_full"], st["idx"], st["k_cache"], st["v_cache"])

    # a plain device-to-device copy of known size: the reference dispatch against which HBM byte
    # counters (FETCH_SIZE / WRITE_SIZE) of a profiler run are scaled
    calib_src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    torch.cuda.synchronize()

    def update_sweep():
        for st in layers:
            B.sdllm_block_step(shape, 1, 1, st["q"][1], st["k_full"], st["v_full"], st["idx"], st["k_cache"], st["v_cache"],
                               st["out"], ws)

    # score_select_us is the stand-alone entry point (its own row-statistics pass over K); inside the
    # cache-update step those statistics come out of the dense attention, see cache_update_step_us
    stages = {"dense_block_attn_us": sweep_us(dense_sweep), "score_select_us": sweep_us(score_sweep),
              "compact_kv_us": sweep_us(compact_sweep), "sparse_attn_us": sparse_launch_us,
              "cache_update_step_us": sweep_us(update_sweep)}
    n_cand = w.seq_len - b
    stage_bytes = {
        "dense_block_attn": attn_bytes(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.seq_len, b, esize),
        "score_select": w.batch * w.n_kv_heads * n_cand * w.head_dim * esize + w.batch * w.n_q_heads * b * w.head_dim * esize
                        + 4 * w.batch * w.n_kv_heads * (2 * n_cand + k_total),
        "compact_kv": 2 * (2 * w.batch * w.n_kv_heads * k_total * w.head_dim * esize) + 4 * w.batch * w.n_kv_heads * k_total,
        "sparse_attn": bytes_sparse,
    }
    stage_gbs = {k: stage_bytes[k] / (stages[k + "_us"] * 1e-6) / 1e9 for k in stage_bytes}

    # what the memory system delivers for the attention kernel's access pattern: a bare streaming
    # read of the sparse step's byte count, rotated over distinct buffers like the layers are
    n_probe = 8
    probe_bufs = [torch.empty(bytes_sparse // 16 * 16, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(n_probe)]
    probe_sink = torch.zeros(1, dtype=torch.int32, device=dev)
    for pb in probe_bufs:
        B.sdllm_stream_read_probe(pb, probe_sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(4):
        for pb in probe_bufs:
            B.sdllm_stream_read_probe(pb, probe_sink)
    e1.record()
    torch.cuda.synchronize()
    probe_us = 1e3 * e0.elapsed_time(e1) / (4 * n_probe)
    read_ceiling_gbs = probe_bufs[0].numel() / (probe_us * 1e-6) / 1e9
    del probe_bufs

    # the row next to the hot path: full-sequence attention of cache states 0/1 (compute-bound)
    dense_full = None
    if w.dtype == "bf16" and w.head_dim == 128:
        st0 = layers[0]
        q_full = torch.randn(w.batch, w.n_q_heads, w.seq_len, w.head_dim, device=dev).to(w.torch_dtype)
        out_full = torch.empty_like(q_full)
        B.sdllm_dense_attn(shape, q_full, st0["k_full"], st0["v_full"], out_full)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(2):
            B.sdllm_dense_attn(shape, q_full, st0["k_full"], st0["v_full"], out_full)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 2
        flops = 4.0 * w.batch * w.n_q_heads * w.seq_len * w.seq_len * w.head_dim
        dense_full = {"entry": "sdllm_dense_attn (one layer, all L query rows)", "ms": ms,
                      "roofline": {"bound": "mfma", "achieved": flops / ms / 1e9, "peak": 2500.0, "unit": "TFLOP/s",
                                   "frac": flops / ms / 1e9 / 2500.0}}
        del q_full, out_full

    traffic, traffic_source = measured_traffic(w.name, args.batch == 0 and args.block_index == 0)
    result = {
        "metric": "sparse block-step attention: block-steps/s per layer + achieved HBM GB/s (% of peak)",
        "value": calls / elapsed,
        "unit": "block-steps/s per layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: {n_layers} layers x (B={w.batch}, Hq={w.n_q_heads}, Hkv={w.n_kv_heads}, "
                               f"d={w.head_dim}), prompt {w.prompt}, gen {w.gen}, block {b}, {T} steps/block, "
                               f"r={w.retention}, pool {w.pool_kernel}, block index {args.block_index}; one step = one decoding block "
                               f"through all layers",
                   "block_steps_per_step": T * n_layers, "retained_per_head": k_total},
        "launch_mode": "hip graph replay" if args.graph else "eager launches",
        "tokens_per_s_attention_path": w.batch * b * args.steps / elapsed,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "attn_mfma_bf16_kernel (sdllm_sparse_attn, cache_state 2)",
                     "algorithmic_bytes_per_launch": bytes_sparse, "avg_launch_us": sparse_launch_us,
                     "launch_us_spread": sparse_spread,
                     "streaming_read_ceiling": {"us_for_same_bytes": probe_us, "GB/s": read_ceiling_gbs,
                                                "achieved_over_ceiling": achieved / read_ceiling_gbs}},
        # the comparator the workload names: a dense full-cache scheme pays the dense block-row attention
        # at every one of the T denoising steps of a block (same kernel over all L keys)
        "vs_dense_full_cache": {
            "sparse_path_us_per_block_per_layer": 1e6 * elapsed / (args.steps * n_layers),
            "dense_cache_us_per_block_per_layer": T * stages["dense_block_attn_us"],
            "attention_path_speedup": T * stages["dense_block_attn_us"] / (1e6 * elapsed / (args.steps * n_layers)),
            "us_per_generated_token_sparse": 1e6 * elapsed / (args.steps * w.batch * b),
            "us_per_generated_token_dense_cache": T * stages["dense_block_attn_us"] * n_layers / (w.batch * b)},
        "stages_us_per_layer_call": stages,
        "full_sequence_attention": dense_full,
        "stages_algorithmic_gbs": stage_gbs,
    }
    # the other single-layer configurations of the workload list, briefly (per layer call, one GPU)
    if not args.no_other_workloads and args.workload == "llada8b_sweep" and args.batch == 0 and not args.graph:
        layers.clear()
        st0 = st = inp = None
        torch.cuda.empty_cache()
        result["other_workloads"] = {n: quick_workload(n, dev) for n in ("llada8b_layer", "dream7b_gqa", "dream_long")}
    if inp0_host is not None:
        result["cpu_baseline"] = cpu_baseline(w, inp0_host, inp0_host["k_full"].shape[0])
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
