/*
 * sdllm_bench.h - measurement aids exported by libsdllm.so next to the product API of sdllm.h.
 * Nothing here is part of the method; benchmarks use it to find what the memory system delivers.
 */
#ifndef SDLLM_BENCH_H
#define SDLLM_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads `bytes` bytes at `src` once with the memory access pattern of the block-attention kernel
 * of Alg. 3 (cache_state 2; non-temporal 16-byte loads, one 512-thread workgroup per contiguous chunk)
 * and discards them.  Timing it gives the bandwidth the memory system delivers for that pattern,
 * the practical ceiling for sdllm_sparse_attn.  `src` must be 16-byte aligned device memory; `sink`
 * is 4 bytes of device memory (may be NULL); `stream` a hipStream_t (NULL = default stream).
 * Returns SDLLM_OK (0), SDLLM_ERR_INVALID_ARG (-1) or SDLLM_ERR_HIP (-4) as in sdllm.h.
 */
int32_t sdllm_stream_read_probe(const void* src, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SDLLM_BENCH_H */
