/*
 * sdllm.h - C ABI of the MI355X (gfx950) Sparse-dLLM block-step attention library.
 *
 * The library implements the per-layer hot path of Sparse-dLLM (delayed bidirectional sparse
 * caching for block-wise diffusion-LLM decoding): saliency scoring of the keys outside the
 * current block, max-pool smoothing, top-k retention, gather-compaction of the retained K/V rows
 * and unmasked attention of the block's queries over the compacted cache plus the block.
 *
 * Conventions for every entry point
 *   - plain C, no exceptions; the return value is a status code (SDLLM_OK == 0, errors < 0);
 *   - every data pointer is a DEVICE pointer on the current HIP device unless marked "host";
 *     the caller owns all buffers, the library never allocates, frees or synchronises;
 *   - work is only enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream);
 *   - tensors are dense in their last axis (head_dim contiguous); the other axes are described
 *     by element strides {batch, head, row} in sdllm_shape_t.  Rows must be 16-byte aligned
 *     (base pointers and strides*sizeof(element) multiples of 16);
 *   - query head h reads KV head h / (n_q_heads / n_kv_heads);
 *   - on an argument error nothing is enqueued.
 *
 * Notation (the paper's): b block length, o offset of the block's first token, L sequence length,
 * N_pre = o, N_suf = L - o - b, N = N_pre + N_suf candidates, r retention ratio, s pool kernel.
 */
#ifndef SDLLM_H
#define SDLLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define SDLLM_OK 0
#define SDLLM_ERR_INVALID_ARG (-1) /* null pointer, bad size, r outside [0,1], even pool kernel, misalignment */
#define SDLLM_ERR_UNSUPPORTED (-2) /* a legal request this build has no kernel for */
#define SDLLM_ERR_WORKSPACE (-3)   /* workspace pointer null or smaller than sdllm_workspace_bytes() */
#define SDLLM_ERR_HIP (-4)         /* a HIP launch reported an error */
#define SDLLM_ERR_STATIC_LIMIT (-5) /* sdllm_sparse_attn_noalloc: the request needs more than SDLLM_STATIC_SCRATCH_BYTES */

/* element types of Q/K/V/O (accumulation is always fp32) */
#define SDLLM_BF16 0
#define SDLLM_F32 1

/* how the per-candidate score is formed from the logits A = Q_b K_f^T / sqrt(d) (Sec. 3.3):
 * SOFTMAX_MEAN normalises each query row over all candidates first ("average attention scores",
 * the sentence introducing Alg. 1); LOGIT_MEAN averages the raw logits (Alg. 1 steps 5-6 literal). */
#define SDLLM_SOFTMAX_MEAN 0
#define SDLLM_LOGIT_MEAN 1

/* PER_SEGMENT pools and ranks prefix and suffix separately, each with its own quota;
 * JOINT pools and ranks the concatenated candidate array as one (Alg. 1 literal). */
#define SDLLM_PER_SEGMENT 0
#define SDLLM_JOINT 1

/* quota rounding: ceil(r*n) or floor(r*n) (Alg. 1 step 9), r*n evaluated in double with a 1e-9 guard */
#define SDLLM_CEIL 0
#define SDLLM_FLOOR 1

/* local aggregation (Sec. 3.3 third equation; AvgPool is the appendix ablation) */
#define SDLLM_MAX_POOL 0
#define SDLLM_AVG_POOL 1

/* which candidates may be evicted: both sides of the block (Alg. 1) or the prefix only, the
 * suffix being kept whole (Alg. 4, the prefix-sparse ablation) */
#define SDLLM_EVICT_BIDIRECTIONAL 0
#define SDLLM_EVICT_PREFIX_ONLY 1

/* cache states (Alg. 2 / Alg. 5) */
#define SDLLM_STATE_FULL 0
#define SDLLM_STATE_UPDATE 1
#define SDLLM_STATE_REUSE 2

/* operations for sdllm_workspace_bytes */
#define SDLLM_OP_SCORE_SELECT 0
#define SDLLM_OP_COMPACT_KV 1
#define SDLLM_OP_SPARSE_ATTN 2
#define SDLLM_OP_BLOCK_STEP 3

typedef struct sdllm_shape {
  int32_t batch;       /* B >= 1 */
  int32_t n_q_heads;   /* Hq, multiple of n_kv_heads */
  int32_t n_kv_heads;  /* Hkv >= 1 */
  int32_t head_dim;    /* d in {64, 128} */
  int32_t seq_len;     /* L */
  int32_t block_off;   /* o, 0 <= o, o + b <= L */
  int32_t block_len;   /* b, 1 <= b <= 64 */
  int32_t dtype;       /* SDLLM_BF16 | SDLLM_F32 */
  int32_t pool_kernel; /* s, odd, >= 1 */
  int32_t score_mode;  /* SDLLM_SOFTMAX_MEAN | SDLLM_LOGIT_MEAN */
  int32_t select_mode; /* SDLLM_PER_SEGMENT | SDLLM_JOINT */
  int32_t k_rounding;  /* SDLLM_CEIL | SDLLM_FLOOR */
  int32_t pool_mode;   /* SDLLM_MAX_POOL | SDLLM_AVG_POOL */
  int32_t evict_scope; /* SDLLM_EVICT_BIDIRECTIONAL | SDLLM_EVICT_PREFIX_ONLY */
  float softmax_scale; /* 0 means 1/sqrt(head_dim) */
  int32_t reserved;    /* must be 0 */
  double retention;    /* r in [0, 1] */
  /* element strides {batch, head, row}; the last axis (head_dim) is contiguous */
  int64_t q_stride[3];     /* block queries            [B, Hq,  b, d] */
  int64_t kv_stride[3];    /* full-sequence K and V    [B, Hkv, L, d] */
  int64_t blk_stride[3];   /* block K_n and V_n        [B, Hkv, b, d] */
  int64_t cache_stride[3]; /* compacted K_c and V_c    [B, Hkv, >= k, d] */
  int64_t out_stride[3];   /* attention output         [B, Hq,  b, d] */
} sdllm_shape_t;

/* Static string for a status code.  Host only. */
const char* sdllm_error_string(int32_t status);

/* Library version, major*10000 + minor*100 + patch.  Host only. */
int32_t sdllm_version(void);

/*
 * Number of retained entries per (batch, KV head) row for this shape (Sec. 3.3: k = (L-b)*r;
 * Alg. 1 step 9).  All outputs are host pointers and may be NULL.  k_total is what
 * sdllm_score_select writes per row.  k_pre / k_suf are the prefix / suffix quotas in
 * PER_SEGMENT mode and -1 in JOINT mode, where the split depends on the data.  With
 * SDLLM_EVICT_PREFIX_ONLY the suffix quota is N_suf.
 */
int32_t sdllm_retained_count(const sdllm_shape_t* shape, int32_t* k_total, int32_t* k_pre, int32_t* k_suf);

/*
 * Bytes of device workspace `op` needs for this shape (host call).  n_cached is the number of
 * cache rows sdllm_sparse_attn will be given (ignored by the other ops; SDLLM_OP_BLOCK_STEP
 * covers every state of the step, including dense attention over all L keys).
 */
int32_t sdllm_workspace_bytes(const sdllm_shape_t* shape, int32_t op, int32_t n_cached, size_t* bytes);

/* Cache state of step `step_in_block` (0-based) under delay x: 2 if i > x, 1 if i == x, else 0
 * (Alg. 2 for x = 1, Alg. 5 in general).  `state` is a host pointer. */
int32_t sdllm_cache_state(int32_t step_in_block, int32_t delay, int32_t* state);

/*
 * Alg. 1 steps 2-10: score every candidate key against the block's queries, smooth, keep the top
 * entries.  q_blk [B,Hq,b,d] (q_stride), k_full [B,Hkv,L,d] (kv_stride).
 *   idx_out    [B,Hkv,k_total] int32, contiguous: retained ABSOLUTE positions, ascending.  Ties in
 *              the pooled score go to the lower position.
 *   pooled_out optional [B,Hkv,N] fp32 contiguous, candidate-indexed (c < o -> position c,
 *              c >= o -> position c + b): the pooled score.  May be NULL.
 *   score_out  optional [B,Hkv,N] fp32: the score before pooling.  May be NULL.
 * A ranked segment (prefix, suffix, or the joint array) of more than 1 048 576 candidates returns
 * SDLLM_ERR_UNSUPPORTED.
 *   ws         workspace of at least sdllm_workspace_bytes(SDLLM_OP_SCORE_SELECT) bytes,
 *              256-byte aligned; contents undefined afterwards.
 */
int32_t sdllm_score_select(const sdllm_shape_t* shape, const void* q_blk, const void* k_full, int32_t* idx_out,
                           float* pooled_out, float* score_out, void* ws, size_t ws_bytes, void* stream);

/*
 * Alg. 1 steps 12-14: K_c[j] = K[idx[j]], V_c[j] = V[idx[j]] for j < k_total, per (batch, KV head).
 * k_full/v_full [B,Hkv,L,d] (kv_stride); idx [B,Hkv,k_total] int32 as written by
 * sdllm_score_select (values must lie in [0, L)); k_cache/v_cache [B,Hkv,>=k_total,d]
 * (cache_stride).  A byte copy: bit-exact.
 */
int32_t sdllm_compact_kv(const sdllm_shape_t* shape, const void* k_full, const void* v_full, const int32_t* idx,
                         void* k_cache, void* v_cache, void* stream);

/*
 * Alg. 3, cache_state == 2: out = softmax(scale * Q_n Concat(K_c,K_n)^T) Concat(V_c,V_n), no mask.
 * q_blk [B,Hq,b,d] (q_stride); k_cache/v_cache [B,Hkv,n_cached,d] (cache_stride), n_cached >= 0
 * (0: attention over the block only; the cache pointers may then be NULL); k_blk/v_blk
 * [B,Hkv,b,d] (blk_stride); out [B,Hq,b,d] (out_stride).  ws as for sdllm_score_select with
 * SDLLM_OP_SPARSE_ATTN and the same n_cached.
 */
int32_t sdllm_sparse_attn(const sdllm_shape_t* shape, const void* q_blk, const void* k_cache, const void* v_cache,
                          int32_t n_cached, const void* k_blk, const void* v_blk, void* out, void* ws,
                          size_t ws_bytes, void* stream);

/*
 * sdllm_sparse_attn for callers that cannot allocate or size a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical results, but the split-KV partials live in an array of SDLLM_STATIC_SCRATCH_BYTES
 * that is part of the library's device image (every GPU the library runs on holds one copy until the
 * process ends).  The call allocates nothing and frees nothing.  A shape whose launch plan needs
 * more scratch than that returns SDLLM_ERR_STATIC_LIMIT and enqueues nothing (use sdllm_sparse_attn
 * with a workspace then).  All calls on one GPU share that GPU's array: calls that overlap in time
 * on one GPU (different streams, or concurrently replayed graphs) race and are not allowed.  The
 * first call on each device resolves the array's address and must not be made under stream capture.
 */
#define SDLLM_STATIC_SCRATCH_BYTES (8u << 20)
int32_t sdllm_sparse_attn_noalloc(const sdllm_shape_t* shape, const void* q_blk, const void* k_cache,
                                  const void* v_cache, int32_t n_cached, const void* k_blk, const void* v_blk,
                                  void* out, void* stream);

/*
 * One denoising step of one layer (Alg. 2/5 -> Alg. 3 -> Alg. 1).  state = cache_state(step, delay).
 *   state 0: k_in/v_in are the full-sequence K,V [B,Hkv,L,d] (kv_stride); out = the block's rows
 *            of dense bidirectional attention over all L keys.  Cache untouched.
 *   state 1: as state 0, and the cache is rebuilt from this step's tensors: idx, k_cache, v_cache
 *            are written (sdllm_score_select + sdllm_compact_kv).
 *   state 2: k_in/v_in are the block's K_n,V_n [B,Hkv,b,d] (blk_stride); out = sparse attention
 *            over the cache (k_total rows per KV head, as sdllm_retained_count reports) + block.
 * idx [B,Hkv,k_total] int32; ws sized by SDLLM_OP_BLOCK_STEP.  `state_out` (host, may be NULL)
 * receives the state that was executed.
 */
int32_t sdllm_block_step(const sdllm_shape_t* shape, int32_t step_in_block, int32_t delay, const void* q_blk,
                         const void* k_in, const void* v_in, int32_t* idx, void* k_cache, void* v_cache, void* out,
                         void* ws, size_t ws_bytes, void* stream, int32_t* state_out);

/*
 * Full bidirectional attention of ALL L positions (Sec. 3.1: the mask predictor recomputes the whole
 * sequence; cache_state 0 and 1 of the cache-management appendix run it for the rows outside the
 * current block, whose block rows sdllm_block_step returns):
 *   out[b,h,i,:] = sum_j softmax_j(scale * <q[b,h,i], k[b,g(h),j]>) v[b,g(h),j],  i, j in [0, L), no mask.
 * q_full/out_full are [B,Hq,L,d] with element strides {batch, head, row} given by q_full_stride /
 * out_full_stride (host pointers to 3 values); k_full/v_full [B,Hkv,L,d] use shape->kv_stride.
 * Only batch, head counts, head_dim, seq_len, dtype, softmax_scale and kv_stride of `shape` are read
 * besides the usual validity checks.  No workspace.
 */
int32_t sdllm_dense_attn(const sdllm_shape_t* shape, const void* q_full, const int64_t* q_full_stride,
                         const void* k_full, const void* v_full, void* out_full, const int64_t* out_full_stride,
                         void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SDLLM_H */
