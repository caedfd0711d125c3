// Internal declarations shared by the C-ABI dispatcher and the kernel launchers.
// Nothing here is exported; the public surface is include/sdllm.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace sdllm {

constexpr int kWave = 64;            // CDNA wavefront
constexpr int kTileKeys = 32;        // keys per MFMA tile (one 32x32 block of logits)
constexpr int kMaxWavesPerWg = 8;    // attention / scoring workgroups hold up to 8 waves
constexpr int kNumCUs = 256;         // MI355X
constexpr int kNumXCDs = 8;

// Workgroup ids are dealt round-robin over the 8 XCDs, each with its own L2.  This renumbering gives
// every XCD one contiguous range of the result instead (XCD x gets the ids it was dealt, in order,
// placed after those of the XCDs before it), for any grid size, so that neighbours in the new
// numbering - the query heads of a KV group, the key splits of a head - share an L2.
__host__ __device__ inline int xcd_contiguous_id(int dealt, int n) {
  const int x = dealt % kNumXCDs, q = n / kNumXCDs, r = n % kNumXCDs;
  return x * q + (x < r ? x : r) + dealt / kNumXCDs;
}

// Kernels that need more than the default 64 KB of dynamic LDS have to opt in, once per device (the
// attribute belongs to the device's copy of the kernel).  One object per kernel remembers which
// devices are done; concurrent host threads at worst both set the same value.
class LdsOptIn {
 public:
  hipError_t ensure(const void* kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    const uint64_t bit = tracked ? uint64_t{1} << dev : 0;
    if (tracked && (done_.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && tracked) done_.fetch_or(bit, std::memory_order_release);
    return e;
  }

 private:
  std::atomic<uint64_t> done_{0};
};

// One source of keys/values: rows of a [B, Hkv, n, d] tensor given by element strides.
struct KvSegment {
  const void* k;
  const void* v;
  int64_t sb, sh, sr;  // element strides: batch, head, row
  int32_t n;           // rows per (batch, head)
};

// Attention of nq query rows per head over Concat(seg[0], seg[1]) (Alg. 3, state 2; with a
// single full-sequence segment it is the dense block-row attention of states 0/1).
struct AttnParams {
  const void* q;
  void* out;
  KvSegment seg[2];
  int64_t q_sb, q_sh, q_sr;
  int64_t o_sb, o_sh, o_sr;
  int32_t batch, hq, hkv, group, nq, d;
  float scale_log2;     // softmax scale * log2(e)
  // split-KV plan
  int32_t n_split;          // workgroups per head
  int32_t tiles_per_split;  // 32-key tiles each workgroup owns
  int32_t waves;            // waves per workgroup
  float* part_o;            // [B*Hq, n_split, nq, d] fp32 partial numerators (n_split > 1)
  float* part_ml;           // [B*Hq, n_split, 2, nq] running max (log2 domain) and denominator
  // Optional by-product of a dense (single-segment) launch: the softmax row statistics of the
  // scoring pass, i.e. (max, sum) per query row over the CANDIDATE keys only, which are the keys
  // outside [cand0_end, cand1_begin).  Layout [B*Hq, n_split, 2, nq], the layout the scoring
  // kernels read their partial statistics in.  Null: not produced.
  float* cand_ml;
  int32_t cand0_end, cand1_begin;
  // Optional second by-product of such a launch (one workgroup per head, no key splits, MHA): the
  // softmax-mean saliency score of every candidate key (Alg. 1 steps 5-6), [B*Hkv, score_stride] floats,
  // written by a second sweep over K that each workgroup runs once its row statistics are final.
  // Null: not produced.
  float* score_out;
  int32_t score_stride;
  float score_inv_count;    // 1 / (block queries x query heads per KV head)
};

// Scoring of the candidates K_f = Concat[K_{:o}, K_{o+b:}] against the block's queries.
struct ScoreParams {
  const void* q;
  const void* k;        // full-sequence keys
  int64_t q_sb, q_sh, q_sr;
  int64_t k_sb, k_sh, k_sr;
  int32_t batch, hq, hkv, group, nq, d;
  int32_t block_off, block_len;
  int32_t n_cand;       // candidates scored (N, or N_pre for prefix-only eviction)
  int32_t softmax;      // 1: SOFTMAX_MEAN, 0: LOGIT_MEAN
  float scale;          // softmax scale
  float scale_log2;     // scale * log2(e)
  float* score;         // [B*Hkv, score_stride], the first n_cand of each row written
  int32_t score_stride;
  // row statistics of the softmax (pass 1 -> pass 2)
  int32_t n_part;       // workgroups per (batch, KV head) row of the scoring kernels
  int32_t tiles_per_part;
  float* part_ml;       // [B*Hq, n_stat_part, 2, nq]
  int32_t n_stat_part;  // partial (max, sum) pairs per query row in part_ml
  int32_t skip_stats;   // 1: part_ml was already filled (by the dense attention of the same step)
  int32_t cols_follow;  // set by the launcher: the statistics kernel runs the column pass itself (n_part == 1)
  int32_t waves;
};

struct SelectParams {
  const float* score;   // [rows, n_cand]
  float* pooled;        // optional [rows, n_cand]: the pooled scores (only when the caller wants them)
  int32_t* idx;         // [rows, k_total]
  int32_t rows;         // B * Hkv
  int32_t n_cand;
  int32_t n_seg;        // 1 or 2 ranked segments
  int32_t seg_begin[2], seg_len[2], seg_k[2], seg_out[2];
  int32_t k_total;
  int32_t pool_half;    // (s-1)/2
  int32_t avg_pool;
  int32_t block_off, block_len;
  // candidates appended unconditionally after the ranked ones (prefix-only eviction keeps the
  // whole suffix): candidate indices [tail_begin, tail_begin + tail_len)
  int32_t tail_begin, tail_len, tail_out;
  // workspace of the path for segments too long for one workgroup (sizes: select_workspace()), else null
  uint32_t* keys;       // [rows, n_cand] order-preserving integer image of the pooled scores, in position order
  uint32_t* sorted;     // [rows, n_cand] the same keys, every chunk of 1024 ordered by leading bits
  uint32_t* bins;       // [rows, 2, chunks] lists of the non-empty leading-bit bins of every chunk
  int32_t chunks;       // set by the launcher: chunks of the longest ranked segment
};

struct SelectWorkspace { size_t keys, sorted, bins; };   // in 32-bit words

struct CompactParams {
  const void* k;
  const void* v;
  const int32_t* idx;
  void* kc;
  void* vc;
  int64_t s_sb, s_sh, s_sr;  // source strides in BYTES
  int64_t c_sb, c_sh, c_sr;  // cache strides in BYTES
  int32_t batch, hkv, k_total, seq_len;
  int32_t row_bytes;
};

// Full-sequence bidirectional attention: L query rows per head over all L keys.
struct DenseFullParams {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  int64_t q_sb, q_sh, q_sr;
  int64_t k_sb, k_sh, k_sr;
  int64_t o_sb, o_sh, o_sr;
  int32_t batch, hq, hkv, group, seq_len, d;
  float scale_log2;
};

// kernel launchers (each returns hipGetLastError() after its launches)
hipError_t launch_attn_mfma_bf16(const AttnParams& p, hipStream_t s);
hipError_t launch_attn_gqa_mfma_bf16(const AttnParams& p, hipStream_t s);
bool attn_gqa_supports_group(int group);
int attn_gqa_waves_per_wg(int group);
hipError_t launch_attn_simple(const AttnParams& p, int dtype, hipStream_t s);
hipError_t launch_attn_combine(const AttnParams& p, int dtype, hipStream_t s);
hipError_t launch_score_mfma_bf16(const ScoreParams& p, hipStream_t s);
bool score_mfma_supports_group(int group);
hipError_t launch_score_simple(const ScoreParams& p, int dtype, hipStream_t s);
hipError_t launch_select(const SelectParams& p, hipStream_t s);
SelectWorkspace select_workspace(const SelectParams& p);
int select_max_segment();
hipError_t launch_compact(const CompactParams& p, hipStream_t s);
// the gather plus the split-KV merge of a bf16 attention launch whose partials are still in the workspace
hipError_t launch_compact_combine(const CompactParams& p, const AttnParams& a, hipStream_t s);
hipError_t launch_dense_full_mfma_bf16(const DenseFullParams& p, hipStream_t s);
hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s);

}  // namespace sdllm
