// C-ABI entry points: argument validation, launch planning and dispatch.  No arithmetic of the
// method lives here except the retained-count rule and the cache-state schedule, which are host
// logic by nature (Alg. 1 step 9; Alg. 2 / Alg. 5).
#include <math.h>
#include <stdlib.h>

#include "sdllm.h"
#include "sdllm_bench.h"
#include "sdllm_internal.h"

using namespace sdllm;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline int elem_size(int dtype) { return dtype == SDLLM_BF16 ? 2 : 4; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int32_t quota(int32_t n, double r, int32_t rounding) {
  const double x = r * (double)n;
  const double k = rounding == SDLLM_CEIL ? ceil(x - 1e-9) : floor(x + 1e-9);
  if (k < 0) return 0;
  if (k > n) return n;
  return (int32_t)k;
}

struct Counts { int32_t n_pre, n_suf, n_cand, k_total, k_pre, k_suf; };

Counts counts_of(const sdllm_shape_t& s) {
  Counts c;
  c.n_pre = s.block_off;
  c.n_suf = s.seq_len - s.block_off - s.block_len;
  c.n_cand = c.n_pre + c.n_suf;
  if (s.evict_scope == SDLLM_EVICT_PREFIX_ONLY) {
    c.k_pre = quota(c.n_pre, s.retention, s.k_rounding);
    c.k_suf = c.n_suf;
    c.k_total = c.k_pre + c.k_suf;
  } else if (s.select_mode == SDLLM_PER_SEGMENT) {
    c.k_pre = quota(c.n_pre, s.retention, s.k_rounding);
    c.k_suf = quota(c.n_suf, s.retention, s.k_rounding);
    c.k_total = c.k_pre + c.k_suf;
  } else {
    c.k_total = quota(c.n_cand, s.retention, s.k_rounding);
    c.k_pre = c.k_suf = -1;
  }
  return c;
}

bool strides_ok(const int64_t* st, int esize) {
  for (int i = 0; i < 3; ++i)
    if (st[i] < 0 || (st[i] * esize) % 16 != 0) return false;
  return true;
}

int32_t check_shape(const sdllm_shape_t* s) {
  if (!s) return SDLLM_ERR_INVALID_ARG;
  if (s->batch < 1 || s->n_kv_heads < 1 || s->n_q_heads < 1 || s->n_q_heads % s->n_kv_heads != 0)
    return SDLLM_ERR_INVALID_ARG;
  if (s->dtype != SDLLM_BF16 && s->dtype != SDLLM_F32) return SDLLM_ERR_INVALID_ARG;
  if (s->block_len < 1 || s->block_off < 0 || s->seq_len < 1 ||
      (int64_t)s->block_off + s->block_len > s->seq_len)
    return SDLLM_ERR_INVALID_ARG;
  if (!(s->retention >= 0.0 && s->retention <= 1.0)) return SDLLM_ERR_INVALID_ARG;
  if (s->pool_kernel < 1 || s->pool_kernel % 2 == 0) return SDLLM_ERR_INVALID_ARG;
  if (s->score_mode != SDLLM_SOFTMAX_MEAN && s->score_mode != SDLLM_LOGIT_MEAN) return SDLLM_ERR_INVALID_ARG;
  if (s->select_mode != SDLLM_PER_SEGMENT && s->select_mode != SDLLM_JOINT) return SDLLM_ERR_INVALID_ARG;
  if (s->k_rounding != SDLLM_CEIL && s->k_rounding != SDLLM_FLOOR) return SDLLM_ERR_INVALID_ARG;
  if (s->pool_mode != SDLLM_MAX_POOL && s->pool_mode != SDLLM_AVG_POOL) return SDLLM_ERR_INVALID_ARG;
  if (s->evict_scope != SDLLM_EVICT_BIDIRECTIONAL && s->evict_scope != SDLLM_EVICT_PREFIX_ONLY)
    return SDLLM_ERR_INVALID_ARG;
  if (!(s->softmax_scale >= 0.f) || !isfinite(s->softmax_scale) || s->reserved != 0) return SDLLM_ERR_INVALID_ARG;
  const int es = elem_size(s->dtype);
  if (!strides_ok(s->q_stride, es) || !strides_ok(s->kv_stride, es) || !strides_ok(s->blk_stride, es) ||
      !strides_ok(s->cache_stride, es) || !strides_ok(s->out_stride, es))
    return SDLLM_ERR_INVALID_ARG;
  if (s->head_dim != 64 && s->head_dim != 128) return SDLLM_ERR_UNSUPPORTED;
  if (s->block_len > 64) return SDLLM_ERR_UNSUPPORTED;
  return SDLLM_OK;
}

bool row_stride_ok(const int64_t* st, int d) { return st[2] >= d; }

float scale_of(const sdllm_shape_t& s) {
  return s.softmax_scale > 0.f ? s.softmax_scale : 1.0f / sqrtf((float)s.head_dim);
}

constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------- attention planning
struct AttnPlan {
  bool mfma;
  bool gqa;   // grouped-query kernel: one workgroup per (batch, KV head), wave = query head
  int n_split, tiles_per_split, waves;
  size_t part_o_bytes, part_ml_bytes;
  size_t ws_bytes() const { return part_o_bytes + part_ml_bytes; }
};

bool seg_fits_u32(int64_t row_stride, int32_t n, int esize) {
  return n <= 0 || ((int64_t)(n - 1) * row_stride + 128) * esize < (int64_t)1 << 31;
}

AttnPlan plan_attn(const sdllm_shape_t& s, int32_t n0, int64_t sr0, int32_t n1, int64_t sr1) {
  AttnPlan pl{};
  pl.mfma = s.dtype == SDLLM_BF16 && s.head_dim == 128 && s.block_len == 32 && seg_fits_u32(sr0, n0, 2) &&
            seg_fits_u32(sr1, n1, 2);
  pl.n_split = 1;
  pl.tiles_per_split = 0;
  pl.waves = 1;
  // Grouped-query heads: either one workgroup per query head (K/V then come G times out of L2, but the
  // eight waves of a head split its keys and merge in LDS) or the shared-tile kernel (K/V read once,
  // one wave per head, key splits merged through fp32 partials and a second launch).  Measured on
  // MI355X (G = 2, 3, 4, 5, 7, 8; batch 1-64; 2k-49k keys; sparse and dense steps), in wave-tiles of
  // work (heads x 32-key tiles): with four waves per workgroup (G = 7, 8) the shared-tile kernel wins
  // from about 30 000, from about 22 000 when each head has 512 tiles or more (long prompts: the
  // dense step of the batch-1 32k-prompt Dream shape 48.6 -> 44.4 us, of the 48k one 65 -> 56 us),
  // and from about 18 000 with 128 heads or more, whose rows need few key splits (140 heads x 136
  // tiles: 37.9 -> 33.4 us; 84 heads x 264 tiles lose, 34.2 against 39.1 us);
  // with two waves per workgroup (G = 2, 4) what decides is the number of heads, sparse and dense
  // step alike: 256 heads lose (G = 4: 28/51 us per head against 34/50 us shared), 384 heads win
  // (G = 4: 46/82 against 42/68 us; G = 2: 54/97 against 50/80 us), 512 heads tie, 640 win.
  const int all_tiles = (n0 + kTileKeys - 1) / kTileKeys + (n1 + kTileKeys - 1) / kTileKeys;
  const int64_t wave_tiles = (int64_t)s.batch * s.n_q_heads * all_tiles;
  const int group = s.n_q_heads / s.n_kv_heads;
  const int heads_all = s.batch * s.n_q_heads;
  pl.gqa = pl.mfma && attn_gqa_supports_group(group) &&
           (attn_gqa_waves_per_wg(group) >= 4
                ? wave_tiles >= 30000 || (all_tiles >= 512 && wave_tiles >= 22000) || (heads_all >= 128 && wave_tiles >= 18000)
                : heads_all >= 320 && wave_tiles >= 26000);
  if (pl.gqa) {
    const int tiles = (n0 + kTileKeys - 1) / kTileKeys + (n1 + kTileKeys - 1) / kTileKeys;
    const int rows = s.batch * s.n_kv_heads;
    // As many key splits as keep the grid within what the CUs hold at once (a few workgroups more
    // would wait for a whole round), but never fewer than 4 tiles (two LDS stages) each.  Four-wave
    // workgroups: two per CU.  Two-wave workgroups: four fit, three per CU measured best (G = 4,
    // 768 heads: 79.6 -> 63.9 us with 2 splits; G = 2, 1024 heads: 90 us with 1 split, 108 with 2).
    const int wg_waves = attn_gqa_waves_per_wg(group);
    const int wgs_per_row = (group + wg_waves - 1) / wg_waves;   // head splits
    const int room = (wg_waves >= 4 ? 2 : 3) * kNumCUs;
    int n_split = room / (rows * wgs_per_row);
    if (n_split < 1) n_split = 1;
    const int max_split = tiles / 4 > 1 ? tiles / 4 : 1;
    if (n_split > max_split) n_split = max_split;
    pl.tiles_per_split = (tiles + n_split - 1) / n_split;
    pl.n_split = (tiles + pl.tiles_per_split - 1) / pl.tiles_per_split;
    pl.waves = s.n_q_heads / s.n_kv_heads;
    if (pl.n_split > 1) {
      const size_t slots = (size_t)s.batch * s.n_q_heads * pl.n_split;
      pl.part_o_bytes = align_up(slots * s.block_len * s.head_dim * sizeof(float));
      pl.part_ml_bytes = align_up(slots * 2 * s.block_len * sizeof(float));
    }
  } else if (pl.mfma) {
    const int tiles = (n0 + kTileKeys - 1) / kTileKeys + (n1 + kTileKeys - 1) / kTileKeys;
    const int heads = s.batch * s.n_q_heads;
    // Split the keys of a head over workgroups only while the grid is small: as many splits as keep
    // the grid within one workgroup per CU (an eight-wave workgroup fills a CU's LDS, so workgroup
    // number 257 waits for a whole round: 56 heads x 4 splits 15.1 us, x 5 splits 22.3 us), at most 8
    // (28 heads, replayed as a HIP graph so that only GPU time counts: 69 tiles 12.6 us with 6 splits and
    // 12.15 us with 8, 137 tiles 16.85 -> 15.2 us, 261 tiles 20.3 -> 18.5 us), and a minimum of tiles per
    // workgroup (below).  Batch-1 shapes are pure latency and a wave with
    // one or two tiles beats a longer chain (28/4 heads x 4352 keys: 17.2 -> 15.0 us with 6 or 7 splits
    // instead of 4).  From 129 heads on there is one workgroup per head.
    int n_split = kNumCUs / heads;
    const int most = 8;
    if (n_split > most) n_split = most;
    // A split costs fp32 partials and a second launch of about 4 us: with up to 32 heads (where three or
    // more splits fit) seven tiles per workgroup repay it, one tile per wave or two (32 heads x 21 tiles,
    // sparse step 12.1 -> 11.6 us, dense step over 41 tiles 14.0 -> 12.9 us with 3 splits); from 64 heads
    // on it takes eleven (128 heads x 21 tiles: 14.5 us unsplit, 15.9 us with 2 splits).
    const int max_split = tiles / (heads <= 32 ? 7 : 11);
    if (n_split > max_split) n_split = max_split;
    if (n_split < 1) n_split = 1;
    pl.tiles_per_split = (tiles + n_split - 1) / n_split;
    pl.waves = pl.tiles_per_split < kMaxWavesPerWg ? pl.tiles_per_split : kMaxWavesPerWg;
    // split workgroups: two tiles per wave when there are fewer than sixteen (28 heads x 69 tiles in 6
    // splits: 12.6 -> 12.35 us with six waves instead of eight; the in-workgroup merge is smaller)
    if (n_split > 1) { const int w2 = (pl.tiles_per_split + 1) / 2; pl.waves = w2 < kMaxWavesPerWg ? w2 : kMaxWavesPerWg; }
    // One workgroup per head: fewer, longer-running waves measured faster than eight (smaller merge at
    // the end, 40-48 KB instead of 64 KB of loads in flight per CU).  With more heads than CUs four
    // waves let two workgroups share a CU, so one streams while the other merges and writes, and no
    // workgroup waits for a second round (B=16 LLaDA shape: 94 -> 89 us; B=8: 47.5 -> 46.3 us with
    // five waves; 280 grouped-query heads, G = 7: 41.4 -> 36.0 us; 320 heads, G = 4: 48.6 -> 43.6 us).
    // With more than two heads per CU, two waves, so that four workgroups fit (544 heads, MHA:
    // 117.9 -> 106.0 us; 640 heads: 134.5 -> 113.8 us; 768 heads of G = 3: 88.8 -> 75.0 us).
    // Up to one head per CU the grouped-query heads keep eight waves: there they are short of
    // arithmetic throughput, not of bandwidth (B=8 Dream shape: 22 -> 26 us with fewer).
    if (n_split == 1) {
      const bool mha = s.n_q_heads == s.n_kv_heads;
      const int cap = heads > 2 * kNumCUs ? 2 : heads > kNumCUs ? 4 : (mha ? 5 : kMaxWavesPerWg);
      if (pl.waves > cap) pl.waves = cap;
    }
    pl.n_split = (tiles + pl.tiles_per_split - 1) / pl.tiles_per_split;   // no empty split
    if (pl.n_split > 1) {
      const size_t slots = (size_t)heads * pl.n_split;
      pl.part_o_bytes = align_up(slots * s.block_len * s.head_dim * sizeof(float));
      pl.part_ml_bytes = align_up(slots * 2 * s.block_len * sizeof(float));
    }
  }
  return pl;
}

// Whether the dense launch of a cache-update step can also leave the saliency scores: multi-head attention
// (one query head per KV head) on the one-workgroup-per-head kernel, no key splits, at least two waves.
bool fuses_columns(const AttnPlan& pl, const sdllm_shape_t& s) {
  return pl.mfma && !pl.gqa && pl.n_split == 1 && pl.waves >= 2 && s.n_q_heads == s.n_kv_heads;
}

// cand_ml != null (dense MFMA launches only): also emit the scoring pass's row statistics over the
// candidate keys, n_split partials per query row.
// deferred != null: when the keys are split over workgroups, leave the merge of the splits to the caller
// (it gets the launch parameters in *deferred and must run launch_compact_combine or launch_attn_combine on
// the same stream before the partials' workspace is reused); deferred->n_split == 1 says nothing is left.
int32_t run_attn(const sdllm_shape_t& s, const void* q, const KvSegment& a, const KvSegment& b, void* out, void* ws,
                 size_t ws_bytes, hipStream_t stream, float* cand_ml = nullptr, int cand0_end = 0, int cand1_begin = 0,
                 AttnParams* deferred = nullptr, float* score_out = nullptr, int score_stride = 0) {
  const AttnPlan pl = plan_attn(s, a.n, a.sr, b.n, b.sr);
  if (pl.ws_bytes() > 0 && (!ws || ws_bytes < pl.ws_bytes())) return SDLLM_ERR_WORKSPACE;
  AttnParams p{};
  p.q = q;
  p.out = out;
  p.seg[0] = a;
  p.seg[1] = b;
  p.q_sb = s.q_stride[0]; p.q_sh = s.q_stride[1]; p.q_sr = s.q_stride[2];
  p.o_sb = s.out_stride[0]; p.o_sh = s.out_stride[1]; p.o_sr = s.out_stride[2];
  p.batch = s.batch; p.hq = s.n_q_heads; p.hkv = s.n_kv_heads; p.group = s.n_q_heads / s.n_kv_heads;
  p.nq = s.block_len; p.d = s.head_dim;
  p.scale_log2 = scale_of(s) * kLog2e;
  p.n_split = pl.n_split; p.tiles_per_split = pl.tiles_per_split; p.waves = pl.waves;
  p.part_o = (float*)ws;
  p.part_ml = (float*)((char*)ws + pl.part_o_bytes);
  p.cand_ml = pl.mfma ? cand_ml : nullptr;
  p.cand0_end = cand0_end;
  p.cand1_begin = cand1_begin;
  // the column sweep rides on the statistics launch of the one-workgroup-per-head kernel (fuses_columns below)
  p.score_out = p.cand_ml ? score_out : nullptr;
  p.score_stride = score_stride;
  p.score_inv_count = 1.f / (float)(s.block_len * (s.n_q_heads / s.n_kv_heads));
  hipError_t e;
  if (pl.mfma) {
    e = pl.gqa ? launch_attn_gqa_mfma_bf16(p, stream) : launch_attn_mfma_bf16(p, stream);
    if (deferred) *deferred = p;
    if (e == hipSuccess && pl.n_split > 1 && !deferred) e = launch_attn_combine(p, s.dtype, stream);
  } else {
    e = launch_attn_simple(p, s.dtype, stream);
    if (deferred) deferred->n_split = 1;
  }
  return e == hipSuccess ? SDLLM_OK : SDLLM_ERR_HIP;
}

// ---------------------------------------------------------------- scoring planning
struct ScorePlan {
  bool mfma;
  int n_scored;       // candidates that get a score
  int n_part, tiles_per_part, waves;
  // workspace: scores, softmax row statistics and, for segments too long for one workgroup, the selection's
  // key buffer, thresholds, bin lists and chunk offsets
  size_t score_bytes, ml_bytes, keys_bytes, sorted_bytes, bins_bytes;
  size_t ws_bytes() const { return score_bytes + ml_bytes + keys_bytes + sorted_bytes + bins_bytes; }
};

// The ranked segments and the unconditional tail of the selection for this shape (Alg. 1 steps 8-10;
// Alg. 4 keeps the suffix whole).
void fill_segments(const sdllm_shape_t& s, const Counts& c, SelectParams& q) {
  q.rows = s.batch * s.n_kv_heads;
  q.n_cand = c.n_cand;
  q.k_total = c.k_total;
  q.pool_half = (s.pool_kernel - 1) / 2;
  q.avg_pool = s.pool_mode == SDLLM_AVG_POOL;
  q.block_off = s.block_off; q.block_len = s.block_len;
  if (s.evict_scope == SDLLM_EVICT_PREFIX_ONLY) {
    q.n_seg = 1;
    q.seg_begin[0] = 0; q.seg_len[0] = c.n_pre; q.seg_k[0] = c.k_pre; q.seg_out[0] = 0;
    q.tail_begin = c.n_pre; q.tail_len = c.n_suf; q.tail_out = c.k_pre;
  } else if (s.select_mode == SDLLM_PER_SEGMENT) {
    q.n_seg = 2;
    q.seg_begin[0] = 0; q.seg_len[0] = c.n_pre; q.seg_k[0] = c.k_pre; q.seg_out[0] = 0;
    q.seg_begin[1] = c.n_pre; q.seg_len[1] = c.n_suf; q.seg_k[1] = c.k_suf; q.seg_out[1] = c.k_pre;
  } else {
    q.n_seg = 1;
    q.seg_begin[0] = 0; q.seg_len[0] = c.n_cand; q.seg_k[0] = c.k_total; q.seg_out[0] = 0;
  }
}

ScorePlan plan_score(const sdllm_shape_t& s) {
  const Counts c = counts_of(s);
  ScorePlan pl{};
  pl.n_scored = s.evict_scope == SDLLM_EVICT_PREFIX_ONLY ? c.n_pre : c.n_cand;
  const size_t rows = (size_t)s.batch * s.n_kv_heads;
  pl.score_bytes = align_up(rows * c.n_cand * sizeof(float));
  {
    SelectParams q{};
    fill_segments(s, c, q);
    const SelectWorkspace sw = select_workspace(q);
    pl.keys_bytes = align_up(sw.keys * sizeof(uint32_t));
    pl.sorted_bytes = align_up(sw.sorted * sizeof(uint32_t));
    pl.bins_bytes = align_up(sw.bins * sizeof(uint32_t));
  }
  pl.mfma = s.dtype == SDLLM_BF16 && s.head_dim == 128 && s.block_len == 32 &&
            score_mfma_supports_group(s.n_q_heads / s.n_kv_heads) && seg_fits_u32(s.kv_stride[2], s.seq_len, 2);
  pl.n_part = 1;
  pl.tiles_per_part = 0;
  pl.waves = 1;
  if (pl.mfma) {
    const int n0 = pl.n_scored < c.n_pre ? pl.n_scored : c.n_pre;
    const int n1 = pl.n_scored - n0;
    int tiles = (n0 + kTileKeys - 1) / kTileKeys + (n1 + kTileKeys - 1) / kTileKeys;
    if (tiles < 1) tiles = 1;
    int waves_per_row = (int)((kNumCUs * kMaxWavesPerWg + rows - 1) / rows);
    if (waves_per_row > tiles) waves_per_row = tiles;
    if (waves_per_row < 1) waves_per_row = 1;
    pl.waves = waves_per_row < kMaxWavesPerWg ? waves_per_row : kMaxWavesPerWg;
    int n_part = (waves_per_row + pl.waves - 1) / pl.waves;
    // never a few workgroups more than there are CUs: with several heads' Q staged in LDS a CU holds
    // one scoring workgroup, and the extra ones would wait for a whole round
    if (rows < (size_t)kNumCUs && n_part > kNumCUs / (int)rows) n_part = kNumCUs / (int)rows;
    pl.tiles_per_part = (tiles + n_part - 1) / n_part;
    pl.n_part = (tiles + pl.tiles_per_part - 1) / pl.tiles_per_part;   // no empty part
  }
  pl.ml_bytes = align_up((size_t)s.batch * s.n_q_heads * pl.n_part * 2 * s.block_len * sizeof(float));
  return pl;
}

int32_t check_q(const sdllm_shape_t& s, const void* q) {
  if (!q || !aligned16(q) || !row_stride_ok(s.q_stride, s.head_dim)) return SDLLM_ERR_INVALID_ARG;
  return SDLLM_OK;
}

// Alg. 1 steps 2-10.  ext_ml != null: the softmax row statistics over the candidates were already
// produced (ext_parts partials per row) and only the column reduction and the selection run.
// scores_ready: the scores are in the workspace's score buffer already; only the selection runs.
int32_t score_select_impl(const sdllm_shape_t& s, const void* q_blk, const void* k_full, int32_t* idx_out,
                          float* pooled_out, float* score_out, void* ws, size_t ws_bytes, hipStream_t hs,
                          float* ext_ml, int ext_parts, bool scores_ready = false) {
  const Counts c = counts_of(s);
  const ScorePlan pl = plan_score(s);
  if (!ws || ws_bytes < pl.ws_bytes() || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return SDLLM_ERR_WORKSPACE;
  if (c.n_cand == 0) return SDLLM_OK;
  {
    SelectParams probe{};
    fill_segments(s, c, probe);
    for (int i = 0; i < probe.n_seg; ++i)
      if (probe.seg_len[i] > select_max_segment()) return SDLLM_ERR_UNSUPPORTED;   // beyond the selection's per-segment tables
  }

  char* at = (char*)ws;
  float* score = score_out ? score_out : (float*)at;
  at += pl.score_bytes;
  float* ml = (float*)at;
  at += pl.ml_bytes;
  uint32_t* keys = pl.keys_bytes ? (uint32_t*)at : nullptr;
  at += pl.keys_bytes;
  uint32_t* sorted = pl.sorted_bytes ? (uint32_t*)at : nullptr;
  at += pl.sorted_bytes;
  uint32_t* bins = pl.bins_bytes ? (uint32_t*)at : nullptr;

  ScoreParams sp{};
  sp.q = q_blk; sp.k = k_full;
  sp.q_sb = s.q_stride[0]; sp.q_sh = s.q_stride[1]; sp.q_sr = s.q_stride[2];
  sp.k_sb = s.kv_stride[0]; sp.k_sh = s.kv_stride[1]; sp.k_sr = s.kv_stride[2];
  sp.batch = s.batch; sp.hq = s.n_q_heads; sp.hkv = s.n_kv_heads; sp.group = s.n_q_heads / s.n_kv_heads;
  sp.nq = s.block_len; sp.d = s.head_dim;
  sp.block_off = s.block_off; sp.block_len = s.block_len;
  sp.n_cand = pl.n_scored;
  sp.score_stride = c.n_cand;
  sp.softmax = s.score_mode == SDLLM_SOFTMAX_MEAN;
  sp.scale = scale_of(s);
  sp.scale_log2 = sp.scale * kLog2e;
  sp.score = score;
  sp.n_part = pl.n_part; sp.tiles_per_part = pl.tiles_per_part; sp.waves = pl.waves;
  sp.part_ml = ext_ml ? ext_ml : ml;
  sp.n_stat_part = ext_ml ? ext_parts : pl.n_part;
  sp.skip_stats = ext_ml != nullptr;
  // scores_ready: the dense attention of this step already left the scores in the workspace's score buffer
  hipError_t e = scores_ready ? hipSuccess : pl.mfma ? launch_score_mfma_bf16(sp, hs) : launch_score_simple(sp, s.dtype, hs);
  if (e != hipSuccess) return SDLLM_ERR_HIP;

  SelectParams q{};
  fill_segments(s, c, q);
  q.score = score; q.pooled = pooled_out; q.idx = idx_out;
  q.keys = keys; q.sorted = sorted; q.bins = bins;
  e = launch_select(q, hs);
  return e == hipSuccess ? SDLLM_OK : SDLLM_ERR_HIP;
}

// Workspace of sdllm_block_step: [0, base) is shared by the attention partials and the scoring
// buffers (used one after the other on the stream); the fused row statistics of the cache-update
// step live behind it because they are written by the attention and read by the scoring.
// Argument checks and launch parameters of the gather (k_total > 0).
int32_t compact_params(const sdllm_shape_t& s, const void* k_full, const void* v_full, const int32_t* idx, void* k_cache,
                       void* v_cache, CompactParams& p) {
  if (!k_full || !v_full || !idx || !k_cache || !v_cache) return SDLLM_ERR_INVALID_ARG;
  if (!aligned16(k_full) || !aligned16(v_full) || !aligned16(k_cache) || !aligned16(v_cache))
    return SDLLM_ERR_INVALID_ARG;
  if (!row_stride_ok(s.kv_stride, s.head_dim) || !row_stride_ok(s.cache_stride, s.head_dim))
    return SDLLM_ERR_INVALID_ARG;
  const int es = elem_size(s.dtype);
  p.k = k_full; p.v = v_full; p.idx = idx; p.kc = k_cache; p.vc = v_cache;
  p.s_sb = s.kv_stride[0] * es; p.s_sh = s.kv_stride[1] * es; p.s_sr = s.kv_stride[2] * es;
  p.c_sb = s.cache_stride[0] * es; p.c_sh = s.cache_stride[1] * es; p.c_sr = s.cache_stride[2] * es;
  p.batch = s.batch; p.hkv = s.n_kv_heads; p.k_total = counts_of(s).k_total; p.seq_len = s.seq_len;
  p.row_bytes = s.head_dim * es;
  return SDLLM_OK;
}

// With split keys at the cache-update step the merge of the splits runs in the compaction's launch, so
// the attention partials stay alive through scoring and selection: those then work behind them (score_off).
struct BlockStepWs { size_t base, stats_bytes, score_off; int stats_parts; bool fuse, fuse_cols; };

BlockStepWs plan_block_step(const sdllm_shape_t& s) {
  const Counts c = counts_of(s);
  const AttnPlan dense = plan_attn(s, s.seq_len, s.kv_stride[2], 0, 0);
  const AttnPlan sparse = plan_attn(s, c.k_total, s.cache_stride[2], s.block_len, s.blk_stride[2]);
  const ScorePlan sc = plan_score(s);
  BlockStepWs w{};
  w.score_off = dense.mfma && dense.n_split > 1 && c.k_total > 0 ? align_up(dense.ws_bytes()) : 0;
  w.base = dense.ws_bytes();
  if (sparse.ws_bytes() > w.base) w.base = sparse.ws_bytes();
  if (w.score_off + sc.ws_bytes() > w.base) w.base = w.score_off + sc.ws_bytes();
  w.base = align_up(w.base);
  w.fuse = dense.mfma && sc.mfma && s.score_mode == SDLLM_SOFTMAX_MEAN && c.n_cand > 0;
  w.stats_parts = dense.n_split;
  w.fuse_cols = w.fuse && fuses_columns(dense, s);
  w.stats_bytes = w.fuse ? align_up((size_t)s.batch * s.n_q_heads * dense.n_split * 64 * sizeof(float)) : 0;
  return w;
}

}  // namespace

// ---------------------------------------------------------------- static scratch (sdllm_sparse_attn_noalloc)
// The array is part of the device image: one copy per GPU, at its own address, alive until the
// process ends.  In host code the name `scratch` is only a handle for hipGetSymbolAddress; kernels
// and launch parameters get the per-device address resolved here.  The declaration carries no `used`
// attribute on purpose: the compiler gives a static device variable that host code refers to external
// linkage in the device image, which is how the runtime finds it, and leaves a `used` one local (the
// runtime then aborts in hipGetSymbolAddress).
static __device__ __align__(256) unsigned char scratch[SDLLM_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Address of the current device's copy of `scratch` (resolved once per device, with that device current).
hipError_t static_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // concurrent first calls resolve the same address
  }
  *out = ptr;
  return hipSuccess;
}

}  // namespace

// ================================================================ exported functions
extern "C" {

const char* sdllm_error_string(int32_t status) {
  switch (status) {
    case SDLLM_OK: return "ok";
    case SDLLM_ERR_INVALID_ARG: return "invalid argument";
    case SDLLM_ERR_UNSUPPORTED: return "unsupported shape or type";
    case SDLLM_ERR_WORKSPACE: return "workspace missing or too small";
    case SDLLM_ERR_HIP: return "HIP launch failed";
    case SDLLM_ERR_STATIC_LIMIT: return "request exceeds the static scratch of sdllm_sparse_attn_noalloc";
    default: return "unknown status";
  }
}

int32_t sdllm_version(void) { return 100; }

int32_t sdllm_retained_count(const sdllm_shape_t* shape, int32_t* k_total, int32_t* k_pre, int32_t* k_suf) {
  const int32_t st = check_shape(shape);
  if (st != SDLLM_OK) return st;
  const Counts c = counts_of(*shape);
  if (k_total) *k_total = c.k_total;
  if (k_pre) *k_pre = c.k_pre;
  if (k_suf) *k_suf = c.k_suf;
  return SDLLM_OK;
}

int32_t sdllm_cache_state(int32_t step_in_block, int32_t delay, int32_t* state) {
  if (!state || step_in_block < 0 || delay < 0) return SDLLM_ERR_INVALID_ARG;
  *state = step_in_block > delay ? SDLLM_STATE_REUSE : (step_in_block == delay ? SDLLM_STATE_UPDATE : SDLLM_STATE_FULL);
  return SDLLM_OK;
}

int32_t sdllm_workspace_bytes(const sdllm_shape_t* shape, int32_t op, int32_t n_cached, size_t* bytes) {
  const int32_t st = check_shape(shape);
  if (st != SDLLM_OK) return st;
  if (!bytes) return SDLLM_ERR_INVALID_ARG;
  const sdllm_shape_t& s = *shape;
  size_t need = 0;
  switch (op) {
    case SDLLM_OP_SCORE_SELECT: need = plan_score(s).ws_bytes(); break;
    case SDLLM_OP_COMPACT_KV: need = 0; break;
    case SDLLM_OP_SPARSE_ATTN:
      if (n_cached < 0) return SDLLM_ERR_INVALID_ARG;
      need = plan_attn(s, n_cached, s.cache_stride[2], s.block_len, s.blk_stride[2]).ws_bytes();
      break;
    case SDLLM_OP_BLOCK_STEP: {
      const BlockStepWs w = plan_block_step(s);
      need = w.base + w.stats_bytes;
      break;
    }
    default: return SDLLM_ERR_INVALID_ARG;
  }
  *bytes = need > 0 ? need : kAlign;   // never zero, so callers can always allocate
  return SDLLM_OK;
}

int32_t sdllm_score_select(const sdllm_shape_t* shape, const void* q_blk, const void* k_full, int32_t* idx_out,
                           float* pooled_out, float* score_out, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_shape(shape);
  if (st != SDLLM_OK) return st;
  const sdllm_shape_t& s = *shape;
  if ((st = check_q(s, q_blk)) != SDLLM_OK) return st;
  if (!k_full || !aligned16(k_full) || !row_stride_ok(s.kv_stride, s.head_dim)) return SDLLM_ERR_INVALID_ARG;
  if (counts_of(s).k_total > 0 && !idx_out) return SDLLM_ERR_INVALID_ARG;
  return score_select_impl(s, q_blk, k_full, idx_out, pooled_out, score_out, ws, ws_bytes, (hipStream_t)stream, nullptr, 0);
}

int32_t sdllm_compact_kv(const sdllm_shape_t* shape, const void* k_full, const void* v_full, const int32_t* idx,
                         void* k_cache, void* v_cache, void* stream) {
  const int32_t st = check_shape(shape);
  if (st != SDLLM_OK) return st;
  if (counts_of(*shape).k_total == 0) return SDLLM_OK;
  CompactParams p{};
  const int32_t sp = compact_params(*shape, k_full, v_full, idx, k_cache, v_cache, p);
  if (sp != SDLLM_OK) return sp;
  return launch_compact(p, (hipStream_t)stream) == hipSuccess ? SDLLM_OK : SDLLM_ERR_HIP;
}

int32_t sdllm_sparse_attn(const sdllm_shape_t* shape, const void* q_blk, const void* k_cache, const void* v_cache,
                          int32_t n_cached, const void* k_blk, const void* v_blk, void* out, void* ws,
                          size_t ws_bytes, void* stream) {
  int32_t st = check_shape(shape);
  if (st != SDLLM_OK) return st;
  const sdllm_shape_t& s = *shape;
  if ((st = check_q(s, q_blk)) != SDLLM_OK) return st;
  if (n_cached < 0) return SDLLM_ERR_INVALID_ARG;
  if (n_cached > 0 && (!k_cache || !v_cache || !aligned16(k_cache) || !aligned16(v_cache) ||
                       !row_stride_ok(s.cache_stride, s.head_dim)))
    return SDLLM_ERR_INVALID_ARG;
  if (!k_blk || !v_blk || !out || !aligned16(k_blk) || !aligned16(v_blk) || !aligned16(out) ||
      !row_stride_ok(s.blk_stride, s.head_dim) || !row_stride_ok(s.out_stride, s.head_dim))
    return SDLLM_ERR_INVALID_ARG;
  KvSegment a{k_cache, v_cache, s.cache_stride[0], s.cache_stride[1], s.cache_stride[2], n_cached};
  KvSegment b{k_blk, v_blk, s.blk_stride[0], s.blk_stride[1], s.blk_stride[2], s.block_len};
  return run_attn(s, q_blk, a, b, out, ws, ws_bytes, (hipStream_t)stream);
}

int32_t sdllm_sparse_attn_noalloc(const sdllm_shape_t* shape, const void* q_blk, const void* k_cache,
                                  const void* v_cache, int32_t n_cached, const void* k_blk, const void* v_blk,
                                  void* out, void* stream) {
  const int32_t st = check_shape(shape);
  if (st != SDLLM_OK) return st;
  if (n_cached < 0) return SDLLM_ERR_INVALID_ARG;
  const sdllm_shape_t& s = *shape;
  const size_t need = plan_attn(s, n_cached, s.cache_stride[2], s.block_len, s.blk_stride[2]).ws_bytes();
  if (need > SDLLM_STATIC_SCRATCH_BYTES) return SDLLM_ERR_STATIC_LIMIT;
  void* ptr = nullptr;
  if (static_scratch(&ptr) != hipSuccess) return SDLLM_ERR_HIP;
  return sdllm_sparse_attn(shape, q_blk, k_cache, v_cache, n_cached, k_blk, v_blk, out, ptr, SDLLM_STATIC_SCRATCH_BYTES, stream);
}

int32_t sdllm_block_step(const sdllm_shape_t* shape, int32_t step_in_block, int32_t delay, const void* q_blk,
                         const void* k_in, const void* v_in, int32_t* idx, void* k_cache, void* v_cache, void* out,
                         void* ws, size_t ws_bytes, void* stream, int32_t* state_out) {
  int32_t st = check_shape(shape);
  if (st != SDLLM_OK) return st;
  const sdllm_shape_t& s = *shape;
  int32_t state;
  if ((st = sdllm_cache_state(step_in_block, delay, &state)) != SDLLM_OK) return st;
  size_t need;
  if ((st = sdllm_workspace_bytes(shape, SDLLM_OP_BLOCK_STEP, 0, &need)) != SDLLM_OK) return st;
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return SDLLM_ERR_WORKSPACE;
  if ((st = check_q(s, q_blk)) != SDLLM_OK) return st;
  if (!k_in || !v_in || !out || !aligned16(k_in) || !aligned16(v_in) || !aligned16(out) ||
      !row_stride_ok(s.out_stride, s.head_dim))
    return SDLLM_ERR_INVALID_ARG;
  const Counts c = counts_of(s);
  if (state_out) *state_out = state;

  if (state == SDLLM_STATE_REUSE) {
    return sdllm_sparse_attn(shape, q_blk, k_cache, v_cache, c.k_total, k_in, v_in, out, ws, ws_bytes, stream);
  }
  // states 0/1: the block's rows of dense attention over all L keys of this step
  if (!row_stride_ok(s.kv_stride, s.head_dim)) return SDLLM_ERR_INVALID_ARG;
  if (state == SDLLM_STATE_UPDATE && c.k_total > 0 && (!idx || !k_cache || !v_cache)) return SDLLM_ERR_INVALID_ARG;
  KvSegment a{k_in, v_in, s.kv_stride[0], s.kv_stride[1], s.kv_stride[2], s.seq_len};
  KvSegment b{nullptr, nullptr, 0, 0, 0, 0};
  const BlockStepWs w = plan_block_step(s);
  AttnParams pending{};           // split-KV merge still to run (cache-update step only)
  pending.n_split = 1;
  AttnParams* defer = state == SDLLM_STATE_UPDATE && w.score_off > 0 ? &pending : nullptr;
  if (state == SDLLM_STATE_FULL || !w.fuse)
    st = run_attn(s, q_blk, a, b, out, ws, ws_bytes, (hipStream_t)stream, nullptr, 0, 0, defer);
  else {
    // cache-update step: the dense attention also leaves the scoring softmax's row statistics
    const int cand1 = s.evict_scope == SDLLM_EVICT_PREFIX_ONLY ? s.seq_len : s.block_off + s.block_len;
    // ... and, where one workgroup owns a head, the saliency scores themselves (first buffer of the scoring workspace)
    st = run_attn(s, q_blk, a, b, out, ws, w.base, (hipStream_t)stream, (float*)((char*)ws + w.base), s.block_off, cand1,
                  defer, w.fuse_cols ? (float*)((char*)ws + w.score_off) : nullptr, c.n_cand);
  }
  if (st != SDLLM_OK || state == SDLLM_STATE_FULL) return st;
  // from here on a pending merge must run whatever else fails: `out` is not complete without it
  auto finish_pending = [&](int32_t status) {
    if (pending.n_split > 1 && launch_attn_combine(pending, s.dtype, (hipStream_t)stream) != hipSuccess && status == SDLLM_OK)
      return (int32_t)SDLLM_ERR_HIP;
    return status;
  };
  if (!row_stride_ok(s.q_stride, s.head_dim)) return finish_pending(SDLLM_ERR_INVALID_ARG);
  st = score_select_impl(s, q_blk, k_in, idx, nullptr, nullptr, (char*)ws + w.score_off, w.base - w.score_off,
                         (hipStream_t)stream, w.fuse ? (float*)((char*)ws + w.base) : nullptr, w.stats_parts, w.fuse_cols);
  if (st != SDLLM_OK) return finish_pending(st);
  if (pending.n_split == 1) return sdllm_compact_kv(shape, k_in, v_in, idx, k_cache, v_cache, stream);
  CompactParams cp{};
  if ((st = compact_params(s, k_in, v_in, idx, k_cache, v_cache, cp)) != SDLLM_OK) return finish_pending(st);
  return launch_compact_combine(cp, pending, (hipStream_t)stream) == hipSuccess ? SDLLM_OK : SDLLM_ERR_HIP;
}

int32_t sdllm_dense_attn(const sdllm_shape_t* shape, const void* q_full, const int64_t* q_full_stride,
                         const void* k_full, const void* v_full, void* out_full, const int64_t* out_full_stride,
                         void* stream) {
  const int32_t st = check_shape(shape);
  if (st != SDLLM_OK) return st;
  const sdllm_shape_t& s = *shape;
  if (!q_full || !k_full || !v_full || !out_full || !q_full_stride || !out_full_stride) return SDLLM_ERR_INVALID_ARG;
  if (!aligned16(q_full) || !aligned16(k_full) || !aligned16(v_full) || !aligned16(out_full)) return SDLLM_ERR_INVALID_ARG;
  const int es = elem_size(s.dtype);
  if (!strides_ok(q_full_stride, es) || !strides_ok(out_full_stride, es) || !row_stride_ok(q_full_stride, s.head_dim) ||
      !row_stride_ok(out_full_stride, s.head_dim) || !row_stride_ok(s.kv_stride, s.head_dim))
    return SDLLM_ERR_INVALID_ARG;
  const float scale_log2 = scale_of(s) * kLog2e;
  hipError_t e;
  if (s.dtype == SDLLM_BF16 && s.head_dim == 128 && seg_fits_u32(s.kv_stride[2], s.seq_len, 2)) {
    DenseFullParams p{};
    p.q = q_full; p.k = k_full; p.v = v_full; p.out = out_full;
    p.q_sb = q_full_stride[0]; p.q_sh = q_full_stride[1]; p.q_sr = q_full_stride[2];
    p.k_sb = s.kv_stride[0]; p.k_sh = s.kv_stride[1]; p.k_sr = s.kv_stride[2];
    p.o_sb = out_full_stride[0]; p.o_sh = out_full_stride[1]; p.o_sr = out_full_stride[2];
    p.batch = s.batch; p.hq = s.n_q_heads; p.hkv = s.n_kv_heads; p.group = s.n_q_heads / s.n_kv_heads;
    p.seq_len = s.seq_len; p.d = s.head_dim;
    p.scale_log2 = scale_log2;
    e = launch_dense_full_mfma_bf16(p, (hipStream_t)stream);
  } else {
    // generic path: one wave per query row over a single key segment
    AttnParams p{};
    p.q = q_full; p.out = out_full;
    p.seg[0] = KvSegment{k_full, v_full, s.kv_stride[0], s.kv_stride[1], s.kv_stride[2], s.seq_len};
    p.seg[1] = KvSegment{nullptr, nullptr, 0, 0, 0, 0};
    p.q_sb = q_full_stride[0]; p.q_sh = q_full_stride[1]; p.q_sr = q_full_stride[2];
    p.o_sb = out_full_stride[0]; p.o_sh = out_full_stride[1]; p.o_sr = out_full_stride[2];
    p.batch = s.batch; p.hq = s.n_q_heads; p.hkv = s.n_kv_heads; p.group = s.n_q_heads / s.n_kv_heads;
    p.nq = s.seq_len; p.d = s.head_dim;
    p.scale_log2 = scale_log2;
    p.n_split = 1; p.waves = 1;
    e = launch_attn_simple(p, s.dtype, (hipStream_t)stream);
  }
  return e == hipSuccess ? SDLLM_OK : SDLLM_ERR_HIP;
}

int32_t sdllm_stream_read_probe(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !aligned16(src)) return SDLLM_ERR_INVALID_ARG;
  return launch_stream_read(src, bytes, (uint32_t*)sink, (hipStream_t)stream) == hipSuccess ? SDLLM_OK : SDLLM_ERR_HIP;
}

}  // extern "C"
