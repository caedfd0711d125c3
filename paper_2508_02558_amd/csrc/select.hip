// Pooling + top-k retention (Sec. 3.3 third equation; Alg. 1 steps 8-10).
//
// Per (batch, KV head) row and ranked segment (prefix / suffix, or the joint array):
//   1. pooling: stride-1 pooling of the score with window s clipped to the segment (-inf padding for
//      max, zero padding and a fixed divisor s for avg); a pooled value is handled as its
//      order-preserving 32-bit integer key (larger float <=> larger key);
//   2. threshold: an MSB-first radix select on the keys finds the exact k-th largest value T and how
//      many entries equal to T have to be kept (k minus the number of larger ones);
//   3. emission: in position order, every key above T and the first entries equal to T are kept, so
//      ties go to the lower position and the output is ascending without a sort.
// Max pooling copies a peak to its neighbours, so T routinely falls inside a group of equal values;
// the tie rule is exercised constantly, not only in corner cases.
//
// Segments of up to 8 x 1024 candidates: one 1024-thread workgroup does all three stages with the keys
// in registers (select_kernel: the score row is read from memory exactly once; four 8-bit radix passes
// with LDS histograms; emission by counting every (chunk, wave) cell, one scan of the cell counts, then
// the writes).
// Longer segments are spread over the machine in three launches:
//   select_pool_kernel     one workgroup per 2048 candidates: pooling, keys to a key buffer, and a compact
//                          list of the non-empty bins of the keys' leading 12 bits;
//   select_resolve_kernel  one workgroup per segment: adds the lists up, finds the bin that holds the k-th
//                          value, collects that bin's members (a few hundred keys as a rule) and resolves
//                          the remaining 20 bits on them alone; then one sweep over the keys leaves, per
//                          1024 candidates, how many entries above and equal to T precede them;
//   select_emit_kernel     one workgroup per 1024 candidates: position-ordered emission from those counts.
#include "sdllm_internal.h"

namespace sdllm {

#ifdef SDLLM_TUNING   // development builds only: timestamps of one workgroup's phases
__device__ unsigned long long g_dbg[32];
#define DBG_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0) g_dbg[i] = wall_clock64(); } while (0)
#else
#define DBG_STAMP(i) do { } while (0)
#endif

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelRegItems = 8;                        // longest register-resident variant (chunks of 1024)
constexpr int kPoolChunks = 2;                         // chunks of 1024 candidates per select_pool_kernel workgroup
constexpr int kPartLen = kPoolChunks * kSelThreads;
constexpr int kBinShift = 20, kBins = 4096;            // leading 12 bits of a key
constexpr int kBinListCap = kPartLen;                  // a part cannot occupy more bins than it has candidates
static_assert(kBinListCap >= 256, "select_resolve_kernel reads the first 256 pairs of every list unconditionally");
constexpr int kBinListStride = 1 + 2 * kBinListCap;    // words per list: count, then (bin, count) pairs
constexpr int kSweep = 32;                            // keys a thread of select_resolve_kernel loads per trip to memory
constexpr int kMemberCap = 8192;                       // members of the threshold bin held in LDS by select_resolve_kernel
constexpr int kEmitThreads = 256;
constexpr int kEmitWaves = kEmitThreads / 64;
constexpr int kEmitItems = 4;
constexpr int kEmitChunk = kEmitThreads * kEmitItems;  // candidates per select_emit_kernel workgroup
static_assert(kEmitChunk == kSelThreads, "select_resolve_kernel counts per chunk of kSelThreads candidates");

__device__ __forceinline__ uint32_t order_key(float v) {
  const uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);   // larger float <=> larger key
}

__device__ __forceinline__ int cand_pos(int c, int block_off, int block_len) {
  return c < block_off ? c : c + block_len;
}

__device__ __forceinline__ float pool_at(const float* score, int c, int len, int half, int avg, float inv_s) {
  const int lo = max(0, c - half), hi = min(len - 1, c + half);
  float v;
  if (avg) {
    v = 0.f;
    for (int j = lo; j <= hi; ++j) v += score[j];
    v *= inv_s;
  } else {
    v = -INFINITY;
    for (int j = lo; j <= hi; ++j) v = fmaxf(v, score[j]);
  }
  return v + 0.f;   // -0 -> +0 so that equal values have equal keys
}

// Histogram building.  A thread walks its keys and counts runs of equal bins in registers (pooled
// softmax scores share their leading bits, so in the first pass a thread's whole walk is usually one
// run); a run ends with one LDS atomic.  The last run of every lane is flushed together: when all
// active lanes of the wave hold the same bin - again the common first-pass case, where 64 atomics on
// one address would serialise - the counts are summed across the wave and added by one lane.
struct BinRun {
  uint32_t bin = 0xffffffffu, count = 0;
};

__device__ __forceinline__ void run_add(uint32_t* hist, BinRun& r, bool active, uint32_t bin) {
  if (!active) return;
  if (bin == r.bin) {
    ++r.count;
  } else {
    if (r.count) atomicAdd(&hist[r.bin], r.count);
    r.bin = bin;
    r.count = 1;
  }
}

__device__ __forceinline__ void run_flush(uint32_t* hist, const BinRun& r, int lane) {
  const bool active = r.count != 0;
  const uint64_t act = __ballot(active);
  if (act == 0) return;
  const int leader = __ffsll((long long)act) - 1;
  const uint32_t lead_bin = (uint32_t)__builtin_amdgcn_readlane((int)r.bin, leader);
  const uint64_t same = __ballot(active && r.bin == lead_bin);
  if (same == act) {
    uint32_t total = r.count;   // 0 in idle lanes
    for (int o = 32; o > 0; o >>= 1) total += __shfl_xor(total, o);
    if (lane == leader) atomicAdd(&hist[lead_bin], total);
  } else if (active) {
    atomicAdd(&hist[r.bin], r.count);
  }
}

// Whole-wave shifts by one lane as DPP moves (no LDS traffic, unlike a general shuffle):
// shr: lane i takes v[i-1], lane 0 takes `fill`; shl: lane i takes v[i+1], lane 63 takes `fill`.
__device__ __forceinline__ float wave_shr1(float v, float fill) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, fill), __builtin_bit_cast(int, v),
                                                               0x138, 0xF, 0xF, false));
}
__device__ __forceinline__ float wave_shl1(float v, float fill) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, fill), __builtin_bit_cast(int, v),
                                                               0x130, 0xF, 0xF, false));
}
__device__ __forceinline__ float lane_value(float v, int src_lane) {   // src_lane: compile-time constant
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src_lane));
}

// Wave 0, after a pass's 256-bin histogram is complete: the bin that holds the `remaining`-th largest
// active key and the number of keys in higher bins (four bins per lane).
__device__ __forceinline__ void pick_bin(const uint32_t* h, uint32_t remaining, int lane, uint32_t* s_bin, uint32_t* s_above) {
  const uint32_t h0 = h[4 * lane], h1 = h[4 * lane + 1], h2 = h[4 * lane + 2], h3 = h[4 * lane + 3];
  const uint32_t lane_sum = h0 + h1 + h2 + h3;
  uint32_t suf = lane_sum;   // inclusive suffix sum over lanes
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_down(suf, o);
    if (lane + o < 64) suf += t;
  }
  const uint32_t a3 = suf - lane_sum, a2 = a3 + h3, a1 = a2 + h2, a0 = a1 + h1;
  if (a3 < remaining && remaining <= a3 + h3) { *s_bin = 4 * lane + 3; *s_above = a3; }
  if (a2 < remaining && remaining <= a2 + h2) { *s_bin = 4 * lane + 2; *s_above = a2; }
  if (a1 < remaining && remaining <= a1 + h1) { *s_bin = 4 * lane + 1; *s_above = a1; }
  if (a0 < remaining && remaining <= a0 + h0) { *s_bin = 4 * lane; *s_above = a0; }
}

// The same over the kBins-bin histogram of the keys' leading bits, by all 1024 threads (four bins per
// thread).  One workgroup barrier inside; the caller synchronises before (histogram complete) and after.
__device__ __forceinline__ void pick_bin_wide(const uint32_t* h, uint32_t remaining, int tid, int lane, int wave,
                                              uint32_t* wave_tot, uint32_t* s_bin, uint32_t* s_above) {
  const uint32_t h0 = h[4 * tid], h1 = h[4 * tid + 1], h2 = h[4 * tid + 2], h3 = h[4 * tid + 3];
  const uint32_t mine = h0 + h1 + h2 + h3;
  uint32_t suf = mine;   // inclusive suffix sum over the lanes of this wave
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_down(suf, o);
    if (lane + o < 64) suf += t;
  }
  if (lane == 0) wave_tot[wave] = suf;
  __syncthreads();
  uint32_t above_waves = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w)
    if (w > wave) above_waves += wave_tot[w];
  const uint32_t a3 = above_waves + suf - mine, a2 = a3 + h3, a1 = a2 + h2, a0 = a1 + h1;
  if (a3 < remaining && remaining <= a3 + h3) { *s_bin = 4 * tid + 3; *s_above = a3; }
  if (a2 < remaining && remaining <= a2 + h2) { *s_bin = 4 * tid + 2; *s_above = a2; }
  if (a1 < remaining && remaining <= a1 + h1) { *s_bin = 4 * tid + 1; *s_above = a1; }
  if (a0 < remaining && remaining <= a0 + h0) { *s_bin = 4 * tid; *s_above = a0; }
}

// Pooled values of U consecutive chunks (it0 .. it0+U-1) of a segment, element c = it*1024 + tid:
// own values first, plus one extra load per chunk in which lanes 0..HALF-1 fetch the HALF candidates
// left of the wave's 64 and lanes HALF..2*HALF-1 the HALF right of them (every load is unconditional
// and independent, so all 2U loads of a thread are in flight together); the window then comes from
// whole-wave shifts.  Same arithmetic as pool_at, term for term.  len >= 1.
template <int U, int HALF>
__device__ __forceinline__ void pool_chunks(const float* score, int len, int it0, int tid, int lane, int avg, float inv_s,
                                            float (&pv)[U]) {
  const float pad = avg ? 0.f : -INFINITY;
  float v[U], edge[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int c = (it0 + u) * kSelThreads + tid;
    v[u] = c < len ? score[c] : pad;
    edge[u] = pad;
    if (HALF > 0) {
      const int first = c - lane;                                           // the wave's first candidate of this chunk
      const int ce = lane < HALF ? first - HALF + lane : first + 64 + (lane - HALF);
      const bool want = lane < 2 * HALF && ce >= 0 && ce < len;
      const float x = score[want ? ce : (c < len ? c : 0)];                   // lanes with nothing to fetch re-read a valid address
      edge[u] = want ? x : pad;
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float win[2 * (HALF > 0 ? HALF : 0) + 1];   // window in ascending position order
    win[HALF > 0 ? HALF : 0] = v[u];
    // k-th neighbour = the (k-1)-th neighbour's array shifted by one more lane; the value that
    // enters at the wave's edge is the matching out-of-wave candidate (edge lanes HALF-k / HALF+k-1)
    float l = v[u], r = v[u];
#pragma unroll
    for (int k = 1; k <= HALF; ++k) {
      l = wave_shr1(l, lane_value(edge[u], HALF - k));
      r = wave_shl1(r, lane_value(edge[u], HALF + k - 1));
      win[HALF - k] = l;
      win[HALF + k] = r;
    }
    float x;
    if (avg) {
      x = 0.f;
#pragma unroll
      for (int j = 0; j < 2 * HALF + 1; ++j) x += win[j];
      x *= inv_s;
    } else {
      x = win[0];
#pragma unroll
      for (int j = 1; j < 2 * HALF + 1; ++j) x = fmaxf(x, win[j]);
    }
    pv[u] = x + 0.f;   // -0 -> +0 so that equal values have equal keys
  }
}

// The pair the emission of a long segment reads per (row, ranked segment): threshold key and number of
// equal keys to keep.  "keep everything" is (0, len): every key is above or equal to 0; "keep nothing"
// is (max, 0).
__device__ __forceinline__ void publish_threshold(uint32_t* thr, int row, int seg, uint32_t key, uint32_t need_eq) {
  thr[(row * 2 + seg) * 2] = key;
  thr[(row * 2 + seg) * 2 + 1] = need_eq;
}

// Exclusive scan, in place, of the n_cells (<= 1024) per-cell counts of the emission pass; cell
// it*16 + wave is the 64 candidates wave `wave` holds in chunk `it`, so index order is position order.
// Two workgroup barriers inside; the caller synchronises before (counts written) and may read after.
__device__ __forceinline__ void scan_cells(uint32_t* cell_gt, uint32_t* cell_eq, int n_cells, uint32_t* wave_gt, uint32_t* wave_eq,
                                           int tid, int lane, int wave) {
  const uint32_t g = tid < n_cells ? cell_gt[tid] : 0u, e = tid < n_cells ? cell_eq[tid] : 0u;
  uint32_t sg = g, se = e;
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t tg = __shfl_up(sg, o), te = __shfl_up(se, o);
    if (lane >= o) { sg += tg; se += te; }
  }
  if (lane == 63) { wave_gt[wave] = sg; wave_eq[wave] = se; }
  __syncthreads();
  uint32_t og = 0, oe = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w)
    if (w < wave) { og += wave_gt[w]; oe += wave_eq[w]; }
  if (tid < n_cells) { cell_gt[tid] = og + sg - g; cell_eq[tid] = oe + se - e; }
  __syncthreads();
}

// ------------------------------------------------------------------ short segments: all three stages in one workgroup
// blockIdx.x >= n_seg is the unconditional tail (prefix-only eviction keeps the whole suffix).
template <int ITEMS, int HALF>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectParams p) {
  constexpr int kCells = ITEMS * kSelWaves;   // (chunk, wave) cells of the emission pass
  __shared__ uint32_t hist[4][256];
  __shared__ uint32_t wave_gt[kSelWaves], wave_eq[kSelWaves];
  __shared__ uint32_t cell_gt[kCells], cell_eq[kCells];
  __shared__ uint32_t s_bin, s_above;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int row = blockIdx.y;
  const int seg = blockIdx.x;
  int32_t* idx_row = p.idx + (size_t)row * p.k_total;

  if (seg >= p.n_seg) {   // candidates kept unconditionally
    for (int j = tid; j < p.tail_len; j += kSelThreads)
      idx_row[p.tail_out + j] = cand_pos(p.tail_begin + j, p.block_off, p.block_len);
    return;
  }

  const int begin = p.seg_begin[seg];
  const int len = p.seg_len[seg];
  const int k = p.seg_k[seg];
  if (len <= 0) return;   // an empty segment (no suffix after the last block, no prefix before the first): no load at all
  const float* score = p.score + (size_t)row * p.n_cand + begin;
  float* pooled = p.pooled ? p.pooled + (size_t)row * p.n_cand + begin : nullptr;
  int32_t* out = idx_row + p.seg_out[seg];

  // 1. pooling
  const int half = p.pool_half;
  const float inv_s = 1.f / (float)(2 * half + 1);
  uint32_t keys[ITEMS];
  float pv[ITEMS];
  if (HALF >= 0) {
    pool_chunks<ITEMS, (HALF >= 0 ? HALF : 0)>(score, len, 0, tid, lane, p.avg_pool, inv_s, pv);
  } else {
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int c = it * kSelThreads + tid;
      pv[it] = c < len ? pool_at(score, c, len, half, p.avg_pool, inv_s) : 0.f;
    }
  }
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {
    const int c = it * kSelThreads + tid;
    keys[it] = 0;
    if (c < len) {
      keys[it] = order_key(pv[it]);
      if (pooled) pooled[c] = pv[it];
    }
  }
  if (k <= 0) return;
  if (k >= len) {
    for (int c = tid; c < len; c += kSelThreads) out[c] = cand_pos(begin + c, p.block_off, p.block_len);
    return;
  }
  for (int i = tid; i < 4 * 256; i += kSelThreads) (&hist[0][0])[i] = 0;
  __syncthreads();

  // 2. radix select: after the loop `prefix` is the key of the k-th largest value and
  //    `remaining` the number of values equal to it that must be kept
  uint32_t prefix = 0, mask = 0, remaining = (uint32_t)k;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    BinRun run;
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int c = it * kSelThreads + tid;
      run_add(hist[pass], run, c < len && (keys[it] & mask) == prefix, (keys[it] >> shift) & 255u);
    }
    run_flush(hist[pass], run, lane);
    __syncthreads();
    if (wave == 0) pick_bin(hist[pass], remaining, lane, &s_bin, &s_above);
    __syncthreads();
    prefix |= s_bin << shift;
    mask |= 255u << shift;
    remaining -= s_above;
  }
  const uint32_t thr = prefix;
  const uint32_t need_eq = remaining;

  // 3. position-ordered emission: cell (it, wave) = the 64 candidates wave `wave` holds in chunk `it`;
  //    cells in index order it*16 + wave are in position order.  Count, scan the cells once, then write.
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  uint32_t my_gt = 0, my_eq = 0;   // lane `it` keeps the counts of cell (it, wave)
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {
    const int c = it * kSelThreads + tid;
    const uint64_t b_gt = __ballot(c < len && keys[it] > thr), b_eq = __ballot(c < len && keys[it] == thr);
    if (lane == it) { my_gt = __popcll(b_gt); my_eq = __popcll(b_eq); }
  }
  if (lane < ITEMS) { cell_gt[lane * kSelWaves + wave] = my_gt; cell_eq[lane * kSelWaves + wave] = my_eq; }
  __syncthreads();
  scan_cells(cell_gt, cell_eq, kCells, wave_gt, wave_eq, tid, lane, wave);
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {
    const int c = it * kSelThreads + tid;
    const bool gt = c < len && keys[it] > thr;
    const bool eq = c < len && keys[it] == thr;
    const uint64_t b_gt = __ballot(gt), b_eq = __ballot(eq);
    const uint32_t gt_before = cell_gt[it * kSelWaves + wave] + __popcll(b_gt & lt_mask);
    const uint32_t eq_before = cell_eq[it * kSelWaves + wave] + __popcll(b_eq & lt_mask);
    if (gt) out[gt_before + min(eq_before, need_eq)] = cand_pos(begin + c, p.block_off, p.block_len);
    else if (eq && eq_before < need_eq) out[gt_before + eq_before] = cand_pos(begin + c, p.block_off, p.block_len);
  }
}

// ------------------------------------------------------------------ stage 1 of long segments, one workgroup per 2048 candidates
template <int HALF>
__global__ __launch_bounds__(kSelThreads) void select_pool_kernel(const SelectParams p) {
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t wave_cnt[kSelWaves];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int part = blockIdx.x;
  const int seg = blockIdx.y;
  const int row = blockIdx.z;
  const int begin = p.seg_begin[seg];
  const int len = p.seg_len[seg];
  const int k = p.seg_k[seg];
  const int c_first = part * kPartLen;
  if (c_first >= len) return;   // a shorter (or empty) segment has fewer parts
  const float* score = p.score + (size_t)row * p.n_cand + begin;
  float* pooled = p.pooled ? p.pooled + (size_t)row * p.n_cand + begin : nullptr;
  uint32_t* key_out = p.keys + (size_t)row * p.n_cand + begin;

  const int half = p.pool_half;
  const float inv_s = 1.f / (float)(2 * half + 1);
  float pv[kPoolChunks];
  if (HALF >= 0) {
    pool_chunks<kPoolChunks, (HALF >= 0 ? HALF : 0)>(score, len, part * kPoolChunks, tid, lane, p.avg_pool, inv_s, pv);
  } else {
#pragma unroll
    for (int u = 0; u < kPoolChunks; ++u) {
      const int c = c_first + u * kSelThreads + tid;
      pv[u] = c < len ? pool_at(score, c, len, half, p.avg_pool, inv_s) : 0.f;
    }
  }
  uint32_t keys[kPoolChunks];
#pragma unroll
  for (int u = 0; u < kPoolChunks; ++u) {
    const int c = c_first + u * kSelThreads + tid;
    keys[u] = 0;
    if (c < len) {
      keys[u] = order_key(pv[u]);
      key_out[c] = keys[u];
      if (pooled) pooled[c] = pv[u];
    }
  }
  if (k <= 0 || k >= len) return;   // nothing to rank: stage 2 publishes keep-nothing / keep-everything

  // histogram of the keys' leading bits, then the list of its non-empty bins
  for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
  __syncthreads();
  BinRun run;
#pragma unroll
  for (int u = 0; u < kPoolChunks; ++u) run_add(hist, run, c_first + u * kSelThreads + tid < len, keys[u] >> kBinShift);
  run_flush(hist, run, lane);
  __syncthreads();
  uint32_t h[4];
  uint32_t n = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    h[j] = hist[4 * tid + j];
    n += h[j] != 0;
  }
  uint32_t incl = n;   // inclusive prefix sum over the lanes of this wave
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_up(incl, o);
    if (lane >= o) incl += t;
  }
  if (lane == 63) wave_cnt[wave] = incl;
  __syncthreads();
  uint32_t at = incl - n;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w)
    if (w < wave) at += wave_cnt[w];
  uint32_t* list = p.bins + ((size_t)(row * 2 + seg) * p.parts + part) * kBinListStride;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (h[j] != 0) {   // at most kPartLen non-empty bins, so at < kBinListCap
      list[1 + 2 * at] = 4 * tid + j;
      list[2 + 2 * at] = h[j];
      ++at;
    }
  if (tid == kSelThreads - 1) list[0] = at;
}

// ------------------------------------------------------------------ stage 2 of long segments, one workgroup per segment
// One workgroup is one CU: a sweep over all keys of a 32k-candidate segment is bound by instruction issue
// (sixteen waves on four SIMDs), so the two sweeps below spend a handful of instructions per 64 keys: no
// bounds checks in full sweeps, counts taken from wave-wide compares (the popcount is scalar work), one LDS
// atomic per wave and sweep (members) or none at all (chunk counts).

// The bin that holds the `remaining`-th largest key of a 1024-bin histogram and the number of keys in
// higher bins, by all 1024 threads (one bin each).  One workgroup barrier inside; the caller synchronises
// before (histogram complete) and after.
__device__ __forceinline__ void pick_bin_1024(const uint32_t* h, uint32_t remaining, int tid, int lane, int wave,
                                              uint32_t* wave_tot, uint32_t* s_bin, uint32_t* s_above) {
  const uint32_t mine = h[tid];
  uint32_t suf = mine;   // inclusive suffix sum over the lanes of this wave
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_down(suf, o);
    if (lane + o < 64) suf += t;
  }
  if (lane == 0) wave_tot[wave] = suf;
  __syncthreads();
  uint32_t above = suf - mine;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w)
    if (w > wave) above += wave_tot[w];
  if (above < remaining && remaining <= above + mine) { *s_bin = tid; *s_above = above; }
}

// This thread's keys of one sweep: element c0 + u*1024 + tid, u < kSweep (zero past the end).
__device__ __forceinline__ void load_sweep(const uint32_t* keys, int c0, int len, int tid, bool full, uint32_t (&key)[kSweep]) {
  if (full) {
#pragma unroll
    for (int u = 0; u < kSweep; ++u) key[u] = keys[c0 + u * kSelThreads + tid];
  } else {
#pragma unroll
    for (int u = 0; u < kSweep; ++u) {
      const int c = c0 + u * kSelThreads + tid;
      key[u] = c < len ? keys[c] : 0u;
    }
  }
}

__global__ __launch_bounds__(kSelThreads) void select_resolve_kernel(const SelectParams p) {
  __shared__ uint32_t members[kMemberCap];
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t hist2[2][1024];
  __shared__ uint32_t wave_tot[kSelWaves];
  __shared__ uint32_t wave_gt[kSelWaves][kSweep], wave_eq[kSelWaves][kSweep];
  __shared__ uint32_t s_bin, s_above, s_members;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int seg = blockIdx.x;
  const int row = blockIdx.y;
  const int len = p.seg_len[seg];
  const int k = p.seg_k[seg];
  if (len <= 0 || k <= 0) {
    if (tid == 0) publish_threshold(p.thr, row, seg, 0xffffffffu, 0u);
    return;
  }
  if (k >= len) {
    if (tid == 0) publish_threshold(p.thr, row, seg, 0u, (uint32_t)len);
    return;
  }
  const uint32_t* keys = p.keys + (size_t)row * p.n_cand + p.seg_begin[seg];

  DBG_STAMP(0);
  for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
  for (int i = tid; i < 2 * 1024; i += kSelThreads) (&hist2[0][0])[i] = 0;
  if (tid == 0) s_members = 0;
  __syncthreads();

  // add up the parts' bin lists: wave w takes parts w, w + 16, ...; the length of a list and its first
  // 256 pairs are requested together (a list seldom has more), so a part costs one trip to memory
  const int parts_used = (len + kPartLen - 1) / kPartLen;
  for (int part = wave; part < parts_used; part += kSelWaves) {
    const uint32_t* list = p.bins + ((size_t)(row * 2 + seg) * p.parts + part) * kBinListStride;
    uint32_t bin[4], cnt[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {   // kBinListCap >= 256: always inside the list's allocation
      bin[u] = list[1 + 2 * (u * 64 + lane)];
      cnt[u] = list[2 + 2 * (u * 64 + lane)];
    }
    const int n = min((int)list[0], kBinListCap);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (u * 64 + lane < n) atomicAdd(&hist[bin[u] & (kBins - 1)], cnt[u]);
    for (int i = 256 + lane; i < n; i += 64) atomicAdd(&hist[list[1 + 2 * i] & (kBins - 1)], list[2 + 2 * i]);
  }
  __syncthreads();
  DBG_STAMP(1);
  pick_bin_wide(hist, (uint32_t)k, tid, lane, wave, wave_tot, &s_bin, &s_above);
  __syncthreads();
  const uint32_t bin1 = s_bin;
  uint32_t remaining = (uint32_t)k - s_above;
  const uint32_t n_members = hist[bin1];
  const bool listed = n_members <= (uint32_t)kMemberCap;

  DBG_STAMP(2);
  // collect the members of the threshold bin (their order is irrelevant: only counts are taken from
  // them); a bin with more members than the list holds is walked in the key buffer in every pass
  if (listed) {
    for (int c0 = 0; c0 < len; c0 += kSweep * kSelThreads) {
      const bool full = c0 + kSweep * kSelThreads <= len;
      uint32_t key[kSweep];
      load_sweep(keys, c0, len, tid, full, key);
      uint32_t wave_members = 0;
#pragma unroll
      for (int u = 0; u < kSweep; ++u) {
        const bool in = (key[u] >> kBinShift) == bin1 && (full || c0 + u * kSelThreads + tid < len);
        wave_members += (uint32_t)__popcll(__ballot(in));
      }
      uint32_t at = 0;
      if (lane == 0 && wave_members) at = atomicAdd(&s_members, wave_members);
      at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
#pragma unroll
      for (int u = 0; u < kSweep; ++u) {
        const bool in = (key[u] >> kBinShift) == bin1 && (full || c0 + u * kSelThreads + tid < len);
        const uint64_t b = __ballot(in);
        const uint32_t mine = at + (uint32_t)__popcll(b & ((1ull << lane) - 1ull));
        if (in && mine < (uint32_t)kMemberCap) members[mine] = key[u];
        at += (uint32_t)__popcll(b);
      }
    }
    __syncthreads();
  }

  DBG_STAMP(3);
  // the remaining 20 bits, MSB first, in two digits of 10 bits
  uint32_t prefix = bin1 << kBinShift, mask = 0xffffffffu << kBinShift;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int shift = pass == 0 ? 10 : 0;
    BinRun run;
    if (listed) {
      for (uint32_t i = tid; i < n_members; i += kSelThreads) {
        const uint32_t key = members[i];
        run_add(hist2[pass], run, (key & mask) == prefix, (key >> shift) & 1023u);
      }
    } else {
      for (int c0 = 0; c0 < len; c0 += kSweep * kSelThreads) {
        uint32_t key[kSweep];
        load_sweep(keys, c0, len, tid, false, key);
#pragma unroll
        for (int u = 0; u < kSweep; ++u)
          run_add(hist2[pass], run, c0 + u * kSelThreads + tid < len && (key[u] & mask) == prefix, (key[u] >> shift) & 1023u);
      }
    }
    run_flush(hist2[pass], run, lane);
    __syncthreads();
    pick_bin_1024(hist2[pass], remaining, tid, lane, wave, wave_tot, &s_bin, &s_above);
    __syncthreads();
    prefix |= s_bin << shift;
    mask |= 1023u << shift;
    remaining -= s_above;
  }
  if (tid == 0) publish_threshold(p.thr, row, seg, prefix, remaining);

  DBG_STAMP(4);
  // For the emission: per chunk of 1024 candidates, the number of entries above / equal to the threshold
  // before it.  Chunk u of a sweep is element u of every thread: every wave counts its 64 entries of each
  // chunk with two wave-wide compares, lane u keeps the counts of chunk u, and wave 0 adds the sixteen
  // waves' counts up, scans them over the sweep's chunks and writes the offsets.
  const uint32_t thr = prefix;
  uint32_t* offs = p.offs + (size_t)(row * 2 + seg) * p.chunks * 2;
  uint32_t base_gt = 0, base_eq = 0;   // running totals (wave 0)
  for (int c0 = 0; c0 < len; c0 += kSweep * kSelThreads) {
    const bool full = c0 + kSweep * kSelThreads <= len;
    uint32_t key[kSweep];
    load_sweep(keys, c0, len, tid, full, key);
    uint32_t my_gt = 0, my_eq = 0;
#pragma unroll
    for (int u = 0; u < kSweep; ++u) {
      const bool in = full || c0 + u * kSelThreads + tid < len;
      const uint32_t g = (uint32_t)__popcll(__ballot(in && key[u] > thr)), e = (uint32_t)__popcll(__ballot(in && key[u] == thr));
      if (lane == u) { my_gt = g; my_eq = e; }
    }
    __syncthreads();   // wave 0 has read the previous sweep's counts
    if (lane < kSweep) { wave_gt[wave][lane] = my_gt; wave_eq[wave][lane] = my_eq; }
    __syncthreads();
    if (wave == 0) {
      uint32_t g = 0, e = 0;
      if (lane < kSweep) {
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) { g += wave_gt[w][lane]; e += wave_eq[w][lane]; }
      }
      uint32_t sg = g, se = e;   // inclusive scan over the sweep's chunks
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t tg = __shfl_up(sg, o), te = __shfl_up(se, o);
        if (lane >= o) { sg += tg; se += te; }
      }
      const int chunk = c0 / kSelThreads + lane;
      if (lane < kSweep && chunk < p.chunks && (int64_t)chunk * kSelThreads < len) {
        offs[2 * chunk] = base_gt + sg - g;
        offs[2 * chunk + 1] = base_eq + se - e;
      }
      base_gt += (uint32_t)__builtin_amdgcn_readlane((int)sg, 63);
      base_eq += (uint32_t)__builtin_amdgcn_readlane((int)se, 63);
    }
  }
  DBG_STAMP(5);
}

// ------------------------------------------------------------------ stage 3 of long segments: position-ordered emission
// One workgroup per kEmitChunk consecutive candidates of a segment; candidate c = chunk*1024 + it*256 + tid.
// blockIdx.y >= n_seg is the unconditional tail (prefix-only eviction keeps the whole suffix).
__global__ __launch_bounds__(kEmitThreads) void select_emit_kernel(const SelectParams p) {
  __shared__ uint32_t cell_gt[kEmitItems * kEmitWaves], cell_eq[kEmitItems * kEmitWaves];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int chunk = blockIdx.x;
  const int sx = blockIdx.y;
  const int row = blockIdx.z;
  const bool tail = sx >= p.n_seg;
  const int begin = tail ? p.tail_begin : p.seg_begin[sx];
  const int len = tail ? p.tail_len : p.seg_len[sx];
  const int out0 = tail ? p.tail_out : p.seg_out[sx];
  const int c0 = chunk * kEmitChunk;
  if (c0 >= len) return;
  int32_t* idx_row = p.idx + (size_t)row * p.k_total + out0;
  if (tail) {
#pragma unroll
    for (int it = 0; it < kEmitItems; ++it) {
      const int c = c0 + it * kEmitThreads + tid;
      if (c < len) idx_row[c] = cand_pos(begin + c, p.block_off, p.block_len);
    }
    return;
  }
  const uint32_t thr = p.thr[(row * 2 + sx) * 2];
  const uint32_t need = p.thr[(row * 2 + sx) * 2 + 1];
  const uint32_t* offs = p.offs + ((size_t)(row * 2 + sx) * p.chunks + chunk) * 2;
  // keep-everything / keep-nothing segments have no counts on file: both follow from the chunk's position
  const bool ranked = p.seg_k[sx] > 0 && p.seg_k[sx] < len;
  const uint32_t gt_b = ranked ? offs[0] : 0u;
  const uint32_t eq_b = ranked ? offs[1] : (uint32_t)c0;
  const uint32_t* keys = p.keys + (size_t)row * p.n_cand + begin;

  // cell (it, wave) = 64 consecutive candidates; cells in index order are in position order
  bool gt[kEmitItems], eq[kEmitItems];
  uint64_t b_gt[kEmitItems], b_eq[kEmitItems];
  uint32_t key[kEmitItems];
#pragma unroll
  for (int it = 0; it < kEmitItems; ++it) {
    const int c = c0 + it * kEmitThreads + tid;
    key[it] = c < len ? keys[c] : 0u;
  }
#pragma unroll
  for (int it = 0; it < kEmitItems; ++it) {
    const bool valid = c0 + it * kEmitThreads + tid < len;
    gt[it] = valid && key[it] > thr;
    eq[it] = valid && key[it] == thr;
    b_gt[it] = __ballot(gt[it]);
    b_eq[it] = __ballot(eq[it]);
    if (lane == 0) {
      cell_gt[it * kEmitWaves + wave] = (uint32_t)__popcll(b_gt[it]);
      cell_eq[it * kEmitWaves + wave] = (uint32_t)__popcll(b_eq[it]);
    }
  }
  __syncthreads();
  uint32_t cg[kEmitItems * kEmitWaves], ce[kEmitItems * kEmitWaves];
#pragma unroll
  for (int j = 0; j < kEmitItems * kEmitWaves; ++j) { cg[j] = cell_gt[j]; ce[j] = cell_eq[j]; }
  const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
  for (int it = 0; it < kEmitItems; ++it) {
    uint32_t og = 0, oe = 0;
#pragma unroll
    for (int j = 0; j < kEmitItems * kEmitWaves; ++j)
      if (j < it * kEmitWaves + wave) { og += cg[j]; oe += ce[j]; }
    const uint32_t gt_before = gt_b + og + (uint32_t)__popcll(b_gt[it] & lt_mask);
    const uint32_t eq_before = eq_b + oe + (uint32_t)__popcll(b_eq[it] & lt_mask);
    const int pos = cand_pos(begin + c0 + it * kEmitThreads + tid, p.block_off, p.block_len);
    if (gt[it]) idx_row[gt_before + min(eq_before, need)] = pos;
    else if (eq[it] && eq_before < need) idx_row[gt_before + eq_before] = pos;
  }
}

// ------------------------------------------------------------------ launchers
static int longest_ranked(const SelectParams& p) {
  int longest = 0;
  for (int i = 0; i < p.n_seg; ++i) longest = p.seg_len[i] > longest ? p.seg_len[i] : longest;
  return longest;
}

// Workspace of the long-segment path, in 32-bit words: key buffer, thresholds, bin lists, chunk offsets
// (all zero when every ranked segment fits one workgroup).
SelectWorkspace select_workspace(const SelectParams& p) {
  SelectWorkspace w{};
  const int longest = longest_ranked(p);
  if (longest <= kSelRegItems * kSelThreads) return w;
  const size_t parts = (size_t)(longest + kPartLen - 1) / kPartLen;
  const size_t chunks = (size_t)(longest + kEmitChunk - 1) / kEmitChunk;
  w.keys = (size_t)p.rows * p.n_cand;
  w.thr = (size_t)p.rows * 4;
  w.bins = (size_t)p.rows * 2 * parts * kBinListStride;
  w.offs = (size_t)p.rows * 2 * chunks * 2;
  return w;
}

template <int ITEMS>
static void launch_items(const SelectParams& p, dim3 grid, hipStream_t s) {
  const dim3 block(kSelThreads);
  switch (p.pool_half) {
    case 0: hipLaunchKernelGGL((select_kernel<ITEMS, 0>), grid, block, 0, s, p); break;
    case 1: hipLaunchKernelGGL((select_kernel<ITEMS, 1>), grid, block, 0, s, p); break;
    case 2: hipLaunchKernelGGL((select_kernel<ITEMS, 2>), grid, block, 0, s, p); break;
    default: hipLaunchKernelGGL((select_kernel<ITEMS, -1>), grid, block, 0, s, p); break;   // wider windows: generic pooling
  }
}

hipError_t launch_select(const SelectParams& q, hipStream_t s) {
  SelectParams p = q;
  const int nx = p.n_seg + (p.tail_len > 0 ? 1 : 0);
  if (nx == 0 || p.rows == 0) return hipSuccess;
  if (p.k_total == 0 && !p.pooled) return hipSuccess;   // nothing retained and nobody wants the pooled scores
  if (p.rows > 65535 || p.n_seg > 2) return hipErrorInvalidValue;
  // every ranked segment and the unconditional tail lie inside a score row of n_cand candidates, so
  // no workgroup reads past rows * n_cand entries of the score or key buffers
  for (int i = 0; i < p.n_seg; ++i)
    if (p.seg_begin[i] < 0 || p.seg_len[i] < 0 || p.seg_begin[i] + p.seg_len[i] > p.n_cand || p.seg_k[i] > p.seg_len[i])
      return hipErrorInvalidValue;
  if (p.tail_len > 0 && (p.tail_begin < 0 || p.tail_begin + p.tail_len > p.n_cand)) return hipErrorInvalidValue;
  if (!p.idx && p.k_total > 0) return hipErrorInvalidValue;
  const int longest = longest_ranked(p);
  const dim3 grid(nx, p.rows);
  if (longest <= 1 * kSelThreads) launch_items<1>(p, grid, s);
  else if (longest <= 2 * kSelThreads) launch_items<2>(p, grid, s);
  else if (longest <= 4 * kSelThreads) launch_items<4>(p, grid, s);
  else if (longest <= kSelRegItems * kSelThreads) launch_items<kSelRegItems>(p, grid, s);
  else {
    if (!p.keys || !p.thr || !p.bins || !p.offs) return hipErrorInvalidValue;
    p.parts = (longest + kPartLen - 1) / kPartLen;
    p.chunks = (longest + kEmitChunk - 1) / kEmitChunk;
    const dim3 pgrid(p.parts, p.n_seg, p.rows), block(kSelThreads);
    switch (p.pool_half) {
      case 0: hipLaunchKernelGGL(select_pool_kernel<0>, pgrid, block, 0, s, p); break;
      case 1: hipLaunchKernelGGL(select_pool_kernel<1>, pgrid, block, 0, s, p); break;
      case 2: hipLaunchKernelGGL(select_pool_kernel<2>, pgrid, block, 0, s, p); break;
      default: hipLaunchKernelGGL(select_pool_kernel<-1>, pgrid, block, 0, s, p); break;
    }
    hipLaunchKernelGGL(select_resolve_kernel, dim3(p.n_seg, p.rows), block, 0, s, p);
    const int longest_any = p.tail_len > longest ? p.tail_len : longest;
    if (p.k_total > 0)
      hipLaunchKernelGGL(select_emit_kernel, dim3((longest_any + kEmitChunk - 1) / kEmitChunk, nx, p.rows), dim3(kEmitThreads), 0, s, p);
  }
  return hipGetLastError();
}

#ifdef SDLLM_TUNING
extern "C" int sdllm_debug_stamps(unsigned long long* out) { return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_dbg), sizeof(g_dbg)); }
#endif

}  // namespace sdllm
