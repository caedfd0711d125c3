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
// Longer segments (up to 1M candidates) are spread over the machine in two launches:
//   select_pool_kernel    one workgroup per 2048 candidates: pooling, keys to a key buffer, and per chunk of
//                         1024 candidates the list of the non-empty bins of the keys' leading 12 bits plus the
//                         chunk's keys ordered by bin;
//   select_finish_kernel  one workgroup per 4096 candidates: finds the segment's threshold from the lists and
//                         the members of the one bin that holds the k-th value (every workgroup of a segment
//                         does this for itself, side by side), counts what precedes its own candidates and
//                         emits them in position order.
#include "sdllm_internal.h"

namespace sdllm {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelRegItems = 8;                        // longest register-resident variant (chunks of 1024)
constexpr int kPoolChunks = 2;                         // chunks of 1024 candidates per select_pool_kernel workgroup
constexpr int kPartLen = kPoolChunks * kSelThreads;
constexpr int kBinShift = 20, kBins = 4096;            // leading 12 bits of a key
constexpr int kBinListCap = kSelThreads;               // a chunk cannot occupy more bins than it has candidates
constexpr int kBinListStride = 1 + 2 * kBinListCap;    // words per list: count, then (bin, count) pairs
static_assert(kBinListCap >= 128, "select_finish_kernel reads the first 128 pairs of every list unconditionally");
constexpr int kMemberCap = 6144;                       // members of the threshold bin held in LDS by select_finish_kernel
constexpr int kFinishChunks = 4;                       // chunks of 1024 candidates one select_finish_kernel workgroup emits
constexpr int kMaxChunks = 1024;                       // chunks per segment the long-segment path handles (1M candidates)

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

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves only (six vector
// instructions; a shuffle-based scan is six dependent trips through the LDS crossbar): four shifts inside
// each row of 16 lanes, then lane 15 of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
// A lane whose source lies outside its row, or whose row is masked out, adds zero.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add(uint32_t v) {
  return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true);
}
__device__ __forceinline__ uint32_t wave_scan_incl(uint32_t v) {
  v = dpp_add<0x111, 0xF>(v);   // row_shr:1
  v = dpp_add<0x112, 0xF>(v);   // row_shr:2
  v = dpp_add<0x114, 0xF>(v);   // row_shr:4
  v = dpp_add<0x118, 0xF>(v);   // row_shr:8
  v = dpp_add<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
  v = dpp_add<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
  return v;
}
// Sum over the wave (the same value in every lane, scalar).
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_readlane((int)wave_scan_incl(v), 63);
}
// Inclusive suffix sum: lane i gets v[i] + v[i+1] + ... + v[63].
__device__ __forceinline__ uint32_t wave_scan_suffix_incl(uint32_t v) {
  const uint32_t pre = wave_scan_incl(v);
  return (uint32_t)__builtin_amdgcn_readlane((int)pre, 63) - pre + v;
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
    const uint32_t total = wave_sum(r.count);   // 0 in idle lanes
    if (lane == leader) atomicAdd(&hist[lead_bin], total);
  } else if (active) {
    atomicAdd(&hist[r.bin], r.count);
  }
}

// Wave 0, after a pass's 256-bin histogram is complete: the bin that holds the `remaining`-th largest
// active key and the number of keys in higher bins (four bins per lane).
__device__ __forceinline__ void pick_bin(const uint32_t* h, uint32_t remaining, int lane, uint32_t* s_bin, uint32_t* s_above) {
  const uint32_t h0 = h[4 * lane], h1 = h[4 * lane + 1], h2 = h[4 * lane + 2], h3 = h[4 * lane + 3];
  const uint32_t lane_sum = h0 + h1 + h2 + h3;
  const uint32_t suf = wave_scan_suffix_incl(lane_sum);
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
  const uint32_t suf = wave_scan_suffix_incl(mine);   // over the lanes of this wave
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

// Exclusive scan, in place, of the n_cells (<= 1024) per-cell counts of the emission pass; cell
// it*16 + wave is the 64 candidates wave `wave` holds in chunk `it`, so index order is position order.
// Two workgroup barriers inside; the caller synchronises before (counts written) and may read after.
__device__ __forceinline__ void scan_cells(uint32_t* cell_gt, uint32_t* cell_eq, int n_cells, uint32_t* wave_gt, uint32_t* wave_eq,
                                           int tid, int lane, int wave) {
  const uint32_t g = tid < n_cells ? cell_gt[tid] : 0u, e = tid < n_cells ? cell_eq[tid] : 0u;
  const uint32_t sg = wave_scan_incl(g), se = wave_scan_incl(e);
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

// ------------------------------------------------------------------ long segments, launch 1: pooling and bucketing
// One workgroup per two chunks of 1024 candidates.  Besides the keys in position order (key buffer) it
// leaves, per chunk, the list of the non-empty bins of the keys' leading 12 bits with their counts, and
// the chunk's keys once more ordered by bin (a counting sort through the chunk's histogram; the order
// inside a bin is arbitrary), so that the second launch can pick the members of any one bin out of a
// chunk without looking at the chunk's other keys.
template <int HALF>
__global__ __launch_bounds__(kSelThreads) void select_pool_kernel(const SelectParams p) {
  __shared__ uint32_t hist[kPoolChunks][kBins];
  __shared__ uint32_t wave_n[kPoolChunks][kSelWaves], wave_s[kPoolChunks][kSelWaves];

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
  uint32_t* sorted = p.sorted + (size_t)row * p.n_cand + begin;

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
  if (k <= 0 || k >= len) return;   // nothing to rank: everything or nothing is kept

  for (int i = tid; i < kPoolChunks * kBins; i += kSelThreads) (&hist[0][0])[i] = 0;
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kPoolChunks; ++u)
    if (c_first + u * kSelThreads + tid < len) atomicAdd(&hist[u][keys[u] >> kBinShift], 1u);
  __syncthreads();
  // thread t owns bins 4t .. 4t+3 of both chunks: number of non-empty bins and of keys before them
  uint32_t h[kPoolChunks][4], n[kPoolChunks], sum[kPoolChunks], n_incl[kPoolChunks], s_incl[kPoolChunks];
#pragma unroll
  for (int u = 0; u < kPoolChunks; ++u) {
    n[u] = sum[u] = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      h[u][j] = hist[u][4 * tid + j];
      n[u] += h[u][j] != 0;
      sum[u] += h[u][j];
    }
    n_incl[u] = wave_scan_incl(n[u]);
    s_incl[u] = wave_scan_incl(sum[u]);
    if (lane == 63) { wave_n[u][wave] = n_incl[u]; wave_s[u][wave] = s_incl[u]; }
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kPoolChunks; ++u) {
    const int chunk = part * kPoolChunks + u;
    if ((int64_t)chunk * kSelThreads >= len) break;   // workgroup-uniform
    uint32_t at = n_incl[u] - n[u], start = s_incl[u] - sum[u];
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w)
      if (w < wave) { at += wave_n[u][w]; start += wave_s[u][w]; }
    uint32_t* list = p.bins + ((size_t)(row * 2 + seg) * p.chunks + chunk) * kBinListStride;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      hist[u][4 * tid + j] = start;   // from here on: where the bin's next key goes in the sorted chunk
      start += h[u][j];
      if (h[u][j] != 0) {             // at most 1024 non-empty bins per chunk, so at < kBinListCap
        list[1 + 2 * at] = 4 * tid + j;
        list[2 + 2 * at] = h[u][j];
        ++at;
      }
    }
    if (tid == kSelThreads - 1) list[0] = at;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kPoolChunks; ++u) {
    const int c = c_first + u * kSelThreads + tid;
    if (c < len) {
      const uint32_t at = atomicAdd(&hist[u][keys[u] >> kBinShift], 1u);   // < number of keys of the chunk
      sorted[(size_t)(part * kPoolChunks + u) * kSelThreads + at] = keys[u];
    }
  }
}

// ------------------------------------------------------------------ long segments, launch 2: threshold and emission
// The bin that holds the `remaining`-th largest key of a 1024-bin histogram and the number of keys in
// higher bins, by all 1024 threads (one bin each).  One workgroup barrier inside; the caller synchronises
// before (histogram complete) and after.
__device__ __forceinline__ void pick_bin_1024(const uint32_t* h, uint32_t remaining, int tid, int lane, int wave,
                                              uint32_t* wave_tot, uint32_t* s_bin, uint32_t* s_above) {
  const uint32_t mine = h[tid];
  const uint32_t suf = wave_scan_suffix_incl(mine);   // over the lanes of this wave
  if (lane == 0) wave_tot[wave] = suf;
  __syncthreads();
  uint32_t above = suf - mine;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w)
    if (w > wave) above += wave_tot[w];
  if (above < remaining && remaining <= above + mine) { *s_bin = tid; *s_above = above; }
}

// One workgroup emits kFinishChunks consecutive chunks of a segment (candidate c = chunk*1024 + tid).  Every
// workgroup of a segment first finds the segment's threshold for itself, from what launch 1 left behind:
// it adds the chunks' bin lists up (a few thousand pairs), finds the bin of the k-th value, fetches that
// bin's members out of the bin-sorted chunks (a few hundred to a few thousand keys) and resolves their
// remaining 20 bits; it then counts, again from lists and members only, the entries above and equal to
// the threshold in the chunks before its own.  That work is the same for all workgroups of a segment, but
// they run side by side on different CUs, which is faster than a launch boundary between a one-workgroup
// threshold kernel and the emission (no kernel here ever walks all keys of a segment on one CU: 32k keys
// cost one CU 6 us per sweep in instruction issue alone).
// blockIdx.y >= n_seg is the unconditional tail (prefix-only eviction keeps the whole suffix).
__global__ __launch_bounds__(kSelThreads) void select_finish_kernel(const SelectParams p) {
  __shared__ uint32_t members[kMemberCap];
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t hist2[2][1024];
  __shared__ uint16_t chunk_above[kMaxChunks], chunk_below[kMaxChunks], chunk_mem[kMaxChunks];
  __shared__ uint32_t wave_tot[kSelWaves], wave_gt[kSelWaves], wave_eq[kSelWaves], scan_gt[kSelWaves], scan_eq[kSelWaves];
  __shared__ uint32_t cell_gt[kFinishChunks * kSelWaves], cell_eq[kFinishChunks * kSelWaves];
  __shared__ uint32_t s_bin, s_above, s_members;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int sx = blockIdx.y;
  const int row = blockIdx.z;
  const bool tail = sx >= p.n_seg;
  const int begin = tail ? p.tail_begin : p.seg_begin[sx];
  const int len = tail ? p.tail_len : p.seg_len[sx];
  const int out0 = tail ? p.tail_out : p.seg_out[sx];
  const int k = tail ? len : p.seg_k[sx];
  const int own0 = blockIdx.x * kFinishChunks;          // first own chunk
  const int c_own = own0 * kSelThreads;
  if (c_own >= len || k <= 0) return;
  int32_t* out = p.idx + (size_t)row * p.k_total + out0;
  if (k >= len) {   // everything is kept
#pragma unroll
    for (int it = 0; it < kFinishChunks; ++it) {
      const int c = c_own + it * kSelThreads + tid;
      if (c < len) out[c] = cand_pos(begin + c, p.block_off, p.block_len);
    }
    return;
  }
  const uint32_t* keys = p.keys + (size_t)row * p.n_cand + begin;
  const uint32_t* sorted = p.sorted + (size_t)row * p.n_cand + begin;
  const uint32_t* lists = p.bins + (size_t)(row * 2 + sx) * p.chunks * kBinListStride;
  const int n_chunks = (len + kSelThreads - 1) / kSelThreads;   // <= kMaxChunks (launcher)

  // own keys: requested now, used at the very end
  uint32_t own_key[kFinishChunks];
#pragma unroll
  for (int it = 0; it < kFinishChunks; ++it) {
    const int c = c_own + it * kSelThreads + tid;
    own_key[it] = c < len ? keys[c] : 0u;
  }

  for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
  for (int i = tid; i < 2 * 1024; i += kSelThreads) (&hist2[0][0])[i] = 0;
  if (tid == 0) s_members = 0;
  __syncthreads();

  // 1. the segment's histogram of leading bits: wave w adds up the lists of chunks w, w + 16, ...; the
  //    length of a list and its first 128 pairs are requested together (a list seldom has more), and
  //    those of a wave's first two chunks stay in registers for step 2
  constexpr int kHeld = 2;
  uint32_t held_bin[kHeld][2], held_cnt[kHeld][2];
  int held_n[kHeld];
#pragma unroll
  for (int j = 0; j < kHeld; ++j) {
    const int c = wave + j * kSelWaves;
    held_n[j] = 0;
    if (c < n_chunks) {   // wave-uniform
      const uint32_t* list = lists + (size_t)c * kBinListStride;
#pragma unroll
      for (int u = 0; u < 2; ++u) {   // inside the list's allocation whatever its length
        held_bin[j][u] = list[1 + 2 * (u * 64 + lane)];
        held_cnt[j][u] = list[2 + 2 * (u * 64 + lane)];
      }
      held_n[j] = min((int)list[0], kBinListCap);
    }
  }
#pragma unroll
  for (int j = 0; j < kHeld; ++j) {
    const int c = wave + j * kSelWaves;
    if (c >= n_chunks) break;
    const uint32_t* list = lists + (size_t)c * kBinListStride;
#pragma unroll
    for (int u = 0; u < 2; ++u)
      if (u * 64 + lane < held_n[j]) atomicAdd(&hist[held_bin[j][u] & (kBins - 1)], held_cnt[j][u]);
    for (int i = 128 + lane; i < held_n[j]; i += 64) atomicAdd(&hist[list[1 + 2 * i] & (kBins - 1)], list[2 + 2 * i]);
  }
  for (int c = wave + kHeld * kSelWaves; c < n_chunks; c += kSelWaves) {
    const uint32_t* list = lists + (size_t)c * kBinListStride;
    const int n = min((int)list[0], kBinListCap);
    for (int i = lane; i < n; i += 64) atomicAdd(&hist[list[1 + 2 * i] & (kBins - 1)], list[2 + 2 * i]);
  }
  __syncthreads();
  pick_bin_wide(hist, (uint32_t)k, tid, lane, wave, wave_tot, &s_bin, &s_above);
  __syncthreads();
  const uint32_t bin1 = s_bin;
  uint32_t remaining = (uint32_t)k - s_above;
  const uint32_t n_members = hist[bin1];
  const bool listed = n_members <= (uint32_t)kMemberCap;

  // 2. per chunk: keys in higher bins, keys in lower bins (= where the threshold bin's members start in
  //    the bin-sorted chunk) and members; the members go to the LDS list.  Keys above and below the
  //    threshold bin are at most 1024 each: packed 16 bits apiece they take one wave reduction, and the
  //    members are the rest of the chunk.
  auto side = [&](uint32_t b, uint32_t ct) { return b > bin1 ? ct : (b < bin1 ? ct << 16 : 0u); };
  auto finish_chunk = [&](int c, uint32_t packed) {
    packed = wave_sum(packed);
    const uint32_t in_chunk = (uint32_t)min(kSelThreads, len - c * kSelThreads);
    const uint32_t above = packed & 0xffffu, below = packed >> 16, mem = in_chunk - above - below;
    if (lane == 0) { chunk_above[c] = (uint16_t)above; chunk_below[c] = (uint16_t)below; chunk_mem[c] = (uint16_t)mem; }
    if (listed && mem) {
      uint32_t at = 0;
      if (lane == 0) at = atomicAdd(&s_members, mem);
      at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
      for (uint32_t i = lane; i < mem; i += 64)
        if (at + i < (uint32_t)kMemberCap) members[at + i] = sorted[(size_t)c * kSelThreads + below + i];
    }
  };
#pragma unroll
  for (int j = 0; j < kHeld; ++j) {
    const int c = wave + j * kSelWaves;
    if (c >= n_chunks) break;
    const uint32_t* list = lists + (size_t)c * kBinListStride;
    uint32_t packed = 0;
#pragma unroll
    for (int u = 0; u < 2; ++u)
      if (u * 64 + lane < held_n[j]) packed += side(held_bin[j][u], held_cnt[j][u]);
    for (int i = 128 + lane; i < held_n[j]; i += 64) packed += side(list[1 + 2 * i], list[2 + 2 * i]);
    finish_chunk(c, packed);
  }
  for (int c = wave + kHeld * kSelWaves; c < n_chunks; c += kSelWaves) {
    const uint32_t* list = lists + (size_t)c * kBinListStride;
    const int n = min((int)list[0], kBinListCap);
    uint32_t packed = 0;
    for (int i = lane; i < n; i += 64) packed += side(list[1 + 2 * i], list[2 + 2 * i]);
    finish_chunk(c, packed);
  }
  __syncthreads();

  // 3. the remaining 20 bits of the threshold, MSB first, in two digits of 10 bits; a bin with more members
  //    than the list holds is read from the bin-sorted chunks in both passes
  uint32_t prefix = bin1 << kBinShift, mask = 0xffffffffu << kBinShift;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int shift = pass == 0 ? 10 : 0;
    if (listed) {   // a few keys per thread, spread over 1024 bins: one LDS atomic each
      for (uint32_t i = tid; i < n_members; i += kSelThreads) {
        const uint32_t key = members[i];
        if ((key & mask) == prefix) atomicAdd(&hist2[pass][(key >> shift) & 1023u], 1u);
      }
    } else {
      BinRun run;
      for (int c = wave; c < n_chunks; c += kSelWaves) {
        const uint32_t below = chunk_below[c], mem = chunk_mem[c];
        for (uint32_t i = lane; i < mem; i += 64) {
          const uint32_t key = sorted[(size_t)c * kSelThreads + below + i];
          run_add(hist2[pass], run, (key & mask) == prefix, (key >> shift) & 1023u);
        }
      }
      run_flush(hist2[pass], run, lane);
    }
    __syncthreads();
    pick_bin_1024(hist2[pass], remaining, tid, lane, wave, wave_tot, &s_bin, &s_above);
    __syncthreads();
    prefix |= s_bin << shift;
    mask |= 1023u << shift;
    remaining -= s_above;
  }
  const uint32_t thr = prefix;
  const uint32_t need_eq = remaining;

  // 4. entries above / equal to the threshold in the chunks before this workgroup's own
  uint32_t gt_b = 0, eq_b = 0;
  for (int c = wave; c < own0; c += kSelWaves) {
    const uint32_t below = chunk_below[c], mem = chunk_mem[c];
    if (lane == 0) gt_b += chunk_above[c];
    for (uint32_t i = lane; i < mem; i += 64) {
      const uint32_t key = sorted[(size_t)c * kSelThreads + below + i];
      gt_b += key > thr;
      eq_b += key == thr;
    }
  }
  gt_b = wave_sum(gt_b);
  eq_b = wave_sum(eq_b);
  if (lane == 0) { wave_gt[wave] = gt_b; wave_eq[wave] = eq_b; }

  // 5. own candidates: cell (it, wave) = 64 consecutive candidates; cells in index order are in position order
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  uint32_t my_gt = 0, my_eq = 0;   // lane `it` keeps the counts of cell (it, wave)
#pragma unroll
  for (int it = 0; it < kFinishChunks; ++it) {
    const bool valid = c_own + it * kSelThreads + tid < len;
    const uint64_t b_gt = __ballot(valid && own_key[it] > thr), b_eq = __ballot(valid && own_key[it] == thr);
    if (lane == it) { my_gt = __popcll(b_gt); my_eq = __popcll(b_eq); }
  }
  if (lane < kFinishChunks) { cell_gt[lane * kSelWaves + wave] = my_gt; cell_eq[lane * kSelWaves + wave] = my_eq; }
  __syncthreads();
  gt_b = eq_b = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) { gt_b += wave_gt[w]; eq_b += wave_eq[w]; }
  scan_cells(cell_gt, cell_eq, kFinishChunks * kSelWaves, scan_gt, scan_eq, tid, lane, wave);
#pragma unroll
  for (int it = 0; it < kFinishChunks; ++it) {
    const int c = c_own + it * kSelThreads + tid;
    const bool gt = c < len && own_key[it] > thr;
    const bool eq = c < len && own_key[it] == thr;
    const uint64_t b_gt = __ballot(gt), b_eq = __ballot(eq);
    const uint32_t gt_before = gt_b + cell_gt[it * kSelWaves + wave] + __popcll(b_gt & lt_mask);
    const uint32_t eq_before = eq_b + cell_eq[it * kSelWaves + wave] + __popcll(b_eq & lt_mask);
    if (gt) out[gt_before + min(eq_before, need_eq)] = cand_pos(begin + c, p.block_off, p.block_len);
    else if (eq && eq_before < need_eq) out[gt_before + eq_before] = cand_pos(begin + c, p.block_off, p.block_len);
  }
}

// ------------------------------------------------------------------ launchers
static int longest_ranked(const SelectParams& p) {
  int longest = 0;
  for (int i = 0; i < p.n_seg; ++i) longest = p.seg_len[i] > longest ? p.seg_len[i] : longest;
  return longest;
}

// Workspace of the long-segment path, in 32-bit words: keys in position order, keys sorted by bin per chunk,
// per-chunk bin lists (all zero when every ranked segment fits one workgroup).
SelectWorkspace select_workspace(const SelectParams& p) {
  SelectWorkspace w{};
  const int longest = longest_ranked(p);
  if (longest <= kSelRegItems * kSelThreads) return w;
  const size_t chunks = (size_t)(longest + kSelThreads - 1) / kSelThreads;
  w.keys = (size_t)p.rows * p.n_cand;
  w.sorted = (size_t)p.rows * p.n_cand;
  w.bins = (size_t)p.rows * 2 * chunks * kBinListStride;
  return w;
}

// Longest ranked segment the selection handles (beyond it the per-chunk tables of select_finish_kernel overflow).
int select_max_segment() { return kMaxChunks * kSelThreads; }

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
    if (!p.keys || !p.sorted || !p.bins || longest > select_max_segment()) return hipErrorInvalidValue;
    p.chunks = (longest + kSelThreads - 1) / kSelThreads;
    const dim3 pgrid((longest + kPartLen - 1) / kPartLen, p.n_seg, p.rows), block(kSelThreads);
    switch (p.pool_half) {
      case 0: hipLaunchKernelGGL(select_pool_kernel<0>, pgrid, block, 0, s, p); break;
      case 1: hipLaunchKernelGGL(select_pool_kernel<1>, pgrid, block, 0, s, p); break;
      case 2: hipLaunchKernelGGL(select_pool_kernel<2>, pgrid, block, 0, s, p); break;
      default: hipLaunchKernelGGL(select_pool_kernel<-1>, pgrid, block, 0, s, p); break;
    }
    const int longest_any = p.tail_len > longest ? p.tail_len : longest;
    const int per_wg = kFinishChunks * kSelThreads;
    if (p.k_total > 0) hipLaunchKernelGGL(select_finish_kernel, dim3((longest_any + per_wg - 1) / per_wg, nx, p.rows), block, 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace sdllm
