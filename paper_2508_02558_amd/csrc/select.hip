// Pooling + top-k retention (Sec. 3.3 third equation; Alg. 1 steps 8-10).
//
// One workgroup ranks one segment of one (batch, KV head) row:
//   1. stride-1 pooling of the score with window s clipped to the segment (-inf padding for max,
//      zero padding and a fixed divisor s for avg);
//   2. a 4-pass, 8-bit MSB-first radix select on the order-preserving integer image of the fp32
//      pooled values finds the exact k-th largest value T;
//   3. one pass in position order keeps every value above T and the first (k - #above) values
//      equal to T, so ties go to the lower position and the output is ascending without a sort.
// Max pooling copies a peak to its neighbours, so T routinely falls inside a group of equal values;
// the tie rule is exercised constantly, not only in corner cases.
//
// The kernel is templated on ITEMS, the pooled values each of the 1024 threads keeps in registers
// (element c = it*1024 + tid, so chunks are in position order): the score row is then read from
// memory exactly once, with all of a thread's loads in flight together.  HALF >= 0 fixes the pooling
// half-width at compile time: a lane gets its window neighbours from the adjacent lanes of its
// wave (they hold the adjacent candidates) and only the lanes at a wave's edge load theirs from
// memory.  The emission pass counts every (chunk, wave) cell first, scans the cell counts once,
// and then writes: three workgroup barriers however many chunks there are.
// Segments of more than 8 x 1024 candidates (up to 36 x 1024) use select_lds_kernel instead: the keys
// live in LDS (144 KB at most) and every phase is a rolled loop over chunks (unrolled over 36
// register-resident chunks the same program was ~55 KB of straight-line code at the 128-register
// limit, and no faster).
// ITEMS = 0 is the unbounded variant that re-reads the pooled row from memory (L2) in every pass.
#include "sdllm_internal.h"

namespace sdllm {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

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

// Wave 0, after a pass's histogram is complete: the bin that holds the `remaining`-th largest
// active key and the number of keys in higher bins (256 bins, four per lane).
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

// Pooled values of U consecutive chunks (it0 .. it0+U-1) of a segment, element c = it*1024 + tid:
// own values first, plus one extra load per chunk in which lanes 0..HALF-1 fetch the HALF candidates
// left of the wave's 64 and lanes HALF..2*HALF-1 the HALF right of them (every load is unconditional
// and independent, so all 2U loads of a thread are in flight together); the window then comes from
// whole-wave shifts.  Same arithmetic as pool_at, term for term.
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

template <int ITEMS, int HALF>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectParams p) {
  constexpr int kCells = (ITEMS > 0 ? ITEMS : 1) * kSelWaves;   // (chunk, wave) cells of the emission pass
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
  const float* score = p.score + (size_t)row * p.n_cand + begin;
  float* pooled = p.pooled ? p.pooled + (size_t)row * p.n_cand + begin : nullptr;
  int32_t* out = idx_row + p.seg_out[seg];
  const int chunks = ITEMS > 0 ? ITEMS : (len + kSelThreads - 1) / kSelThreads;
  if (len <= 0) return;   // an empty segment (no suffix after the last block, no prefix before the first): no load at all

  // 1. pooling
  const int half = p.pool_half;
  const float inv_s = 1.f / (float)(2 * half + 1);
  uint32_t keys[ITEMS > 0 ? ITEMS : 1];
  if (ITEMS > 0 && HALF >= 0) {
    float pv[ITEMS > 0 ? ITEMS : 1];
    pool_chunks<(ITEMS > 0 ? ITEMS : 1), (HALF >= 0 ? HALF : 0)>(score, len, 0, tid, lane, p.avg_pool, inv_s, pv);
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int c = it * kSelThreads + tid;
      keys[it] = 0;
      if (c < len) {
        keys[it] = order_key(pv[it]);
        if (pooled) pooled[c] = pv[it];
      }
    }
  } else if (ITEMS > 0) {
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int c = it * kSelThreads + tid;
      keys[it] = 0;
      if (c < len) {
        const float v = pool_at(score, c, len, half, p.avg_pool, inv_s);
        keys[it] = order_key(v);
        if (pooled) pooled[c] = v;
      }
    }
  } else {
    for (int c = tid; c < len; c += kSelThreads) pooled[c] = pool_at(score, c, len, half, p.avg_pool, inv_s);
  }
  if (k <= 0) return;
  if (k >= len) {
    for (int c = tid; c < len; c += kSelThreads) out[c] = cand_pos(begin + c, p.block_off, p.block_len);
    return;
  }
  for (int i = tid; i < 4 * 256; i += kSelThreads) (&hist[0][0])[i] = 0;
  __syncthreads();   // histograms cleared; (ITEMS == 0) pooled[] written by other threads is read below

  auto key_at = [&](int it, int c) -> uint32_t { return ITEMS > 0 ? keys[ITEMS > 0 ? it : 0] : order_key(pooled[c]); };

  // 2. radix select: after the loop `prefix` is the key of the k-th largest value and
  //    `remaining` the number of values equal to it that must be kept
  uint32_t prefix = 0, mask = 0, remaining = (uint32_t)k;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    BinRun run;
#pragma unroll
    for (int it = 0; it < chunks; ++it) {
      const int c = it * kSelThreads + tid;
      uint32_t key = 0;
      if (c < len) key = key_at(it, c);
      run_add(hist[pass], run, c < len && (key & mask) == prefix, (key >> shift) & 255u);
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

  // 3. position-ordered emission
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  if (ITEMS > 0) {
    // cell (it, wave) = the 64 candidates wave `wave` holds in chunk `it`; cells in index order
    // it*16 + wave are in position order.  Count, scan the cells once, then write.
    uint32_t my_gt = 0, my_eq = 0;   // lane `it` keeps the counts of cell (it, wave)
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int c = it * kSelThreads + tid;
      const uint32_t key = keys[ITEMS > 0 ? it : 0];
      const uint64_t b_gt = __ballot(c < len && key > thr), b_eq = __ballot(c < len && key == thr);
      if (lane == it) { my_gt = __popcll(b_gt); my_eq = __popcll(b_eq); }
    }
    if (lane < ITEMS) { cell_gt[lane * kSelWaves + wave] = my_gt; cell_eq[lane * kSelWaves + wave] = my_eq; }
    __syncthreads();
    scan_cells(cell_gt, cell_eq, kCells, wave_gt, wave_eq, tid, lane, wave);
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int c = it * kSelThreads + tid;
      const uint32_t key = keys[ITEMS > 0 ? it : 0];
      const bool gt = c < len && key > thr;
      const bool eq = c < len && key == thr;
      const uint64_t b_gt = __ballot(gt), b_eq = __ballot(eq);
      const uint32_t gt_before = cell_gt[it * kSelWaves + wave] + __popcll(b_gt & lt_mask);
      const uint32_t eq_before = cell_eq[it * kSelWaves + wave] + __popcll(b_eq & lt_mask);
      if (gt) out[gt_before + min(eq_before, need_eq)] = cand_pos(begin + c, p.block_off, p.block_len);
      else if (eq && eq_before < need_eq) out[gt_before + eq_before] = cand_pos(begin + c, p.block_off, p.block_len);
    }
    return;
  }
  // unbounded variant: one chunk of 1024 candidates at a time
  uint32_t run_gt = 0, run_eq = 0;
  for (int it = 0; it < chunks; ++it) {
    const int c = it * kSelThreads + tid;
    uint32_t key = 0;
    if (c < len) key = key_at(it, c);
    const bool gt = c < len && key > thr;
    const bool eq = c < len && key == thr;
    const uint64_t b_gt = __ballot(gt), b_eq = __ballot(eq);
    if (lane == 0) { wave_gt[wave] = __popcll(b_gt); wave_eq[wave] = __popcll(b_eq); }
    __syncthreads();
    uint32_t off_gt = 0, off_eq = 0, tot_gt = 0, tot_eq = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const uint32_t g = wave_gt[w], e = wave_eq[w];
      if (w < wave) { off_gt += g; off_eq += e; }
      tot_gt += g; tot_eq += e;
    }
    const uint32_t gt_before = run_gt + off_gt + __popcll(b_gt & lt_mask);
    const uint32_t eq_before = run_eq + off_eq + __popcll(b_eq & lt_mask);
    if (gt) out[gt_before + min(eq_before, need_eq)] = cand_pos(begin + c, p.block_off, p.block_len);
    else if (eq && eq_before < need_eq) out[gt_before + eq_before] = cand_pos(begin + c, p.block_off, p.block_len);
    run_gt += tot_gt;
    run_eq += tot_eq;
    __syncthreads();
  }
}

constexpr int kSelMaxItems = 36;   // chunks of 1024 candidates whose keys fit in LDS
constexpr int kSelRegItems = 8;    // longest register-resident variant
constexpr int kSelBatch = 12;      // chunks pooled together (their loads in flight together) by select_lds_kernel
constexpr int kSelRead = 8;        // keys a thread fetches from LDS together in the later phases

// This thread's keys of chunks it0 .. it0 + kSelRead - 1, all requested before any is used (one LDS
// latency per eight keys instead of one per key; a rolled loop with an atomic in its body is not
// pipelined by the compiler).  Slots past the end of the segment read as 0 and are never active.
// 33 248 candidates x 4 rows: 43.2 -> 40.1 us; of those, pooling is 8 us, emission 14 us and the four
// radix passes the rest, which is the LDS atomic rate of the two passes in which nearly every key is
// still active (about 33 000 single-key runs each).
__device__ __forceinline__ void lds_read_keys(const uint32_t* lds_keys, int it0, int tid, int len, uint32_t (&key)[kSelRead]) {
#pragma unroll
  for (int u = 0; u < kSelRead; ++u) {
    const int c = (it0 + u) * kSelThreads + tid;
    key[u] = c < len ? lds_keys[c] : 0u;
  }
}

size_t select_lds_bytes(int chunks) { return (size_t)chunks * kSelThreads * sizeof(uint32_t); }

// Long segments: same three phases with the keys in dynamic LDS ([chunk][thread], so every thread
// reads back the slots it wrote and no phase needs more synchronisation than in select_kernel) and
// rolled loops over the chunks.
template <int HALF>
__global__ __launch_bounds__(kSelThreads) void select_lds_kernel(const SelectParams p) {
  extern __shared__ uint32_t lds_keys[];
  __shared__ uint32_t hist[4][256];
  __shared__ uint32_t wave_gt[kSelWaves], wave_eq[kSelWaves];
  __shared__ uint32_t cell_gt[kSelMaxItems * kSelWaves], cell_eq[kSelMaxItems * kSelWaves];
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
  const float* score = p.score + (size_t)row * p.n_cand + begin;
  float* pooled = p.pooled ? p.pooled + (size_t)row * p.n_cand + begin : nullptr;
  int32_t* out = idx_row + p.seg_out[seg];
  const int chunks = (len + kSelThreads - 1) / kSelThreads;   // <= kSelMaxItems (launcher)
  if (len <= 0) return;   // an empty segment: no load at all

  // 1. pooling, kSelBatch chunks at a time
  const int half = p.pool_half;
  const float inv_s = 1.f / (float)(2 * half + 1);
  for (int it0 = 0; it0 < chunks; it0 += kSelBatch) {
    float pv[kSelBatch];
    if (HALF >= 0) {
      pool_chunks<kSelBatch, (HALF >= 0 ? HALF : 0)>(score, len, it0, tid, lane, p.avg_pool, inv_s, pv);
    } else {
#pragma unroll
      for (int u = 0; u < kSelBatch; ++u) {
        const int c = (it0 + u) * kSelThreads + tid;
        pv[u] = c < len ? pool_at(score, c, len, half, p.avg_pool, inv_s) : 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < kSelBatch; ++u) {
      const int c = (it0 + u) * kSelThreads + tid;
      if (c < len) {
        lds_keys[c] = order_key(pv[u]);
        if (pooled) pooled[c] = pv[u];
      }
    }
  }
  if (k <= 0) return;
  if (k >= len) {
    for (int c = tid; c < len; c += kSelThreads) out[c] = cand_pos(begin + c, p.block_off, p.block_len);
    return;
  }
  for (int i = tid; i < 4 * 256; i += kSelThreads) (&hist[0][0])[i] = 0;
  __syncthreads();

  // 2. radix select
  uint32_t prefix = 0, mask = 0, remaining = (uint32_t)k;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    BinRun run;
    for (int it0 = 0; it0 < chunks; it0 += kSelRead) {
      uint32_t key[kSelRead];
      lds_read_keys(lds_keys, it0, tid, len, key);
#pragma unroll
      for (int u = 0; u < kSelRead; ++u) {
        const int c = (it0 + u) * kSelThreads + tid;
        run_add(hist[pass], run, c < len && (key[u] & mask) == prefix, (key[u] >> shift) & 255u);
      }
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

  // 3. position-ordered emission: count every (chunk, wave) cell, scan the cells once, write
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  uint32_t my_gt = 0, my_eq = 0;   // lane `it` keeps the counts of cell (it, wave)
  for (int it0 = 0; it0 < chunks; it0 += kSelRead) {
    uint32_t key[kSelRead];
    lds_read_keys(lds_keys, it0, tid, len, key);
#pragma unroll
    for (int u = 0; u < kSelRead; ++u) {
      const int c = (it0 + u) * kSelThreads + tid;
      const uint64_t b_gt = __ballot(c < len && key[u] > thr), b_eq = __ballot(c < len && key[u] == thr);
      if (lane == it0 + u) { my_gt = __popcll(b_gt); my_eq = __popcll(b_eq); }
    }
  }
  if (lane < chunks) { cell_gt[lane * kSelWaves + wave] = my_gt; cell_eq[lane * kSelWaves + wave] = my_eq; }
  __syncthreads();
  scan_cells(cell_gt, cell_eq, chunks * kSelWaves, wave_gt, wave_eq, tid, lane, wave);
  for (int it0 = 0; it0 < chunks; it0 += kSelRead) {
    uint32_t key[kSelRead], cg[kSelRead], ce[kSelRead];
    lds_read_keys(lds_keys, it0, tid, len, key);
#pragma unroll
    for (int u = 0; u < kSelRead; ++u) {
      const int cell = min(it0 + u, chunks - 1) * kSelWaves + wave;
      cg[u] = cell_gt[cell];
      ce[u] = cell_eq[cell];
    }
#pragma unroll
    for (int u = 0; u < kSelRead; ++u) {
      const int c = (it0 + u) * kSelThreads + tid;
      const bool gt = c < len && key[u] > thr;
      const bool eq = c < len && key[u] == thr;
      const uint64_t b_gt = __ballot(gt), b_eq = __ballot(eq);
      const uint32_t gt_before = cg[u] + __popcll(b_gt & lt_mask);
      const uint32_t eq_before = ce[u] + __popcll(b_eq & lt_mask);
      if (gt) out[gt_before + min(eq_before, need_eq)] = cand_pos(begin + c, p.block_off, p.block_len);
      else if (eq && eq_before < need_eq) out[gt_before + eq_before] = cand_pos(begin + c, p.block_off, p.block_len);
    }
  }
}

// true when the segment is too long for the variants that keep the pooled keys on chip, which is the
// only case in which the pooled row has to exist in memory
bool select_needs_pooled_buffer(const SelectParams& p) {
  for (int i = 0; i < p.n_seg; ++i)
    if (p.seg_len[i] > kSelMaxItems * kSelThreads) return true;
  return false;
}

template <int ITEMS>
static void launch_items(const SelectParams& p, dim3 grid, hipStream_t s) {
  const dim3 block(kSelThreads);
  if constexpr (ITEMS == 0) {
    hipLaunchKernelGGL((select_kernel<0, -1>), grid, block, 0, s, p);
    return;
  }
  switch (p.pool_half) {
    case 0: hipLaunchKernelGGL((select_kernel<ITEMS, 0>), grid, block, 0, s, p); break;
    case 1: hipLaunchKernelGGL((select_kernel<ITEMS, 1>), grid, block, 0, s, p); break;
    case 2: hipLaunchKernelGGL((select_kernel<ITEMS, 2>), grid, block, 0, s, p); break;
    default: hipLaunchKernelGGL((select_kernel<ITEMS, -1>), grid, block, 0, s, p); break;   // wider windows: generic pooling
  }
}

template <int HALF>
static hipError_t launch_lds(const SelectParams& p, dim3 grid, int chunks, hipStream_t s) {
  static LdsOptIn lds;
  const hipError_t e = lds.ensure(reinterpret_cast<const void*>(select_lds_kernel<HALF>), (int)select_lds_bytes(kSelMaxItems));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(select_lds_kernel<HALF>, grid, dim3(kSelThreads), select_lds_bytes(chunks), s, p);
  return hipGetLastError();
}

hipError_t launch_select(const SelectParams& p, hipStream_t s) {
  const int nx = p.n_seg + (p.tail_len > 0 ? 1 : 0);
  if (nx == 0 || p.rows == 0) return hipSuccess;
  // every ranked segment and the unconditional tail lie inside a score row of n_cand candidates, so
  // no workgroup reads past rows * n_cand floats of the score buffer
  for (int i = 0; i < p.n_seg; ++i)
    if (p.seg_begin[i] < 0 || p.seg_len[i] < 0 || p.seg_begin[i] + p.seg_len[i] > p.n_cand || p.seg_k[i] > p.seg_len[i])
      return hipErrorInvalidValue;
  if (p.tail_len > 0 && (p.tail_begin < 0 || p.tail_begin + p.tail_len > p.n_cand)) return hipErrorInvalidValue;
  int longest = 0;
  for (int i = 0; i < p.n_seg; ++i) longest = p.seg_len[i] > longest ? p.seg_len[i] : longest;
  const dim3 grid(nx, p.rows);
  if (longest <= 1 * kSelThreads) launch_items<1>(p, grid, s);
  else if (longest <= 2 * kSelThreads) launch_items<2>(p, grid, s);
  else if (longest <= 4 * kSelThreads) launch_items<4>(p, grid, s);
  else if (longest <= kSelRegItems * kSelThreads) launch_items<kSelRegItems>(p, grid, s);
  else if (longest <= kSelMaxItems * kSelThreads) {
    const int chunks = (longest + kSelThreads - 1) / kSelThreads;
    switch (p.pool_half) {
      case 0: return launch_lds<0>(p, grid, chunks, s);
      case 1: return launch_lds<1>(p, grid, chunks, s);
      case 2: return launch_lds<2>(p, grid, chunks, s);
      default: return launch_lds<-1>(p, grid, chunks, s);
    }
  } else launch_items<0>(p, grid, s);
  return hipGetLastError();
}

}  // namespace sdllm
