// Pooling + top-k retention (Sec. 3.3 third equation; Alg. 1 steps 8-10) and, fused into the last
// stage, the gather of the retained K/V rows (Sec. 3.3 fourth equation; Alg. 1 steps 12-14).
//
// Three stages per (batch, KV head) row and ranked segment (prefix / suffix, or the joint array):
//   1. pooling: stride-1 pooling of the score with window s clipped to the segment (-inf padding for
//      max, zero padding and a fixed divisor s for avg); the pooled values are kept as order-preserving
//      32-bit integer keys (larger float <=> larger key) in a key buffer;
//   2. threshold: an MSB-first radix select on the keys finds the exact k-th largest value T and how
//      many entries equal to T have to be kept (k minus the number of larger ones);
//   3. emission: in position order, every key above T and the first entries equal to T are kept, so
//      ties go to the lower position and the output is ascending without a sort; the workgroup that
//      emits a run of retained positions also copies their K/V rows into the cache (the retained
//      entries of a run of candidates occupy consecutive cache rows).
// Max pooling copies a peak to its neighbours, so T routinely falls inside a group of equal values;
// the tie rule is exercised constantly, not only in corner cases.
//
// Segments of up to 8 x 1024 candidates: one 1024-thread workgroup does stages 1 and 2
// (select_threshold_kernel: keys in registers, four 8-bit radix passes with LDS histograms).
// Longer segments: stage 1 is spread over one workgroup per 2048 candidates (select_pool_kernel),
// each of which also leaves a compact list of the non-empty bins of its keys' leading 12 bits; one
// workgroup per segment (select_resolve_kernel) adds the lists up, finds the bin that holds the k-th
// value, collects that bin's members (a few hundred keys as a rule) and resolves the remaining 20 bits
// on them alone.  Stage 3 (select_emit_kernel) is always one 256-thread workgroup per 1024 candidates;
// it recounts the entries before its own candidates itself, so stage 2 only has to publish T.
#include "sdllm_internal.h"

namespace sdllm {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelRegItems = 8;                        // longest register-resident variant (chunks of 1024)
constexpr int kPoolChunks = 2;                         // chunks of 1024 candidates per select_pool_kernel workgroup
constexpr int kPartLen = kPoolChunks * kSelThreads;
constexpr int kBinShift = 20, kBins = 4096;            // leading 12 bits of a key
constexpr int kBinListCap = kPartLen;                  // a part cannot occupy more bins than it has candidates
constexpr int kBinListStride = 1 + 2 * kBinListCap;    // words per list: count, then (bin, count) pairs
constexpr int kMemberCap = 8192;                       // members of the threshold bin held in LDS by select_resolve_kernel
constexpr int kEmitThreads = 256;
constexpr int kEmitWaves = kEmitThreads / 64;
constexpr int kEmitItems = 4;
constexpr int kEmitChunk = kEmitThreads * kEmitItems;  // candidates per select_emit_kernel workgroup

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

// The pair stage 3 reads per (row, ranked segment): threshold key and number of equal keys to keep.
// "keep everything" is (0, len): every key is above or equal to 0; "keep nothing" is (max, 0).
__device__ __forceinline__ void publish_threshold(uint32_t* thr, int row, int seg, uint32_t key, uint32_t need_eq) {
  thr[(row * 2 + seg) * 2] = key;
  thr[(row * 2 + seg) * 2 + 1] = need_eq;
}

// ------------------------------------------------------------------ stages 1 + 2, one workgroup per segment
template <int ITEMS, int HALF>
__global__ __launch_bounds__(kSelThreads) void select_threshold_kernel(const SelectParams p) {
  __shared__ uint32_t hist[4][256];
  __shared__ uint32_t s_bin, s_above;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int row = blockIdx.y;
  const int seg = blockIdx.x;
  const int begin = p.seg_begin[seg];
  const int len = p.seg_len[seg];
  const int k = p.seg_k[seg];
  if (len <= 0 || k <= 0) {   // an empty segment (no suffix after the last block, no prefix before the first): no load at all
    if (tid == 0) publish_threshold(p.thr, row, seg, 0xffffffffu, 0u);
    if (len <= 0) return;
  } else if (k >= len) {
    if (tid == 0) publish_threshold(p.thr, row, seg, 0u, (uint32_t)len);
  }
  const float* score = p.score + (size_t)row * p.n_cand + begin;
  float* pooled = p.pooled ? p.pooled + (size_t)row * p.n_cand + begin : nullptr;
  uint32_t* key_out = p.keys + (size_t)row * p.n_cand + begin;

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
      key_out[c] = keys[it];
      if (pooled) pooled[c] = pv[it];
    }
  }
  if (k <= 0 || k >= len) return;
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
  if (tid == 0) publish_threshold(p.thr, row, seg, prefix, remaining);
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
__global__ __launch_bounds__(kSelThreads) void select_resolve_kernel(const SelectParams p) {
  __shared__ uint32_t members[kMemberCap];
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t hist2[3][256];
  __shared__ uint32_t wave_tot[kSelWaves];
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

  for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
  for (int i = tid; i < 3 * 256; i += kSelThreads) (&hist2[0][0])[i] = 0;
  if (tid == 0) s_members = 0;
  __syncthreads();

  // add up the parts' bin lists: wave w takes parts w, w + 16, ...
  const int parts_used = (len + kPartLen - 1) / kPartLen;
  for (int part = wave; part < parts_used; part += kSelWaves) {
    const uint32_t* list = p.bins + ((size_t)(row * 2 + seg) * p.parts + part) * kBinListStride;
    const int n = min((int)list[0], kBinListCap);
    for (int i0 = 0; i0 < n; i0 += 4 * 64) {
      uint32_t bin[4], cnt[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = min(i0 + u * 64 + lane, n - 1);
        bin[u] = list[1 + 2 * i];
        cnt[u] = list[2 + 2 * i];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (i0 + u * 64 + lane < n) atomicAdd(&hist[bin[u] & (kBins - 1)], cnt[u]);
    }
  }
  __syncthreads();
  pick_bin_wide(hist, (uint32_t)k, tid, lane, wave, wave_tot, &s_bin, &s_above);
  __syncthreads();
  const uint32_t bin1 = s_bin;
  uint32_t remaining = (uint32_t)k - s_above;
  const uint32_t n_members = hist[bin1];
  const bool listed = n_members <= (uint32_t)kMemberCap;

  // collect the members of the threshold bin (their order is irrelevant: only counts are taken from
  // them); a bin with more members than the list holds is walked in the key buffer in every pass
  if (listed) {
    for (int c0 = 0; c0 < len; c0 += 8 * kSelThreads) {
      uint32_t key[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int c = c0 + u * kSelThreads + tid;
        key[u] = c < len ? keys[c] : 0u;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool in = c0 + u * kSelThreads + tid < len && (key[u] >> kBinShift) == bin1;
        const uint64_t b = __ballot(in);
        if (b != 0) {
          uint32_t base = 0;
          if (lane == 0) base = atomicAdd(&s_members, (uint32_t)__popcll(b));
          base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
          const uint32_t at = base + (uint32_t)__popcll(b & ((1ull << lane) - 1ull));
          if (in && at < (uint32_t)kMemberCap) members[at] = key[u];
        }
      }
    }
    __syncthreads();
  }

  // the remaining 20 bits, MSB first: digits of 8, 8 and 4 bits
  uint32_t prefix = bin1 << kBinShift, mask = 0xffffffffu << kBinShift;
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 12 : (pass == 1 ? 4 : 0);
    const uint32_t digit = pass == 2 ? 15u : 255u;
    BinRun run;
    if (listed) {
      for (uint32_t i = tid; i < n_members; i += kSelThreads) {
        const uint32_t key = members[i];
        run_add(hist2[pass], run, (key & mask) == prefix, (key >> shift) & digit);
      }
    } else {
      for (int c0 = 0; c0 < len; c0 += 8 * kSelThreads) {
        uint32_t key[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int c = c0 + u * kSelThreads + tid;
          key[u] = c < len ? keys[c] : 0u;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          run_add(hist2[pass], run, c0 + u * kSelThreads + tid < len && (key[u] & mask) == prefix, (key[u] >> shift) & digit);
      }
    }
    run_flush(hist2[pass], run, lane);
    __syncthreads();
    if (wave == 0) pick_bin(hist2[pass], remaining, lane, &s_bin, &s_above);
    __syncthreads();
    prefix |= s_bin << shift;
    mask |= digit << shift;
    remaining -= s_above;
  }
  if (tid == 0) publish_threshold(p.thr, row, seg, prefix, remaining);
}

// ------------------------------------------------------------------ stage 3: position-ordered emission (+ gather)
// One workgroup per kEmitChunk consecutive candidates of a segment; candidate c = chunk*1024 + it*256 + tid.
// blockIdx.y >= n_seg is the unconditional tail (prefix-only eviction keeps the whole suffix).
template <bool GATHER>
__global__ __launch_bounds__(kEmitThreads) void select_emit_kernel(const SelectParams p) {
  __shared__ uint32_t red_gt[kEmitWaves], red_eq[kEmitWaves];
  __shared__ uint32_t cell_gt[kEmitItems * kEmitWaves], cell_eq[kEmitItems * kEmitWaves];
  __shared__ int32_t pos_list[kEmitChunk];

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
  const uint32_t thr = tail ? 0u : p.thr[(row * 2 + sx) * 2];
  const uint32_t need = tail ? 0u : p.thr[(row * 2 + sx) * 2 + 1];
  const uint32_t* keys = p.keys + (size_t)row * p.n_cand + begin;
  int32_t* idx_row = p.idx + (size_t)row * p.k_total + out0;

  // entries above / equal to the threshold among the candidates before this workgroup's
  uint32_t gt_b = 0, eq_b = 0;
  if (tail) {
    gt_b = (uint32_t)c0;
  } else if (c0 > 0) {
    for (int cb = 0; cb < c0; cb += 8 * kEmitThreads) {
      uint32_t key[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int c = cb + u * kEmitThreads + tid;
        key[u] = c < c0 ? keys[c] : 0u;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool in = cb + u * kEmitThreads + tid < c0;
        gt_b += in && key[u] > thr;
        eq_b += in && key[u] == thr;
      }
    }
    for (int o = 32; o > 0; o >>= 1) {
      gt_b += __shfl_xor(gt_b, o);
      eq_b += __shfl_xor(eq_b, o);
    }
    if (lane == 0) { red_gt[wave] = gt_b; red_eq[wave] = eq_b; }
    __syncthreads();
    gt_b = eq_b = 0;
#pragma unroll
    for (int w = 0; w < kEmitWaves; ++w) { gt_b += red_gt[w]; eq_b += red_eq[w]; }
  }

  // own candidates: cell (it, wave) = 64 consecutive candidates; cells in index order are in position order
  bool gt[kEmitItems], eq[kEmitItems];
  uint64_t b_gt[kEmitItems], b_eq[kEmitItems];
  {
    uint32_t key[kEmitItems];
#pragma unroll
    for (int it = 0; it < kEmitItems; ++it) {
      const int c = c0 + it * kEmitThreads + tid;
      key[it] = (c < len && !tail) ? keys[c] : 0u;
    }
#pragma unroll
    for (int it = 0; it < kEmitItems; ++it) {
      const bool valid = c0 + it * kEmitThreads + tid < len;
      gt[it] = valid && (tail || key[it] > thr);
      eq[it] = valid && !tail && key[it] == thr;
      b_gt[it] = __ballot(gt[it]);
      b_eq[it] = __ballot(eq[it]);
      if (lane == 0) {
        cell_gt[it * kEmitWaves + wave] = (uint32_t)__popcll(b_gt[it]);
        cell_eq[it * kEmitWaves + wave] = (uint32_t)__popcll(b_eq[it]);
      }
    }
  }
  __syncthreads();
  uint32_t cg[kEmitItems * kEmitWaves], ce[kEmitItems * kEmitWaves];
#pragma unroll
  for (int j = 0; j < kEmitItems * kEmitWaves; ++j) { cg[j] = cell_gt[j]; ce[j] = cell_eq[j]; }
  // slot (relative to the segment's first output) of this workgroup's first retained candidate, and how many it retains
  const uint32_t s0 = gt_b + min(eq_b, need);
  uint32_t tot_gt = 0, tot_eq = 0;
#pragma unroll
  for (int j = 0; j < kEmitItems * kEmitWaves; ++j) { tot_gt += cg[j]; tot_eq += ce[j]; }
  const uint32_t eq_room = need > eq_b ? need - eq_b : 0u;
  const uint32_t m = tot_gt + min(tot_eq, eq_room);
  const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
  for (int it = 0; it < kEmitItems; ++it) {
    uint32_t og = 0, oe = 0;
#pragma unroll
    for (int j = 0; j < kEmitItems * kEmitWaves; ++j)
      if (j < it * kEmitWaves + wave) { og += cg[j]; oe += ce[j]; }
    const uint32_t gt_before = gt_b + og + (uint32_t)__popcll(b_gt[it] & lt_mask);
    const uint32_t eq_before = eq_b + oe + (uint32_t)__popcll(b_eq[it] & lt_mask);
    const bool kept = gt[it] || (eq[it] && eq_before < need);
    if (kept) {
      const uint32_t slot = gt[it] ? gt_before + min(eq_before, need) : gt_before + eq_before;
      const int pos = cand_pos(begin + c0 + it * kEmitThreads + tid, p.block_off, p.block_len);
      idx_row[slot] = pos;
      if (GATHER) pos_list[slot - s0] = pos;   // 0 <= slot - s0 < m <= kEmitChunk
    }
  }
  if (!GATHER) return;

  // the m retained rows go to m consecutive cache rows: pieces of 16 bytes, `lanes` threads per row,
  // two rows of K and of V in flight per thread, non-temporal both ways
  __syncthreads();
  if (m == 0) return;
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  const int b = row / p.hkv;
  const int g = row - b * p.hkv;
  const int lanes = p.row_bytes >> 4;            // 8, 16 or 32: divides kEmitThreads
  const int rows_per_pass = kEmitThreads / lanes;
  const int r_in = tid / lanes;
  const int64_t c16 = (int64_t)(tid - r_in * lanes) << 4;
  const char* src_k = (const char*)p.k + b * p.s_sb + g * p.s_sh + c16;
  const char* src_v = (const char*)p.v + b * p.s_sb + g * p.s_sh + c16;
  char* dst_k = (char*)p.kc + b * p.c_sb + g * p.c_sh + (int64_t)(out0 + s0) * p.c_sr + c16;
  char* dst_v = (char*)p.vc + b * p.c_sb + g * p.c_sh + (int64_t)(out0 + s0) * p.c_sr + c16;
  for (uint32_t r0 = 0; r0 < m; r0 += 2 * rows_per_pass) {
    const uint32_t ra = r0 + r_in, rb = ra + rows_per_pass;
    const bool oka = ra < m, okb = rb < m;
    const int64_t pa = pos_list[oka ? ra : 0], pb = pos_list[okb ? rb : 0];   // entry 0 is valid (m >= 1)
    const u32x4 ka = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src_k + pa * p.s_sr));
    const u32x4 va = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src_v + pa * p.s_sr));
    const u32x4 kb = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src_k + pb * p.s_sr));
    const u32x4 vb = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src_v + pb * p.s_sr));
    if (oka) {
      __builtin_nontemporal_store(ka, reinterpret_cast<u32x4*>(dst_k + (int64_t)ra * p.c_sr));
      __builtin_nontemporal_store(va, reinterpret_cast<u32x4*>(dst_v + (int64_t)ra * p.c_sr));
    }
    if (okb) {
      __builtin_nontemporal_store(kb, reinterpret_cast<u32x4*>(dst_k + (int64_t)rb * p.c_sr));
      __builtin_nontemporal_store(vb, reinterpret_cast<u32x4*>(dst_v + (int64_t)rb * p.c_sr));
    }
  }
}

// ------------------------------------------------------------------ launchers
size_t select_bins_words(const SelectParams& p) {   // workspace words of the bin lists (0: no long segment)
  int longest = 0;
  for (int i = 0; i < p.n_seg; ++i) longest = p.seg_len[i] > longest ? p.seg_len[i] : longest;
  if (longest <= kSelRegItems * kSelThreads) return 0;
  const size_t parts = (size_t)(longest + kPartLen - 1) / kPartLen;
  return (size_t)p.rows * 2 * parts * kBinListStride;
}

template <int ITEMS>
static void launch_threshold(const SelectParams& p, dim3 grid, hipStream_t s) {
  const dim3 block(kSelThreads);
  switch (p.pool_half) {
    case 0: hipLaunchKernelGGL((select_threshold_kernel<ITEMS, 0>), grid, block, 0, s, p); break;
    case 1: hipLaunchKernelGGL((select_threshold_kernel<ITEMS, 1>), grid, block, 0, s, p); break;
    case 2: hipLaunchKernelGGL((select_threshold_kernel<ITEMS, 2>), grid, block, 0, s, p); break;
    default: hipLaunchKernelGGL((select_threshold_kernel<ITEMS, -1>), grid, block, 0, s, p); break;   // wider windows: generic pooling
  }
}

hipError_t launch_select(const SelectParams& q, hipStream_t s) {
  SelectParams p = q;
  const int nx = p.n_seg + (p.tail_len > 0 ? 1 : 0);
  if (nx == 0 || p.rows == 0) return hipSuccess;
  if (p.rows > 65535 || p.n_seg > 2) return hipErrorInvalidValue;
  // every ranked segment and the unconditional tail lie inside a score row of n_cand candidates, so
  // no workgroup reads past rows * n_cand entries of the score or key buffers
  int longest = 0, longest_any = p.tail_len > 0 ? p.tail_len : 0;
  for (int i = 0; i < p.n_seg; ++i) {
    if (p.seg_begin[i] < 0 || p.seg_len[i] < 0 || p.seg_begin[i] + p.seg_len[i] > p.n_cand || p.seg_k[i] > p.seg_len[i])
      return hipErrorInvalidValue;
    longest = p.seg_len[i] > longest ? p.seg_len[i] : longest;
  }
  if (p.tail_len > 0 && (p.tail_begin < 0 || p.tail_begin + p.tail_len > p.n_cand)) return hipErrorInvalidValue;
  if (longest > longest_any) longest_any = longest;
  if (!p.keys || !p.thr || (!p.idx && p.k_total > 0)) return hipErrorInvalidValue;
  if (p.k && ((p.row_bytes & 15) != 0 || p.row_bytes < 16 || p.row_bytes > 16 * kEmitThreads || kEmitThreads % (p.row_bytes >> 4) != 0))
    return hipErrorInvalidValue;

  if (p.n_seg > 0 && longest > 0) {
    const dim3 grid(p.n_seg, p.rows);
    if (longest <= 1 * kSelThreads) launch_threshold<1>(p, grid, s);
    else if (longest <= 2 * kSelThreads) launch_threshold<2>(p, grid, s);
    else if (longest <= 4 * kSelThreads) launch_threshold<4>(p, grid, s);
    else if (longest <= kSelRegItems * kSelThreads) launch_threshold<kSelRegItems>(p, grid, s);
    else {
      if (!p.bins) return hipErrorInvalidValue;
      p.parts = (longest + kPartLen - 1) / kPartLen;
      const dim3 pgrid(p.parts, p.n_seg, p.rows), block(kSelThreads);
      switch (p.pool_half) {
        case 0: hipLaunchKernelGGL(select_pool_kernel<0>, pgrid, block, 0, s, p); break;
        case 1: hipLaunchKernelGGL(select_pool_kernel<1>, pgrid, block, 0, s, p); break;
        case 2: hipLaunchKernelGGL(select_pool_kernel<2>, pgrid, block, 0, s, p); break;
        default: hipLaunchKernelGGL(select_pool_kernel<-1>, pgrid, block, 0, s, p); break;
      }
      hipLaunchKernelGGL(select_resolve_kernel, grid, block, 0, s, p);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const dim3 egrid((longest_any + kEmitChunk - 1) / kEmitChunk, nx, p.rows);
  if (egrid.x > 0 && p.k_total > 0) {   // nothing retained (r = 0): no index to write, no row to copy
    if (p.k) hipLaunchKernelGGL(select_emit_kernel<true>, egrid, dim3(kEmitThreads), 0, s, p);
    else hipLaunchKernelGGL(select_emit_kernel<false>, egrid, dim3(kEmitThreads), 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace sdllm
