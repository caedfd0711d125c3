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
// memory exactly once.  ITEMS = 0 is the unbounded variant that re-reads the pooled row from
// memory (L2) in every pass.
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

// Histogram increment that collapses the common case "every active lane of the wave hits the
// same bin" (softmax scores share their exponent byte) into one LDS atomic.
__device__ __forceinline__ void hist_add(uint32_t* hist, bool active, uint32_t bin, int lane) {
  const uint64_t act = __ballot(active);
  if (act == 0) return;
  const int leader = __ffsll((long long)act) - 1;
  const uint32_t lead_bin = __shfl(bin, leader);
  const uint64_t same = __ballot(active && bin == lead_bin);
  if (same == act) {
    if (lane == leader) atomicAdd(&hist[lead_bin], (uint32_t)__popcll(act));
  } else if (active) {
    atomicAdd(&hist[bin], 1u);
  }
}

template <int ITEMS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectParams p) {
  __shared__ uint32_t hist[4][256];
  __shared__ uint32_t wave_gt[kSelWaves], wave_eq[kSelWaves];
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

  // 1. pooling
  const int half = p.pool_half;
  const float inv_s = 1.f / (float)(2 * half + 1);
  uint32_t keys[ITEMS > 0 ? ITEMS : 1];
  if (ITEMS > 0) {
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
#pragma unroll
    for (int it = 0; it < chunks; ++it) {
      const int c = it * kSelThreads + tid;
      uint32_t key = 0;
      if (c < len) key = key_at(it, c);
      hist_add(hist[pass], c < len && (key & mask) == prefix, (key >> shift) & 255u, lane);
    }
    __syncthreads();
    if (wave == 0) {
      const uint32_t* h = hist[pass];
      const uint32_t h0 = h[4 * lane], h1 = h[4 * lane + 1], h2 = h[4 * lane + 2], h3 = h[4 * lane + 3];
      const uint32_t lane_sum = h0 + h1 + h2 + h3;
      uint32_t suf = lane_sum;   // inclusive suffix sum over lanes
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_down(suf, o);
        if (lane + o < 64) suf += t;
      }
      const uint32_t a3 = suf - lane_sum, a2 = a3 + h3, a1 = a2 + h2, a0 = a1 + h1;
      if (a3 < remaining && remaining <= a3 + h3) { s_bin = 4 * lane + 3; s_above = a3; }
      if (a2 < remaining && remaining <= a2 + h2) { s_bin = 4 * lane + 2; s_above = a2; }
      if (a1 < remaining && remaining <= a1 + h1) { s_bin = 4 * lane + 1; s_above = a1; }
      if (a0 < remaining && remaining <= a0 + h0) { s_bin = 4 * lane; s_above = a0; }
    }
    __syncthreads();
    prefix |= s_bin << shift;
    mask |= 255u << shift;
    remaining -= s_above;
  }
  const uint32_t thr = prefix;
  const uint32_t need_eq = remaining;

  // 3. position-ordered emission
  uint32_t run_gt = 0, run_eq = 0;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
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

constexpr int kSelMaxItems = 36;

// true when the segment is too long for the register-resident variants, which is the only case in
// which the pooled row has to exist in memory
bool select_needs_pooled_buffer(const SelectParams& p) {
  for (int i = 0; i < p.n_seg; ++i)
    if (p.seg_len[i] > kSelMaxItems * kSelThreads) return true;
  return false;
}

hipError_t launch_select(const SelectParams& p, hipStream_t s) {
  const int nx = p.n_seg + (p.tail_len > 0 ? 1 : 0);
  if (nx == 0 || p.rows == 0) return hipSuccess;
  int longest = 0;
  for (int i = 0; i < p.n_seg; ++i) longest = p.seg_len[i] > longest ? p.seg_len[i] : longest;
  const dim3 grid(nx, p.rows), block(kSelThreads);
  if (longest <= 1 * kSelThreads) hipLaunchKernelGGL(select_kernel<1>, grid, block, 0, s, p);
  else if (longest <= 2 * kSelThreads) hipLaunchKernelGGL(select_kernel<2>, grid, block, 0, s, p);
  else if (longest <= 4 * kSelThreads) hipLaunchKernelGGL(select_kernel<4>, grid, block, 0, s, p);
  else if (longest <= 8 * kSelThreads) hipLaunchKernelGGL(select_kernel<8>, grid, block, 0, s, p);
  else if (longest <= 16 * kSelThreads) hipLaunchKernelGGL(select_kernel<16>, grid, block, 0, s, p);
  else if (longest <= kSelMaxItems * kSelThreads) hipLaunchKernelGGL(select_kernel<kSelMaxItems>, grid, block, 0, s, p);
  else hipLaunchKernelGGL(select_kernel<0>, grid, block, 0, s, p);
  return hipGetLastError();
}

}  // namespace sdllm
