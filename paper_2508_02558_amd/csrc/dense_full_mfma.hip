// Full-sequence bidirectional attention (every one of the L query rows over all L keys, no mask)
// for bf16, head_dim 128: what cache states 0 and 1 run for the rows outside the current block
// (the mask predictor recomputes the whole sequence at those steps; Sec. 3.1 and the description of
// cache_state 0 in the cache-management appendix).  Compute-bound (2 L^2 d flops per head against
// 4 L d bytes), so this one is organised for the matrix cores rather than for HBM:
//   * a workgroup of 8 waves owns 256 consecutive query rows of one head, wave w the 32-row block w
//     (one 32x32 MFMA block, same fragment layout as the block-step kernels);
//   * all L keys stream through a double-buffered LDS stage of two 32-key tiles, loaded once per
//     workgroup with coalesced 16-byte loads and shared by the 8 waves: each K/V byte fetched from
//     L2 feeds 256 query rows; one workgroup barrier per 64 keys, the next stage's global loads in
//     flight meanwhile;
//   * each wave alternates one block of sixteen MFMAs (logits of tile t+1 interleaved with the PV
//     product of tile t) with one block of vector-ALU work (softmax of tile t+1), the LDS operand
//     reads for the next MFMA block requested in between: while one wave of a SIMD is in its MFMA
//     block the other one's softmax runs under it;
//   * the query-block workgroups of one head (and of the G heads of a KV group) are adjacent in the
//     grid and, after the XCD renumbering, share an L2.
#include "attn_tile_math.h"

namespace sdllm {

constexpr int kFullWaves = 8;
constexpr int kFullRowsPerWg = kFullWaves * 32;
constexpr int kFullStageTiles = 2;
constexpr int kFullKvTileBytes = kTileBytes + kVTileBytes;             // K tile + V tile
constexpr int kFullStageBytes = kFullStageTiles * kFullKvTileBytes;

size_t dense_full_lds_bytes() { return 2 * (size_t)kFullStageBytes; }

// 512 threads load one stage: thread tid takes 16-byte chunk tid%16 of row tid/16 of K and of V, of
// each of the stage's tiles.
__device__ __forceinline__ void full_load_stage(const char* k_base, const char* v_base, uint32_t stride, int first_key,
                                                int n_keys, int tid, u32x4 (&kreg)[kFullStageTiles],
                                                u32x4 (&vreg)[kFullStageTiles]) {
#pragma unroll
  for (int j = 0; j < kFullStageTiles; ++j) {
    int r = first_key + j * kTileKeys + (tid >> 4);
    r = r < n_keys ? r : n_keys - 1;          // past the end: re-read the last key, masked later
    const uint32_t off = (uint32_t)r * stride + ((tid & 15) << 4);
    kreg[j] = *reinterpret_cast<const u32x4*>(k_base + off);   // re-read by the other query blocks: keep in L2
    vreg[j] = *reinterpret_cast<const u32x4*>(v_base + off);
  }
}

__device__ __forceinline__ void full_store_stage(uint8_t* stage, int tid, const u32x4 (&kreg)[kFullStageTiles],
                                                 const u32x4 (&vreg)[kFullStageTiles]) {
#pragma unroll
  for (int j = 0; j < kFullStageTiles; ++j) {
    *reinterpret_cast<u32x4*>(stage + j * kFullKvTileBytes + tile_off(tid >> 4, tid & 15)) = kreg[j];
    *reinterpret_cast<u32x4*>(stage + j * kFullKvTileBytes + kTileBytes + vtile_off(tid >> 4, tid & 15)) = vreg[j];
  }
}

__global__ __launch_bounds__(512) void dense_full_mfma_bf16_kernel(const DenseFullParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5;
  const int col = lane & 31;

  // renumber workgroups so that consecutive ids (which go round-robin over the XCDs) of one head's
  // query blocks end up on the same XCD
  const int wg = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int qblocks = (p.seq_len + kFullRowsPerWg - 1) / kFullRowsPerWg;
  const int qb = wg % qblocks;
  const int head = wg / qblocks;
  const int b = head / p.hq;
  const int h = head - b * p.hq;
  const int g = h / p.group;

  // rows past the end of the sequence compute on a copy of the last row and are not written back:
  // every wave then runs the same program, barriers included
  const int q_row = qb * kFullRowsPerWg + wave * 32 + col;
  const bool row_valid = q_row < p.seq_len;
  const int q_row_c = row_valid ? q_row : p.seq_len - 1;
  bf16x8 qf[8];
  load_q_frags((const char*)p.q + 2 * (b * p.q_sb + h * p.q_sh + (int64_t)q_row_c * p.q_sr), half, qf);

  const char* k_base = (const char*)p.k + 2 * (b * p.k_sb + g * p.k_sh);
  const char* v_base = (const char*)p.v + 2 * (b * p.k_sb + g * p.k_sh);
  const uint32_t stride = (uint32_t)(p.k_sr * 2);
  const int n_keys = p.seq_len;
  const int stage_keys = kFullStageTiles * kTileKeys;
  const int nstages = (n_keys + stage_keys - 1) / stage_keys;
  const int ntiles = (n_keys + kTileKeys - 1) / kTileKeys;

  f32x16 acc[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[e][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // Pipeline state between iterations: pb = softmax numerators of the current tile t (bf16), f = its V
  // fragments, a = the K fragments of tile t+1.  Iteration t issues one MFMA block (logits of t+1, PV
  // of t), requests the fragments the next block needs from LDS, and runs the softmax of t+1 while
  // they arrive.  Tile t lives in stage t/2; stage s+1 is published (and the barrier met) in the even
  // iteration 2s, after the last read of stage s (V of tile 2s+1) has been requested and before the
  // first read of stage s+1 (K of tile 2s+2).
  u32x4 kreg[kFullStageTiles], vreg[kFullStageTiles];
  full_load_stage(k_base, v_base, stride, 0, n_keys, tid, kreg, vreg);
  full_store_stage(smem, tid, kreg, vreg);
  __syncthreads();
  if (nstages > 1) full_load_stage(k_base, v_base, stride, stage_keys, n_keys, tid, kreg, vreg);

  bf16x8 a[8], pb[2];
  PvFrags f;
  f32x16 sn;
  tile_k_load(smem, half, col, a);
  __builtin_amdgcn_sched_barrier(0);
  tile_logits_mma(a, qf, sn);
  tile_pv_load(smem + kTileBytes, lane, f);
  if (ntiles > 1) tile_k_load(smem + kFullKvTileBytes, half, col, a);
  __builtin_amdgcn_sched_barrier(0);
  softmax_block(sn, min(kTileKeys, n_keys), p.scale_log2, half, m_run, l_run, acc, pb);

  for (int t = 0; t + 1 < ntiles; ++t) {   // t = current tile
    const int s = t >> 1;
    const bool even = (t & 1) == 0;
    const uint8_t* stage = smem + (s & 1) * kFullStageBytes;
    uint8_t* next_stage = smem + ((s + 1) & 1) * kFullStageBytes;
    __builtin_amdgcn_sched_barrier(0);
    mfma_block(a, qf, sn, f, pb, acc);
    __builtin_amdgcn_sched_barrier(0);
    // V of tile t+1: second tile of stage s (its last read) or first tile of stage s+1
    tile_pv_load((even ? stage + kFullKvTileBytes : next_stage) + kTileBytes, lane, f);
    if (even && s + 1 < nstages) {
      full_store_stage(next_stage, tid, kreg, vreg);
      __syncthreads();
      if (s + 2 < nstages) full_load_stage(k_base, v_base, stride, (s + 2) * stage_keys, n_keys, tid, kreg, vreg);
    }
    // K of tile t+2: first or second tile of stage s+1
    if (t + 2 < ntiles) tile_k_load(even ? next_stage : next_stage + kFullKvTileBytes, half, col, a);
    __builtin_amdgcn_sched_barrier(0);
    softmax_block(sn, min(kTileKeys, n_keys - (t + 1) * kTileKeys), p.scale_log2, half, m_run, l_run, acc, pb);
  }
  // PV product of the last tile
  __builtin_amdgcn_sched_barrier(0);
  pv_block(f, pb, acc);

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (row_valid) {
    char* out_row = (char*)p.out + 2 * (b * p.o_sb + h * p.o_sh + (int64_t)q_row * p.o_sr);
    write_wave_result(acc, m_run, l_tot, lane, half, true, out_row, nullptr, nullptr);
  }
}

hipError_t launch_dense_full_mfma_bf16(const DenseFullParams& p, hipStream_t s) {
  static LdsOptIn lds;
  const hipError_t e = lds.ensure(reinterpret_cast<const void*>(dense_full_mfma_bf16_kernel), (int)dense_full_lds_bytes());
  if (e != hipSuccess) return e;
  const int qblocks = (p.seq_len + kFullRowsPerWg - 1) / kFullRowsPerWg;
  hipLaunchKernelGGL(dense_full_mfma_bf16_kernel, dim3(qblocks * p.batch * p.hq), dim3(512), dense_full_lds_bytes(), s, p);
  return hipGetLastError();
}

}  // namespace sdllm
