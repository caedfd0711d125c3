// Full-sequence bidirectional attention (every one of the L query rows over all L keys, no mask)
// for bf16, head_dim 128: what cache states 0 and 1 run for the rows outside the current block
// (the mask predictor recomputes the whole sequence at those steps; Sec. 3.1 and the description of
// cache_state 0 in the cache-management appendix).  Compute-bound (2 L^2 d flops per head against
// 4 L d bytes), so this one is organised for the matrix cores rather than for HBM:
//   * a workgroup of 8 waves owns 256 consecutive query rows of one head, wave w the 32-row block w
//     (one 32x32 MFMA block, same fragment layout as the block-step kernels);
//   * all L keys stream through a double-buffered LDS stage of two 32-key tiles, loaded once per
//     workgroup with coalesced 16-byte loads and shared by the 8 waves: each K/V byte fetched from
//     L2 feeds 256 query rows;
//   * one workgroup barrier per 64 keys, the next stage's global loads in flight meanwhile;
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
  int wg = blockIdx.x;
  const int nwg = gridDim.x;
  if ((nwg & (kNumXCDs - 1)) == 0) wg = (wg & (kNumXCDs - 1)) * (nwg / kNumXCDs) + wg / kNumXCDs;
  const int qblocks = (p.seq_len + kFullRowsPerWg - 1) / kFullRowsPerWg;
  const int qb = wg % qblocks;
  const int head = wg / qblocks;
  const int b = head / p.hq;
  const int h = head - b * p.hq;
  const int g = h / p.group;

  const int q_row = qb * kFullRowsPerWg + wave * 32 + col;
  const bool row_valid = q_row < p.seq_len;
  const bool wave_valid = qb * kFullRowsPerWg + wave * 32 < p.seq_len;
  const int q_row_c = row_valid ? q_row : p.seq_len - 1;
  bf16x8 qf[8];
  load_q_frags((const char*)p.q + 2 * (b * p.q_sb + h * p.q_sh + (int64_t)q_row_c * p.q_sr), half, qf);

  const char* k_base = (const char*)p.k + 2 * (b * p.k_sb + g * p.k_sh);
  const char* v_base = (const char*)p.v + 2 * (b * p.k_sb + g * p.k_sh);
  const uint32_t stride = (uint32_t)(p.k_sr * 2);
  const int n_keys = p.seq_len;
  const int stage_keys = kFullStageTiles * kTileKeys;
  const int nstages = (n_keys + stage_keys - 1) / stage_keys;

  f32x16 acc[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[e][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  u32x4 kreg[kFullStageTiles], vreg[kFullStageTiles];
  full_load_stage(k_base, v_base, stride, 0, n_keys, tid, kreg, vreg);
  full_store_stage(smem, tid, kreg, vreg);
  __syncthreads();

  for (int s = 0; s < nstages; ++s) {
    if (s + 1 < nstages) full_load_stage(k_base, v_base, stride, (s + 1) * stage_keys, n_keys, tid, kreg, vreg);
    const uint8_t* stage = smem + (s & 1) * kFullStageBytes;
    if (wave_valid)
      tiles_pipelined<kFullStageTiles>(stage, kFullKvTileBytes, qf, n_keys - s * stage_keys, p.scale_log2, lane, m_run,
                                       l_run, acc);
    if (s + 1 < nstages) full_store_stage(smem + ((s + 1) & 1) * kFullStageBytes, tid, kreg, vreg);
    __syncthreads();
  }

  if (!wave_valid) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (row_valid) {
    char* out_row = (char*)p.out + 2 * (b * p.o_sb + h * p.o_sh + (int64_t)q_row * p.o_sr);
    write_wave_result(acc, m_run, l_tot, lane, half, col, true, out_row, nullptr, nullptr);
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
