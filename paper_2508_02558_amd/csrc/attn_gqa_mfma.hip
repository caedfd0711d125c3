// Grouped-query variant of the bf16 MFMA block attention (Alg. 3, cache_state == 2, and the dense
// block rows of states 0/1) for models whose G query heads share one KV head (2 <= G <= 8).
//
// One workgroup serves one (batch, KV head) and a range of key tiles; wave w is query head
// g*G + w.  The K/V tiles are loaded ONCE per workgroup, cooperatively and fully coalesced, into a
// double-buffered LDS stage of one 32-key tile (K and V: 18.5 KB), and all G waves run their own
// logits / online softmax / PV product against the same stage, so K and V leave HBM (and L2) once
// however many query heads read them.  One workgroup barrier per tile; the next tile's global
// loads are in flight while the current one is computed.  Each wave owns its head's result, so there
// is no cross-wave merge; key splits write fp32 partials for the combine kernel.
#include "attn_tile_math.h"

namespace sdllm {

constexpr int kStageBytes = kTileBytes + kVTileBytes;   // one 32-key tile: K, V
constexpr int kTileChunks = 512;              // 16-byte pieces of one tensor of a tile
constexpr int kMaxStageIters = 4;             // pieces per thread and tensor with the fewest threads (G = 2)

size_t attn_gqa_lds_bytes() { return 2 * (size_t)kStageBytes; }

// K and V of one tile into registers, all threads of the workgroup together: piece c = tid + j*T is
// 16-byte chunk c%16 of row c/16.  The tile base is workgroup-uniform and K and V share offsets.
__device__ __forceinline__ void load_stage(const TileSrc& ts, uint32_t stride, int tid, int nthreads,
                                           u32x4 (&kreg)[kMaxStageIters], u32x4 (&vreg)[kMaxStageIters]) {
#pragma unroll
  for (int j = 0; j < kMaxStageIters; ++j) {
    const int c = tid + j * nthreads;
    if (c < kTileChunks) {
      int r = c >> 4;
      r = r < ts.rows ? r : ts.rows - 1;       // rows past the end re-read the last key; masked later
      const uint32_t off = (uint32_t)r * stride + ((c & 15) << 4);
      kreg[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ts.k + off));
      vreg[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ts.v + off));
    }
  }
}

__device__ __forceinline__ void store_stage(uint8_t* stage, int tid, int nthreads, const u32x4 (&kreg)[kMaxStageIters],
                                            const u32x4 (&vreg)[kMaxStageIters]) {
#pragma unroll
  for (int j = 0; j < kMaxStageIters; ++j) {
    const int c = tid + j * nthreads;
    if (c < kTileChunks) {
      *reinterpret_cast<u32x4*>(stage + tile_off(c >> 4, c & 15)) = kreg[j];
      *reinterpret_cast<u32x4*>(stage + kTileBytes + vtile_off(c >> 4, c & 15)) = vreg[j];
    }
  }
}

template <int NSEG>
__global__ __launch_bounds__(512) void attn_gqa_mfma_bf16_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  const int tid = threadIdx.x;
  const int nthreads = blockDim.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // query head within the group
  const int half = lane >> 5;
  const int col = lane & 31;
  const int split = blockIdx.x;
  const int bg = blockIdx.y;
  const int b = bg / p.hkv;
  const int g = bg - b * p.hkv;
  const int h = g * p.group + wave;
  const int head = b * p.hq + h;

  const SegPtrs sp = seg_ptrs(p, b, g, NSEG == 2);
  const int ntiles = sp.tiles0 + (sp.n1 + kTileKeys - 1) / kTileKeys;
  const int t_begin = split * p.tiles_per_split;
  const int t_end = min(ntiles, t_begin + p.tiles_per_split);

  bf16x8 qf[8];
  load_q_frags((const char*)p.q + 2 * (b * p.q_sb + h * p.q_sh + col * p.q_sr), half, qf);

  f32x16 acc[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[e][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  u32x4 kreg[kMaxStageIters], vreg[kMaxStageIters];
  uint32_t stride = 0;
  TileSrc ts = tile_src(sp, t_begin, stride);
  load_stage(ts, stride, tid, nthreads, kreg, vreg);
  store_stage(smem, tid, nthreads, kreg, vreg);
  int rows = ts.rows;
  __syncthreads();

  for (int t = t_begin; t < t_end; ++t) {
    const bool more = t + 1 < t_end;
    if (more) {
      ts = tile_src(sp, t + 1, stride);
      load_stage(ts, stride, tid, nthreads, kreg, vreg);   // in flight while this tile is computed
    }
    const uint8_t* stage = smem + ((t - t_begin) & 1) * kStageBytes;
    f32x16 sc;
    const float m_loc = tile_logits(stage, qf, rows, p.scale_log2, half, col, sc);
    tile_softmax(sc, m_loc, p.scale_log2, m_run, l_run, acc);
    tile_pv(stage + kTileBytes, sc, lane, acc);
    if (more) {
      store_stage(smem + ((t + 1 - t_begin) & 1) * kStageBytes, tid, nthreads, kreg, vreg);
      rows = ts.rows;
    }
    __syncthreads();
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const size_t slot = (size_t)head * p.n_split + split;
  write_wave_result(acc, m_run, l_tot, lane, half, col, p.n_split == 1,
                    (char*)p.out + 2 * (b * p.o_sb + h * p.o_sh + col * p.o_sr), p.part_o + (slot * 32 + col) * 128,
                    p.part_ml + slot * 64);
}

template <int NSEG>
static hipError_t launch_nseg(const AttnParams& p, hipStream_t s) {
  static LdsOptIn lds;
  const hipError_t e = lds.ensure(reinterpret_cast<const void*>(attn_gqa_mfma_bf16_kernel<NSEG>), (int)attn_gqa_lds_bytes());
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_gqa_mfma_bf16_kernel<NSEG>, dim3(p.n_split, p.batch * p.hkv), dim3(p.group * kWave),
                     attn_gqa_lds_bytes(), s, p);
  return hipGetLastError();
}

bool attn_gqa_supports_group(int group) { return group >= 2 && group <= 8; }

hipError_t launch_attn_gqa_mfma_bf16(const AttnParams& p, hipStream_t s) {
  if (p.seg[0].n > 0 && p.seg[1].n > 0) return launch_nseg<2>(p, s);
  if (p.seg[1].n > 0) {   // empty cache: the block is the only key tensor
    AttnParams q = p;
    q.seg[0] = p.seg[1];
    q.seg[1].n = 0;
    return launch_nseg<1>(q, s);
  }
  return launch_nseg<1>(p, s);
}

}  // namespace sdllm
