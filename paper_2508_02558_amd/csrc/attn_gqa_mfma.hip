// Grouped-query variant of the bf16 MFMA block attention (Alg. 3, cache_state == 2, and the dense
// block rows of states 0/1) for models whose G query heads share one KV head (G = 2, 4, 7 or 8).
//
// A workgroup serves one (batch, KV head), a range of key tiles and W of the group's query heads
// (wave w = one head).  The K/V tiles are loaded ONCE per workgroup, cooperatively and fully coalesced,
// into a double-buffered LDS stage (two 32-key tiles of K and V with 4 waves, one tile with fewer, so
// that the staging registers stay at 32 per lane), and all W waves run against the same stage.
// With several heads per key the kernel is bound by the matrix and vector pipes rather than by HBM, and
// each wave runs the software pipeline of the full-sequence kernel: one block of sixteen MFMAs (logits
// of tile j+1 interleaved with the PV product of tile j), the LDS fragment requests for the next
// block, then the softmax of tile j+1.
// Groups of 4, 7 and 8 heads are served by TWO workgroups of ceil(G/2) waves that stream the same keys:
// a CU holds 8 such waves either way, but two workgroups keep two stages of global loads in flight
// and one's load latency hides under the other's arithmetic (one 7- or 8-wave workgroup per CU spent
// a third of its time waiting for its single stage).  The pair is given linear workgroup ids 8 apart,
// so both land on the same XCD and the second read of a K/V line is an L2 hit.
// Each wave owns its head's result, so there is no cross-wave merge; key splits write fp32 partials
// for the combine kernel.
// STATS (dense launches of the cache-update step): also leave each query row's softmax (max, sum)
// over the CANDIDATE keys only, which is the row-statistics pass of the saliency scoring (Sec. 3.3,
// Alg. 1 steps 2-6).  The tiles made of candidates alone are visited first, so up to there the
// running attention statistics ARE the candidate statistics and a copy of them is all it takes; the
// one or two tiles that also hold the block's own keys (with prefix-only eviction: the suffix too)
// come last and add their candidates to that copy with a masked pass of their own.
#include "attn_tile_math.h"

namespace sdllm {

constexpr int kKvTileBytes = kTileBytes + kVTileBytes;   // one 32-key tile: K, V
constexpr int kTileChunks = 512;                         // 16-byte pieces of one tensor of a tile

constexpr int gqa_stage_tiles(int waves) { return waves >= 4 ? 2 : 1; }
constexpr int gqa_chunks(int waves) { return (kTileChunks + waves * kWave - 1) / (waves * kWave); }   // per thread, tensor and tile
constexpr size_t gqa_lds_bytes(int waves) { return 2 * (size_t)gqa_stage_tiles(waves) * kKvTileBytes; }
constexpr int gqa_head_splits(int group) { return group >= 4 ? 2 : 1; }

// Stage the tiles first_tile, ... of this workgroup's range (positions in its visiting order; tile_of
// gives the tile in memory) into registers, all threads together: piece c = tid + i*T of a tile is
// 16-byte chunk c%16 of row c/16.  A tile never straddles the two key
// segments, so its base is workgroup-uniform and K and V share offsets.
// KEEP_K: plain instead of non-temporal loads for K, because the scoring pass that follows a statistics
// launch reads the same K rows again and finds them in L2 / the memory-side cache.
template <int W, bool KEEP_K, class TileMap>
__device__ __forceinline__ void gqa_load_stage(const SegPtrs& sp, int first_tile, int t_end, int tid, const TileMap& tile_of,
                                               u32x4 (&kreg)[gqa_stage_tiles(W) * gqa_chunks(W)],
                                               u32x4 (&vreg)[gqa_stage_tiles(W) * gqa_chunks(W)]) {
  constexpr int NT = gqa_stage_tiles(W), CH = gqa_chunks(W), T = W * kWave;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    if (first_tile + j >= t_end) break;      // workgroup-uniform
    uint32_t stride;
    const TileSrc ts = tile_src(sp, tile_of(first_tile + j), stride);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = tid + i * T;
      if (CH * T == kTileChunks || c < kTileChunks) {
        int r = c >> 4;
        r = r < ts.rows ? r : ts.rows - 1;   // rows past the end re-read the last key; masked later
        const uint32_t off = (uint32_t)r * stride + ((c & 15) << 4);
        const u32x4* kp = reinterpret_cast<const u32x4*>(ts.k + off);
        kreg[j * CH + i] = KEEP_K ? *kp : __builtin_nontemporal_load(kp);
        vreg[j * CH + i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ts.v + off));
      }
    }
  }
}

template <int W>
__device__ __forceinline__ void gqa_store_stage(uint8_t* stage, int tid, const u32x4 (&kreg)[gqa_stage_tiles(W) * gqa_chunks(W)],
                                                const u32x4 (&vreg)[gqa_stage_tiles(W) * gqa_chunks(W)]) {
  constexpr int NT = gqa_stage_tiles(W), CH = gqa_chunks(W), T = W * kWave;
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = tid + i * T;
      if (CH * T == kTileChunks || c < kTileChunks) {
        *reinterpret_cast<u32x4*>(stage + j * kKvTileBytes + tile_off(c >> 4, c & 15)) = kreg[j * CH + i];
        *reinterpret_cast<u32x4*>(stage + j * kKvTileBytes + kTileBytes + vtile_off(c >> 4, c & 15)) = vreg[j * CH + i];
      }
    }
}

// Adds the candidates among a tile's keys to a row's running candidate-only (max, sum): register i of
// the raw logits is key position pos0 + 8*(i/4) + i%4; candidates are the positions before
// cand0_end or from cand1_begin on, within the sequence.  The reference mc_run is common to the two
// half-lanes of a row, the sum is per half-lane (like the attention's own pair).
__device__ __forceinline__ void tile_candidate_stats(const f32x16& sn, int pos0, const AttnParams& p, float& mc_run, float& lc_run) {
  float sc[16];
  float mc_loc = -INFINITY;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int pos = pos0 + (i >> 2) * 8 + (i & 3);
    sc[i] = ((pos < p.cand0_end || pos >= p.cand1_begin) && pos < p.seg[0].n) ? sn[i] * p.scale_log2 : -INFINITY;
    mc_loc = fmaxf(mc_loc, sc[i]);
  }
  mc_loc = fmaxf(mc_loc, __shfl_xor(mc_loc, 32));
  const float mc_new = fmaxf(mc_run, mc_loc);
  if (mc_new != -INFINITY) {
    float lc_loc = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) lc_loc += __builtin_amdgcn_exp2f(sc[i] - mc_new);
    lc_run = lc_run * __builtin_amdgcn_exp2f(mc_run - mc_new) + lc_loc;
    mc_run = mc_new;
  }
}

// two waves per SIMD (256 registers each) whatever the workgroup size: a CU has to hold 8 of these waves
template <int NSEG, int W, bool STATS>
__global__ __launch_bounds__(W * kWave) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_gqa_mfma_bf16_kernel(const AttnParams p, const int head_splits) {
  constexpr int NT = gqa_stage_tiles(W);
  constexpr int kStageBytes = NT * kKvTileBytes;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5;
  const int col = lane & 31;

  // linear id -> (key split, batch * KV head, head split); the two head splits of a pair sit 8 ids
  // apart (same XCD under round-robin dispatch)
  const int lid = blockIdx.x;
  int pair = lid, hs = 0;
  if (head_splits == 2) {
    if ((gridDim.x & 15) == 0) {
      hs = (lid >> 3) & 1;
      pair = ((lid >> 4) << 3) | (lid & 7);
    } else {
      // any other grid: neighbours in the XCD-contiguous numbering (dealt ids 8 apart, same XCD)
      const int cid = xcd_contiguous_id(lid, gridDim.x);
      hs = cid & 1;
      pair = cid >> 1;
    }
  }
  const int split = pair % p.n_split;
  const int bg = pair / p.n_split;
  const int b = bg / p.hkv;
  const int g = bg - b * p.hkv;
  // a wave past the end of the group (odd G) takes part in staging and barriers only
  const int hg = hs * W + wave;
  const bool head_valid = hg < p.group;
  const int h = g * p.group + (head_valid ? hg : p.group - 1);
  const int head = b * p.hq + h;

  const SegPtrs sp = seg_ptrs(p, b, g, NSEG == 2);
  const int ntiles = sp.tiles0 + (sp.n1 + kTileKeys - 1) / kTileKeys;
  const int t_begin = split * p.tiles_per_split;
  const int t_end = min(ntiles, t_begin + p.tiles_per_split);
  const int nt = t_end - t_begin;            // >= 1: the planner leaves no split empty
  const int nstages = (nt + NT - 1) / NT;

  // Visiting order (STATS; one key segment): tiles [x0, x0 + n_mixed) hold keys that are not
  // candidates and are visited last, positions [n_pure, ntiles) of the order.
  int x0 = 0, n_mixed = 0;
  if (STATS) {
    x0 = p.cand0_end / kTileKeys;
    n_mixed = max(min(ntiles, (p.cand1_begin + kTileKeys - 1) / kTileKeys) - x0, 0);
  }
  const int n_pure = ntiles - n_mixed;
  auto tile_of = [&](int t) { return !STATS || t < x0 ? t : (t < n_pure ? t + n_mixed : x0 + (t - n_pure)); };

  bf16x8 qf[8];
  load_q_frags((const char*)p.q + 2 * (b * p.q_sb + h * p.q_sh + col * p.q_sr), half, qf);

  f32x16 acc[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[e][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  float mc_run = -INFINITY, lc_run = 0.f;   // the same over candidate keys only (STATS)

  // valid keys of local tile j (only the last tile of a segment is ragged)
  auto rows_of = [&](int j) {
    const int t = tile_of(t_begin + j);
    return t < sp.tiles0 ? min(kTileKeys, sp.n0 - t * kTileKeys) : min(kTileKeys, sp.n1 - (t - sp.tiles0) * kTileKeys);
  };
  // LDS address of local tile j: stage j / NT (double-buffered), slot j % NT
  auto tile_lds = [&](int j) { return smem + ((j / NT) & 1) * kStageBytes + (j % NT) * kKvTileBytes; };

  u32x4 kreg[NT * gqa_chunks(W)], vreg[NT * gqa_chunks(W)];
  gqa_load_stage<W, STATS>(sp, t_begin, t_end, tid, tile_of, kreg, vreg);
  gqa_store_stage<W>(smem, tid, kreg, vreg);
  if (nstages > 1) gqa_load_stage<W, STATS>(sp, t_begin + NT, t_end, tid, tile_of, kreg, vreg);
  __syncthreads();

  // Pipeline state between iterations: pb = softmax numerators of the current tile j (bf16), f = its V
  // fragments, a = the K fragments of tile j+1.  After the MFMA block of iteration j the wave requests
  // V of tile j+1 and K of tile j+2.  When tile j+2 opens a new stage k, that stage is published first
  // (registers -> LDS, workgroup barrier): the V request just made was this wave's last read of stage
  // k-1, and the buffer being overwritten held stage k-2, whose last read every wave had requested
  // before the previous publication's barrier.
  bf16x8 a[8], pb[2];
  PvFrags f;
  f32x16 sn;

  auto after_mfma = [&](int j) {   // j = current tile (-1 in the prologue)
    if (head_valid) tile_pv_load(tile_lds(j + 1) + kTileBytes, lane, f);
    if (j + 2 < nt && (j + 2) % NT == 0) {
      const int s_new = (j + 2) / NT;
      gqa_store_stage<W>(smem + (s_new & 1) * kStageBytes, tid, kreg, vreg);
      __syncthreads();
      if (s_new + 1 < nstages) gqa_load_stage<W, STATS>(sp, t_begin + (s_new + 1) * NT, t_end, tid, tile_of, kreg, vreg);
    }
    if (!head_valid) return;
    if (j + 2 < nt) tile_k_load(tile_lds(j + 2), half, col, a);
    __builtin_amdgcn_sched_barrier(0);
    if (STATS) {
      const int pos = t_begin + j + 1;   // of tile j+1 in the visiting order
      if (pos >= n_pure) {
        // first tile with other keys: what the attention has accumulated so far covers candidates only
        if (pos == max(n_pure, t_begin)) { mc_run = m_run; lc_run = l_run; }
        tile_candidate_stats(sn, tile_of(pos) * kTileKeys + half * 4, p, mc_run, lc_run);
      }
    }
    softmax_block(sn, rows_of(j + 1), p.scale_log2, half, m_run, l_run, acc, pb);
  };

  // a wave past the end of the group (odd G) only stages and synchronises
  if (head_valid) {
    tile_k_load(smem, half, col, a);
    __builtin_amdgcn_sched_barrier(0);
    tile_logits_mma(a, qf, sn);
    __builtin_amdgcn_sched_barrier(0);
  }
  after_mfma(-1);

  for (int j = 0; j + 1 < nt; ++j) {
    if (head_valid) {
      __builtin_amdgcn_sched_barrier(0);
      mfma_block(a, qf, sn, f, pb, acc);
      __builtin_amdgcn_sched_barrier(0);
    }
    after_mfma(j);
  }
  if (!head_valid) return;
  // PV product of the last tile
  __builtin_amdgcn_sched_barrier(0);
  pv_block(f, pb, acc);

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const size_t slot = (size_t)head * p.n_split + split;
  if (STATS) {
    if (t_end <= n_pure) { mc_run = m_run; lc_run = l_run; }   // this split saw candidates only
    const float lc_tot = lc_run + __shfl_xor(lc_run, 32);
    if (lane < 32) {
      p.cand_ml[slot * 64 + lane] = mc_run;
      p.cand_ml[slot * 64 + 32 + lane] = lc_tot;
    }
  }
  write_wave_result(acc, m_run, l_tot, lane, half, p.n_split == 1,
                    (char*)p.out + 2 * (b * p.o_sb + h * p.o_sh + col * p.o_sr), p.part_o + (slot * 32 + col) * 128,
                    p.part_ml + slot * 64);
}

template <int NSEG, int W, bool STATS>
static hipError_t launch_w(const AttnParams& p, int head_splits, hipStream_t s) {
  static LdsOptIn lds;
  const hipError_t e = lds.ensure(reinterpret_cast<const void*>(attn_gqa_mfma_bf16_kernel<NSEG, W, STATS>), (int)gqa_lds_bytes(W));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_gqa_mfma_bf16_kernel<NSEG, W, STATS>), dim3(p.n_split * p.batch * p.hkv * head_splits), dim3(W * kWave),
                     gqa_lds_bytes(W), s, p, head_splits);
  return hipGetLastError();
}

template <int NSEG, bool STATS>
static hipError_t launch_nseg(const AttnParams& p, hipStream_t s) {
  const int hs = gqa_head_splits(p.group);
  switch ((p.group + hs - 1) / hs) {   // waves per workgroup
    case 2: return launch_w<NSEG, 2, STATS>(p, hs, s);
    case 4: return launch_w<NSEG, 4, STATS>(p, hs, s);
    default: return hipErrorInvalidValue;
  }
}

// Workgroups of two or four waves.  The three-wave shapes (G = 3, 5, 6: uneven staging pieces, one
// tile per LDS stage) lost to the one-workgroup-per-head kernel at every size measured (G = 3, batch
// 32, 2208 keys: 137 against 85 us) and are not instantiated.
bool attn_gqa_supports_group(int group) { return group == 2 || group == 4 || group == 7 || group == 8; }

int attn_gqa_waves_per_wg(int group) {
  const int hs = gqa_head_splits(group);
  return (group + hs - 1) / hs;
}

hipError_t launch_attn_gqa_mfma_bf16(const AttnParams& p, hipStream_t s) {
  if (p.seg[0].n > 0 && p.seg[1].n > 0) return launch_nseg<2, false>(p, s);
  if (p.seg[1].n > 0) {   // empty cache: the block is the only key tensor
    AttnParams q = p;
    q.seg[0] = p.seg[1];
    q.seg[1].n = 0;
    return launch_nseg<1, false>(q, s);
  }
  return p.cand_ml ? launch_nseg<1, true>(p, s) : launch_nseg<1, false>(p, s);
}

}  // namespace sdllm
