// Block-query attention over Concat(cache, block) for bf16, head_dim 128, 32 query rows
// (Alg. 3 of the paper, cache_state == 2; the same kernel run over the full sequence is the
// dense block-row attention of cache states 0 and 1).
//
// Design for gfx950.  The 32 query rows of one head make exactly one 32x32 MFMA block, so a
// wavefront owns whole 32-key tiles: logits^T = K_tile * Q^T (K rows as the A operand, so each
// lane ends up holding 16 logits of ONE query row and the softmax row reduction stays in
// registers), then O^T += V_tile^T * P^T.  With 32 queries per 8 KB of K the kernel is bound by
// HBM (about 31 flop/byte), so the structure is chosen for bytes in flight, not for MFMA rate:
//   * each wave streams its own tiles; there is no workgroup barrier in the main loop;
//   * global loads are full-row coalesced (16 lanes x 16 B per 256-byte row), held in registers
//     for one tile of look-ahead, then written to a wave-private, row-padded LDS tile from
//     which the MFMA operand fragments are read without bank conflicts;
//   * the V^T operands come straight out of the row-major V tile through the transposing LDS read
//     (ds_read_b64_tr_b16), four MFMAs covering the 128 columns (MFMA e produces columns 32e + m);
//   * up to 8 waves per workgroup (the planner picks 4 or 5 for unsplit MHA heads) split the keys of
//     one head and merge their running (max, sum, numerator) through LDS; more workgroups per head
//     (split-KV) write fp32 partials that a small combine kernel merges.
#include <type_traits>

#include "attn_tile_math.h"

namespace sdllm {

constexpr int kWaveLds = kTileBytes + kVTileBytes + 512;    // K tile, V tile (later: 64 lanes x 272 B of accumulators), (max, sum)

size_t attn_mfma_lds_bytes(int waves) { return (size_t)waves * kWaveLds; }

// NSEG = 2: keys are Concat(cache, block) (sparse step); NSEG = 1: one key tensor (dense step, or a
// sparse step with an empty cache).  The two instantiations also show up as separate kernels in a
// profile, which keeps sparse and dense launches apart.
// STATS (dense launches of the cache-update step only): also accumulate each query row's (max, sum)
// over the candidate keys, so the scoring pass that follows need not stream K for them again.
// DEEP: prefetch K and V of the next tile together (one memory latency per tile instead of two, twice
// the bytes in flight).  Chosen for small grids, which are latency-bound; large grids saturate HBM and
// run faster with the shallower alternating scheme.
// SHARED_KV: the G query heads of a KV group run as separate workgroups (grouped-query attention on
// a small grid); their K/V reads are then plain loads so that the siblings hit in L2.  K is also read
// with plain loads by the statistics launches: the scoring that follows (the column sweep at the end of
// this kernel, or the scoring kernel) reads the same rows again and finds part of them in L2 and the
// memory-side cache (B=8 LLaDA shape, cache-update step: 234 -> 226 us).
template <int NSEG, bool STATS, bool DEEP, bool SHARED_KV>
__global__ __launch_bounds__(512) void attn_mfma_bf16_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6;
  const int half = lane >> 5;
  const int col = lane & 31;

  // Consecutive workgroup ids go round-robin over the 8 XCDs; renumber so that the workgroups of
  // one KV group (its query heads and key splits) sit on one XCD and share that XCD's L2.
  const int wg = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int split = wg % p.n_split;
  const int head = wg / p.n_split;
  const int b = head / p.hq;
  const int h = head - b * p.hq;
  const int g = h / p.group;

  const SegPtrs sp = seg_ptrs(p, b, g, NSEG == 2);
  const int ntiles = sp.tiles0 + (sp.n1 + kTileKeys - 1) / kTileKeys;
  const int t_begin = split * p.tiles_per_split;
  const int t_end = min(ntiles, t_begin + p.tiles_per_split);

  // Q^T fragments (B operand): lane (col = query row, half) holds head-dim [16t + 8 half, +8)
  bf16x8 qf[8];
  load_q_frags((const char*)p.q + 2 * (b * p.q_sb + h * p.q_sh + col * p.q_sr), half, qf);

  uint8_t* lds_k = smem + wave * kWaveLds;
  uint8_t* lds_v = lds_k + kTileBytes;

  f32x16 acc[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[e][i] = 0.f;
  float m_run = -INFINITY;   // softmax reference of the row (log2 domain, within 8 of the running max), same in both halves
  float l_run = 0.f;         // running row sum over the keys this half-lane has seen
  float mc_run = -INFINITY, lc_run = 0.f;   // the same over candidate keys only (STATS)

  // Shallow scheme: one staging register set, used alternately for the K and the V tile, so a wave
  // keeps exactly one 8 KB tensor tile in flight (40-64 KB per CU with 5-8 waves).  Measured on MI355X, a
  // streaming read is fastest with 32-64 KB outstanding per CU and loses ~5 % at 128 KB, so K(t+1)
  // flies under the PV product of tile t and V(t) under its logits/softmax.
  u32x4 reg[8], reg2[DEEP ? 8 : 1];
  int t = t_begin + wave;
  uint32_t stride = 0;
  TileSrc ts{};
  if (t < t_end) {
    ts = tile_src(sp, t, stride);
    load_rows<!(SHARED_KV || STATS)>(ts.k, ts.rows, stride, lane, reg);
    if (DEEP) load_rows<!SHARED_KV>(ts.v, ts.rows, stride, lane, reinterpret_cast<u32x4(&)[8]>(reg2));
  }

  for (; t < t_end; t += nw) {
    const int rows = ts.rows;
    const int tn = t + nw;
    store_rows(lds_k, lane, reg);
    if (DEEP) {
      store_rows_v(lds_v, lane, reinterpret_cast<u32x4(&)[8]>(reg2));
      wave_lds_sync();
      if (tn < t_end) {                              // both tensors of tile t+1 fly during tile t
        ts = tile_src(sp, tn, stride);
        load_rows<!(SHARED_KV || STATS)>(ts.k, ts.rows, stride, lane, reg);
        load_rows<!SHARED_KV>(ts.v, ts.rows, stride, lane, reinterpret_cast<u32x4(&)[8]>(reg2));
      }
    } else {
      wave_lds_sync();
      load_rows<!SHARED_KV>(ts.v, ts.rows, stride, lane, reg);   // V(t) flies during the logits and the softmax
    }

    // logits^T[key, query] = K_tile Q^T (raw), row max in the scaled log2 domain
    f32x16 s;
    const float m_loc = tile_logits(lds_k, qf, rows, p.scale_log2, half, col, s);
    const int key0 = half * 4;
    if (STATS) {
      // single segment: register i is absolute position 32 t + key; the block's own keys (and, for
      // prefix-only eviction, the suffix) are not candidates
      const int pos0 = t * kTileKeys + key0;
      float sc[16];
      float mc_loc = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int pos = pos0 + (i >> 2) * 8 + (i & 3);
        sc[i] = (pos < p.cand0_end || pos >= p.cand1_begin) ? s[i] * p.scale_log2 : -INFINITY;
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
    tile_softmax(s, m_loc, p.scale_log2, m_run, l_run, acc);

    if (!DEEP) {
      store_rows_v(lds_v, lane, reg);
      wave_lds_sync();
      if (tn < t_end) {                              // K(t+1) flies during the PV product
        ts = tile_src(sp, tn, stride);
        load_rows<!(SHARED_KV || STATS)>(ts.k, ts.rows, stride, lane, reg);
      }
    }

    tile_pv(lds_v, s, lane, acc);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  float l_tot = l_run + __shfl_xor(l_run, 32);
  const float lc_tot = lc_run + __shfl_xor(lc_run, 32);
  const size_t slot = (size_t)head * p.n_split + split;

  if (nw == 1) {
    // a single wave owns the whole result: straight from registers
    if (STATS && lane < 32) {
      p.cand_ml[slot * 64 + lane] = mc_run;
      p.cand_ml[slot * 64 + 32 + lane] = lc_tot;
    }
    write_wave_result(acc, m_run, l_tot, lane, half, p.n_split == 1,
                      (char*)p.out + 2 * (b * p.o_sb + h * p.o_sh + col * p.o_sr), p.part_o + (slot * 32 + col) * 128,
                      p.part_ml + slot * 64);
    return;
  }

  // Merge the waves of the workgroup, all waves working: every wave parks its 64 accumulator
  // registers per lane in its own LDS region ([lane][e][i], lane stride 272 B) together with its
  // row (max, sum); after one barrier wave w reduces the 4-register slots w, w+nw, ... (of 16) over all waves.
  // All LDS reads of a slot are issued before any is used, so the merge costs a few hundred cycles.
  {
    uint8_t* mine = smem + wave * kWaveLds;
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 v = {acc[e][i4 * 4], acc[e][i4 * 4 + 1], acc[e][i4 * 4 + 2], acc[e][i4 * 4 + 3]};
        *reinterpret_cast<f32x4*>(mine + lane * kRowBytes + (e * 4 + i4) * 16) = v;
      }
    float* my_ml = reinterpret_cast<float*>(mine + 64 * kRowBytes);
    if (lane < 32) {
      my_ml[lane] = m_run; my_ml[32 + lane] = l_tot;
      if (STATS) { my_ml[64 + lane] = mc_run; my_ml[96 + lane] = lc_tot; }
    }
  }
  __syncthreads();
  if (STATS && wave == 0 && lane < 32) {
    float mc = -INFINITY, lc = 0.f;
    for (int w = 0; w < nw; ++w)
      mc = fmaxf(mc, reinterpret_cast<const float*>(smem + w * kWaveLds + 64 * kRowBytes)[64 + lane]);
    for (int w = 0; w < nw; ++w) {
      const float* ml = reinterpret_cast<const float*>(smem + w * kWaveLds + 64 * kRowBytes);
      if (ml[64 + lane] != -INFINITY) lc += ml[96 + lane] * __builtin_amdgcn_exp2f(ml[64 + lane] - mc);
    }
    p.cand_ml[slot * 64 + lane] = mc;
    p.cand_ml[slot * 64 + 32 + lane] = lc;
    if (p.score_out) {   // merged statistics for the column sweep below, in wave 0's own slots
      float* st = reinterpret_cast<float*>(smem + 64 * kRowBytes) + 64;
      st[lane] = mc;
      st[32 + lane] = 1.f / lc;
    }
  }
  // With the wave count a compile-time constant every LDS read of the merge (the waves' (max, sum) and the
  // up to ceil(16 / NW) slots this wave reduces) is requested before the first is used: one LDS round trip
  // instead of one per slot.
  auto merge = [&](auto nw_tag) {
    constexpr int NW = decltype(nw_tag)::value;
    constexpr int NJ = (16 + NW - 1) / NW;
    float m_w[NW], l_w[NW], f_w[NW];
    f32x4 part[NJ][NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float* ml = reinterpret_cast<const float*>(smem + w * kWaveLds + 64 * kRowBytes);
      m_w[w] = ml[col];
      l_w[w] = ml[32 + col];
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int i = min(wave + j * NW, 15);   // past the last slot (some waves, last round): re-read slot 15, not stored
#pragma unroll
      for (int w = 0; w < NW; ++w)
        part[j][w] = *reinterpret_cast<const f32x4*>(smem + w * kWaveLds + lane * kRowBytes + i * 16);
    }
    __builtin_amdgcn_sched_barrier(0);
    float m_tot = -INFINITY, l_all = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) m_tot = fmaxf(m_tot, m_w[w]);
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      // a wave that saw no tile parked (-inf, 0, 0): factor 0
      f_w[w] = m_w[w] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_w[w] - m_tot);
      l_all += f_w[w] * l_w[w];
    }
    const float inv = 1.f / l_all;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int i = wave + j * NW;
      if (i < 16) {
        f32x4 o4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) o4 += part[j][w] * f_w[w];
        const int d0 = out_col0(i >> 2, i & 3, half);   // slot i = (e, i4): four consecutive output columns
        if (p.n_split == 1) {
          bf16x4 ob;
#pragma unroll
          for (int r = 0; r < 4; ++r) ob[r] = (__bf16)(o4[r] * inv);
          char* op = (char*)p.out + 2 * (b * p.o_sb + h * p.o_sh + col * p.o_sr);
          *reinterpret_cast<bf16x4*>(op + d0 * 2) = ob;
        } else {
          *reinterpret_cast<f32x4*>(p.part_o + (slot * 32 + col) * 128 + d0) = o4;
        }
      }
    }
    if (p.n_split > 1 && wave == 0 && lane < 32) {
      p.part_ml[slot * 64 + lane] = m_tot;
      p.part_ml[slot * 64 + 32 + lane] = l_all;
    }
  };
  switch (nw) {
    case 2: merge(std::integral_constant<int, 2>{}); break;
    case 3: merge(std::integral_constant<int, 3>{}); break;
    case 4: merge(std::integral_constant<int, 4>{}); break;
    case 5: merge(std::integral_constant<int, 5>{}); break;
    case 6: merge(std::integral_constant<int, 6>{}); break;
    case 7: merge(std::integral_constant<int, 7>{}); break;
    default: merge(std::integral_constant<int, 8>{}); break;
  }

  // Column sweep (cache-update step, MHA, no key splits): with the row statistics of the scoring softmax
  // final, the workgroup walks its head's keys once more, LAST TILE FIRST (the most recently read K rows
  // are the ones the memory-side cache may still hold), and leaves each candidate key's softmax-mean
  // saliency score (Alg. 1 steps 5-6).  Same fragments as the attention, operands swapped: Q rows as the A
  // operand, so a lane holds ONE key (lane % 32) against 16 query rows (8*(i/4) + 4*half + i%4).
  if (STATS && p.score_out) {
    __syncthreads();   // statistics visible; every wave is done with the parked accumulators
    const float* st = reinterpret_cast<const float*>(smem + 64 * kRowBytes) + 64;
    float row_m[16], row_il[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = (i >> 2) * 8 + half * 4 + (i & 3);
      row_m[i] = st[row];
      row_il[i] = st[32 + row];
    }
    float* score_row = p.score_out + (size_t)(b * p.hkv + g) * p.score_stride;
    const int gap = p.cand1_begin - p.cand0_end;
    int tc = ntiles - 1 - wave;
    if (tc >= 0) {
      ts = tile_src(sp, tc, stride);
      load_rows<true>(ts.k, ts.rows, stride, lane, reg);
    }
    for (; tc >= 0; tc -= nw) {
      const int rows = ts.rows;
      store_rows(lds_k, lane, reg);
      wave_lds_sync();
      if (tc - nw >= 0) {
        ts = tile_src(sp, tc - nw, stride);
        load_rows<true>(ts.k, ts.rows, stride, lane, reg);
      }
      bf16x8 a[8];
      tile_k_load(lds_k, half, col, a);
      __builtin_amdgcn_sched_barrier(0);
      f32x16 sc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sc[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[kk], a[kk], sc, 0, 0, 0);
      float total = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) total += __builtin_amdgcn_exp2f(__builtin_fmaf(sc[i], p.scale_log2, -row_m[i])) * row_il[i];
      total += __shfl_xor(total, 32);
      const int pos = tc * kTileKeys + col;
      const bool cand = pos < p.cand0_end || pos >= p.cand1_begin;
      if (half == 0 && col < rows && cand) score_row[pos < p.cand0_end ? pos : pos - gap] = total * p.score_inv_count;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

template <int NSEG, bool STATS, bool DEEP, bool SHARED_KV>
static hipError_t launch_variant(const AttnParams& p, hipStream_t s) {
  const int nwg = p.batch * p.hq * p.n_split;
  static LdsOptIn lds;
  const hipError_t e = lds.ensure(reinterpret_cast<const void*>(attn_mfma_bf16_kernel<NSEG, STATS, DEEP, SHARED_KV>),
                                  (int)attn_mfma_lds_bytes(kMaxWavesPerWg));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_mfma_bf16_kernel<NSEG, STATS, DEEP, SHARED_KV>), dim3(nwg), dim3(p.waves * kWave),
                     attn_mfma_lds_bytes(p.waves), s, p);
  return hipGetLastError();
}

template <int NSEG, bool STATS>
static hipError_t launch_nseg(const AttnParams& p, hipStream_t s) {
  // at most half the CUs busy: latency-bound, take the deep prefetch
  const bool deep = p.batch * p.hq * p.n_split <= kNumCUs / 2;
  if (p.group > 1) return deep ? launch_variant<NSEG, STATS, true, true>(p, s) : launch_variant<NSEG, STATS, false, true>(p, s);
  return deep ? launch_variant<NSEG, STATS, true, false>(p, s) : launch_variant<NSEG, STATS, false, false>(p, s);
}

hipError_t launch_attn_mfma_bf16(const AttnParams& p, hipStream_t s) {
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
