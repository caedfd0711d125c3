// Saliency scoring on the matrix cores for bf16, head_dim 128, 32 query rows (Sec. 3.3 second
// equation, aggregated over the block's queries and the query heads of a KV group as in Alg. 1).
//
// The softmax-normalised score needs each query row's max and sum over ALL candidates before any
// column can be reduced, so it takes two streaming passes over K (the logits are recomputed; they
// are cheap next to the K read):
//   pass 1 (row_stats): logits^T = K_tile Q_h^T, lane = query row, online (max, sum) per row;
//   pass 2 (col_reduce): logits = Q_h K_tile^T, lane = candidate key, p = exp2(s - max)/sum summed
//                        over the 32 rows (in registers) and over the G query heads of the group.
// A workgroup serves one (batch, KV head) and a contiguous range of candidate tiles; its waves take
// tiles round-robin into wave-private LDS tiles (no barrier in the loop) and the Q fragments of all G
// heads sit in LDS once per workgroup, so K is read from HBM once per pass however large G is.
// Probabilities stay fp32 end to end: the retained set must match a float64 reference except for
// scores within 1e-4 relative of the k-th value.
#include "mfma_tile.h"

namespace sdllm {

struct CandTiles {
  const char* k0; const char* k1;   // first row of the prefix / suffix candidates of this (b, g)
  uint32_t stride;                  // bytes per key row
  int n0, n1, tiles0;
};

__device__ __forceinline__ CandTiles cand_tiles(const ScoreParams& p, int b, int g) {
  CandTiles ct;
  ct.stride = (uint32_t)(p.k_sr * 2);
  const char* base = (const char*)p.k + 2 * (b * p.k_sb + g * p.k_sh);
  ct.k0 = base;
  ct.k1 = base + (size_t)(p.block_off + p.block_len) * ct.stride;
  ct.n0 = min(p.n_cand, p.block_off);
  ct.n1 = p.n_cand - ct.n0;
  ct.tiles0 = (ct.n0 + kTileKeys - 1) / kTileKeys;
  return ct;
}

// tile -> (first row pointer, valid rows, candidate index of its first row)
__device__ __forceinline__ const char* tile_rows(const CandTiles& ct, int tile, int& rows, int& cand0) {
  if (tile < ct.tiles0) {
    cand0 = tile * kTileKeys;
    rows = min(kTileKeys, ct.n0 - cand0);
    return ct.k0 + (size_t)cand0 * ct.stride;
  }
  const int first = (tile - ct.tiles0) * kTileKeys;
  cand0 = ct.n0 + first;
  rows = min(kTileKeys, ct.n1 - first);
  return ct.k1 + (size_t)first * ct.stride;
}

// Q rows of all G heads of the group -> LDS, padded like a K tile so both are read the same way.
template <int G>
__device__ __forceinline__ void stage_queries(const ScoreParams& p, int b, int g, uint8_t* lds_q) {
  for (int i = threadIdx.x; i < G * 32 * 16; i += blockDim.x) {
    const int chunk = i & 15, row = (i >> 4) & 31, hh = i >> 9;
    const char* src = (const char*)p.q + 2 * (b * p.q_sb + (int64_t)(g * G + hh) * p.q_sh + row * p.q_sr) + chunk * 16;
    *reinterpret_cast<u32x4*>(lds_q + hh * kTileBytes + tile_off(row, chunk)) = *reinterpret_cast<const u32x4*>(src);
  }
}

// The column reduction over this workgroup's tiles (pass 2): lds_q holds the group's Q rows, lds_ml the
// final (max, 1/sum) of every (head, row).
template <int G, bool BACKWARDS>
__device__ __forceinline__ void score_columns(const ScoreParams& p, int b, int g, int bg, int part, const uint8_t* lds_q,
                                              uint8_t* lds_k, const float2* lds_ml, int wave, int nw, int lane, int half,
                                              int col) {
  const CandTiles ct = cand_tiles(p, b, g);
  const int ntiles = ct.tiles0 + (ct.n1 + kTileKeys - 1) / kTileKeys;
  const int t_begin = part * p.tiles_per_part;
  const int t_end = min(ntiles, t_begin + p.tiles_per_part);
  const float inv_count = 1.f / (float)(G * 32);
  float* score_row = p.score + (size_t)bg * p.score_stride;

  u32x4 kreg[8];
  int rows = 0, cand0 = 0;
  // BACKWARDS (the sweep that follows the statistics pass inside one launch): last tile first, because
  // the rows that pass read last are the ones this XCD's L2 may still hold
  const int n_mine = t_end - t_begin;
  auto tile_at = [&](int i) { return BACKWARDS ? t_end - 1 - i : t_begin + i; };   // i-th tile of this workgroup's walk
  int i_t = wave;
  if (i_t < n_mine) {
    const char* src = tile_rows(ct, tile_at(i_t), rows, cand0);
    load_rows(src, rows, ct.stride, lane, kreg);
  }
  for (; i_t < n_mine; i_t += nw) {
    store_rows(lds_k, lane, kreg);
    wave_lds_sync();
    const int rows_now = rows, cand_now = cand0;
    if (i_t + nw < n_mine) {
      const char* src = tile_rows(ct, tile_at(i_t + nw), rows, cand0);
      load_rows(src, rows, ct.stride, lane, kreg);
    }
    bf16x8 kf[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kf[kk] = *reinterpret_cast<const bf16x8*>(lds_k + tile_off(col, kk * 2 + half));
    float total = 0.f;
    if (G > 1 && p.softmax) {
      // Software pipeline over the heads: while the vector ALU turns head hh's logits into
      // probabilities, the matrix core works on head hh+1 and the LDS returns the Q fragments of
      // head hh+2.  A wave issues in order, so the three streams are interleaved in program order
      // (one MFMA, its share of LDS reads and of ALU work, eight times per head); a modest gain,
      // 20.5 -> 19.4 us with seven heads per group at batch 8.
      bf16x8 qf[2][8];
      f32x16 sn[2];
      auto q_frag = [&](int hh, int kk) {
        return *reinterpret_cast<const bf16x8*>(lds_q + hh * kTileBytes + tile_off(col, kk * 2 + half));
      };
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) qf[0][kk] = q_frag(0, kk);
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) qf[1][kk] = q_frag(1, kk);
#pragma unroll
      for (int i = 0; i < 16; ++i) sn[0][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) sn[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[0][kk], kf[kk], sn[0], 0, 0, 0);
      // row statistics of register i of head hh: query row 8*(i/4) + 4*half + i%4 (this lane's key is `col`)
      auto row_ml = [&](int hh, int i) { return lds_ml[hh * 32 + (i >> 2) * 8 + half * 4 + (i & 3)]; };
      float2 ml[2] = {row_ml(0, 0), row_ml(0, 1)};
#pragma unroll
      for (int hh = 0; hh < G; ++hh) {
        const int cur = hh & 1, nxt = cur ^ 1;
        if (hh + 1 < G) {
#pragma unroll
          for (int i = 0; i < 16; ++i) sn[nxt][i] = 0.f;
        }
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          if (hh + 1 < G) sn[nxt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[nxt][kk], kf[kk], sn[nxt], 0, 0, 0);
          if (hh + 2 < G) qf[cur][kk] = q_frag(hh + 2, kk);
          // the statistics are requested one group ahead of their use
          float2 ml_next[2] = {ml[0], ml[1]};
          if (kk < 7) { ml_next[0] = row_ml(hh, 2 * kk + 2); ml_next[1] = row_ml(hh, 2 * kk + 3); }
          else if (hh + 1 < G) { ml_next[0] = row_ml(hh + 1, 0); ml_next[1] = row_ml(hh + 1, 1); }
          total += __builtin_amdgcn_exp2f(sn[cur][2 * kk] * p.scale_log2 - ml[0].x) * ml[0].y;
          total += __builtin_amdgcn_exp2f(sn[cur][2 * kk + 1] * p.scale_log2 - ml[1].x) * ml[1].y;
          ml[0] = ml_next[0]; ml[1] = ml_next[1];
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);   // 3 LDS reads
          __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);   // 6 vector ALU
        }
      }
    } else {
#pragma unroll
      for (int hh = 0; hh < G; ++hh) {
        f32x16 s;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          const bf16x8 qf = *reinterpret_cast<const bf16x8*>(lds_q + hh * kTileBytes + tile_off(col, kk * 2 + half));
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[kk], s, 0, 0, 0);   // rows = queries, columns = keys
        }
        // register i is query row 8*(i/4) + 4*half + i%4, this lane's key is `col`
        float part_sum = 0.f;
        if (p.softmax) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float2 ml = lds_ml[hh * 32 + (i >> 2) * 8 + half * 4 + (i & 3)];
            part_sum += __builtin_amdgcn_exp2f(s[i] * p.scale_log2 - ml.x) * ml.y;
          }
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i) part_sum += s[i];
          part_sum *= p.scale;
        }
        total += part_sum;
      }
    }
    total += __shfl_xor(total, 32);
    if (half == 0 && col < rows_now) score_row[cand_now + col] = total * inv_count;
    wave_lds_sync();
  }
}

// ------------------------------------------------------------------ pass 1: row statistics
template <int G>
__global__ __launch_bounds__(512) void score_stats_mfma_kernel(const ScoreParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int part = blockIdx.x;
  const int bg = blockIdx.y;
  const int b = bg / p.hkv, g = bg - b * p.hkv;

  uint8_t* lds_q = smem;
  uint8_t* lds_k = smem + G * kTileBytes + wave * kTileBytes;
  float2* lds_ml = reinterpret_cast<float2*>(smem + (G + nw) * kTileBytes);
  stage_queries<G>(p, b, g, lds_q);
  __syncthreads();

  const CandTiles ct = cand_tiles(p, b, g);
  const int ntiles = ct.tiles0 + (ct.n1 + kTileKeys - 1) / kTileKeys;
  const int t_begin = part * p.tiles_per_part;
  const int t_end = min(ntiles, t_begin + p.tiles_per_part);

  float m_run[G], l_run[G];
#pragma unroll
  for (int hh = 0; hh < G; ++hh) { m_run[hh] = -INFINITY; l_run[hh] = 0.f; }

  u32x4 kreg[8];
  int rows = 0, cand0 = 0;
  int t = t_begin + wave;
  if (t < t_end) {
    const char* src = tile_rows(ct, t, rows, cand0);
    load_rows<false>(src, rows, ct.stride, lane, kreg);   // plain: the column pass reads these rows again
  }
  for (; t < t_end; t += nw) {
    store_rows(lds_k, lane, kreg);
    wave_lds_sync();
    const int rows_now = rows;
    const int tn = t + nw;
    if (tn < t_end) {
      const char* src = tile_rows(ct, tn, rows, cand0);
      load_rows<false>(src, rows, ct.stride, lane, kreg);   // plain: the column pass reads these rows again
    }
    bf16x8 kf[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kf[kk] = *reinterpret_cast<const bf16x8*>(lds_k + tile_off(col, kk * 2 + half));
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
      f32x16 s;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const bf16x8 qf = *reinterpret_cast<const bf16x8*>(lds_q + hh * kTileBytes + tile_off(col, kk * 2 + half));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf, s, 0, 0, 0);   // rows = keys, columns = queries
      }
      // each half-lane keeps the (max, sum) of the keys it has seen itself (the two halves of a row
      // are merged once, after the loop); the max is taken on the raw logits and the scale folded
      // into the exponent's multiply-add
      if (rows_now < kTileKeys) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if ((i >> 2) * 8 + half * 4 + (i & 3) >= rows_now) s[i] = -INFINITY;
      }
      float m_loc = s[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) m_loc = fmaxf(m_loc, s[i]);
      if (m_loc != -INFINITY) {   // a ragged tile can leave a half-lane without any key
        const float m_new = fmaxf(m_run[hh], m_loc * p.scale_log2);
        float l_loc = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) l_loc += __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], p.scale_log2, -m_new));
        l_run[hh] = l_run[hh] * __builtin_amdgcn_exp2f(m_run[hh] - m_new) + l_loc;
        m_run[hh] = m_new;
      }
    }
    wave_lds_sync();
  }

  // merge the waves: every wave parks (max, sum) per head and row in its own tile region
  float* mine = reinterpret_cast<float*>(lds_k);
#pragma unroll
  for (int hh = 0; hh < G; ++hh) {
    const float m_other = __shfl_xor(m_run[hh], 32), l_other = __shfl_xor(l_run[hh], 32);
    const float m_row = fmaxf(m_run[hh], m_other);
    float l_tot = 0.f;
    if (m_run[hh] != -INFINITY) l_tot += l_run[hh] * __builtin_amdgcn_exp2f(m_run[hh] - m_row);
    if (m_other != -INFINITY) l_tot += l_other * __builtin_amdgcn_exp2f(m_other - m_row);
    if (lane < 32) { mine[hh * 64 + lane] = m_row; mine[hh * 64 + 32 + lane] = l_tot; }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < G * 32; i += blockDim.x) {
    const int hh = i >> 5, row = i & 31;
    float m_tot = -INFINITY;
    for (int w = 0; w < nw; ++w)
      m_tot = fmaxf(m_tot, reinterpret_cast<const float*>(smem + (G + w) * kTileBytes)[hh * 64 + row]);
    float l_tot = 0.f;
    for (int w = 0; w < nw; ++w) {
      const float* o = reinterpret_cast<const float*>(smem + (G + w) * kTileBytes);
      const float m_w = o[hh * 64 + row];
      if (m_w != -INFINITY) l_tot += o[hh * 64 + 32 + row] * __builtin_amdgcn_exp2f(m_w - m_tot);
    }
    const size_t head = (size_t)b * p.hq + g * G + hh;
    float* dst = p.part_ml + (head * p.n_part + part) * 64;
    dst[row] = m_tot;
    dst[32 + row] = l_tot;
    if (p.cols_follow) lds_ml[i] = make_float2(m_tot, 1.f / l_tot);
  }
  // One workgroup per row: its statistics are final, and the column pass follows in the same launch
  // (no second launch with its fill and drain, and the walk back starts on rows still in L2).
  if (p.cols_follow) {
    __syncthreads();
    score_columns<G, true>(p, b, g, bg, part, lds_q, lds_k, lds_ml, wave, nw, lane, half, col);
  }
}

// ------------------------------------------------------------------ pass 2: column reduction
template <int G>
__global__ __launch_bounds__(512) void score_cols_mfma_kernel(const ScoreParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int part = blockIdx.x;
  const int bg = blockIdx.y;
  const int b = bg / p.hkv, g = bg - b * p.hkv;

  uint8_t* lds_q = smem;
  uint8_t* lds_k = smem + G * kTileBytes + wave * kTileBytes;
  // per (head, row): max (log2 domain) and 1/sum of the whole row, from the partials of pass 1
  float2* lds_ml = reinterpret_cast<float2*>(smem + (G + nw) * kTileBytes);
  stage_queries<G>(p, b, g, lds_q);
  if (p.softmax) {
    for (int i = threadIdx.x; i < G * 32; i += blockDim.x) {
      const int hh = i >> 5, row = i & 31;
      const size_t head = (size_t)b * p.hq + g * G + hh;
      const float* src = p.part_ml + head * p.n_stat_part * 64;
      // merge the partial (max, sum) pairs of pass 1 in one sweep (there can be dozens per row and
      // every load is a trip to L2: sixteen pairs are requested together, then folded in)
      float m_tot = -INFINITY, l_tot = 0.f;
#pragma unroll 16
      for (int s = 0; s < p.n_stat_part; ++s) {
        const float m_s = src[s * 64 + row];
        const float l_s = src[s * 64 + 32 + row];
        const float m_new = fmaxf(m_tot, m_s);
        if (m_new != -INFINITY)
          l_tot = l_tot * __builtin_amdgcn_exp2f(m_tot - m_new) + l_s * __builtin_amdgcn_exp2f(m_s - m_new);
        m_tot = m_new;
      }
      lds_ml[i] = make_float2(m_tot, 1.f / l_tot);
    }
  }
  __syncthreads();

  score_columns<G, false>(p, b, g, bg, part, lds_q, lds_k, lds_ml, wave, nw, lane, half, col);
}

static size_t score_lds_bytes(int group, int waves) { return (size_t)(group + waves) * kTileBytes + (size_t)group * 32 * 8; }

template <int G>
static hipError_t launch_g(const ScoreParams& p, hipStream_t s) {
  const size_t lds = score_lds_bytes(G, p.waves);
  static LdsOptIn lds_stats, lds_cols;
  const int max_lds = (int)score_lds_bytes(G, kMaxWavesPerWg);
  hipError_t e = lds_stats.ensure(reinterpret_cast<const void*>(score_stats_mfma_kernel<G>), max_lds);
  if (e != hipSuccess) return e;
  e = lds_cols.ensure(reinterpret_cast<const void*>(score_cols_mfma_kernel<G>), max_lds);
  if (e != hipSuccess) return e;
  const dim3 grid(p.n_part, p.batch * p.hkv), block(p.waves * kWave);
  if (p.softmax && !p.skip_stats) {
    ScoreParams q = p;
    q.cols_follow = p.n_part == 1;   // statistics final inside the workgroup: one launch does both passes
    hipLaunchKernelGGL(score_stats_mfma_kernel<G>, grid, block, lds, s, q);
    if (q.cols_follow) return hipGetLastError();
  }
  hipLaunchKernelGGL(score_cols_mfma_kernel<G>, grid, block, lds, s, p);
  return hipGetLastError();
}

bool score_mfma_supports_group(int group) { return group >= 1 && group <= 8; }

hipError_t launch_score_mfma_bf16(const ScoreParams& p, hipStream_t s) {
  if (p.n_cand <= 0) return hipSuccess;
  switch (p.group) {
    case 1: return launch_g<1>(p, s);
    case 2: return launch_g<2>(p, s);
    case 3: return launch_g<3>(p, s);
    case 4: return launch_g<4>(p, s);
    case 5: return launch_g<5>(p, s);
    case 6: return launch_g<6>(p, s);
    case 7: return launch_g<7>(p, s);
    case 8: return launch_g<8>(p, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sdllm
