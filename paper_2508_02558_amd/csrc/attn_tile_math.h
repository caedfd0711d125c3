// Per-tile arithmetic shared by the bf16 MFMA attention kernels: one wavefront, 32 query rows of
// one head, one 32-key tile of K and V in LDS (padded layout of mfma_tile.h).
//
// Fragment conventions (v_mfma_f32_32x32x16_bf16): lane = (col = lane % 32, half = lane / 32).
//   logits^T = K_tile Q^T: K rows are the A operand, Q^T the B operand; register i of a lane is key
//   8*(i/4) + 4*half + i%4 of the tile for query row `col`, so softmax row reductions are in-lane
//   plus one exchange between the two halves.
//   O^T += V_tile^T P^T: P^T (registers 8*step .. 8*step+7 of the logits, as bf16) is the B operand;
//   V^T fragments come from the row-major V tile through the transposing LDS read; MFMA e (0..3)
//   produces columns 32e + m, m = 8*(i/4) + 4*half + i%4.
#pragma once

#include "mfma_tile.h"

namespace sdllm {

// Q^T fragments of query row `col` (16-byte pieces of the row, straight from global memory).
__device__ __forceinline__ void load_q_frags(const char* q_row, int half, bf16x8 (&qf)[8]) {
  const u32x4* qp = reinterpret_cast<const u32x4*>(q_row);
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const u32x4 raw = qp[t * 2 + half];
    qf[t] = __builtin_bit_cast(bf16x8, raw);
  }
}

// The eight K fragments (A operands) of one tile, all requested together.
__device__ __forceinline__ void tile_k_load(const uint8_t* lds_k, int half, int col, bf16x8 (&a)[8]) {
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) a[kk] = *reinterpret_cast<const bf16x8*>(lds_k + tile_off(col, kk * 2 + half));
}

// logits^T = K_tile Q^T from fragments already in registers: raw, unscaled.
__device__ __forceinline__ void tile_logits_mma(const bf16x8 (&a)[8], const bf16x8 (&qf)[8], f32x16& s) {
#pragma unroll
  for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], qf[kk], s, 0, 0, 0);
}

// Keys >= rows become -inf; returns the max over the 16 keys THIS half-lane holds, in the scaled
// log2 domain (scale_log2 > 0).  The two halves of a row are only exchanged when tile_softmax finds
// that the reference has to move.
__device__ __forceinline__ float tile_mask_max(f32x16& s, int rows, float scale_log2, int half) {
  if (rows < kTileKeys) {   // only the last tile of a segment is ragged (wave-uniform)
    // the empty asm keeps this a real branch: if-converted, the 32 compare/select instructions
    // would run on every tile of kernels that are short of vector-ALU issue slots
    asm volatile("");
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = half * 4 + (i >> 2) * 8 + (i & 3);
      s[i] = key < rows ? s[i] : -INFINITY;
    }
  }
  float m_loc = s[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) m_loc = fmaxf(m_loc, s[i]);
  return m_loc * scale_log2;
}

// Raw logits of one tile (unscaled; keys >= rows become -inf).  Returns this half-lane's max over the
// tile in the scaled log2 domain.  All eight K fragments are requested before the first MFMA (the
// scheduling barrier keeps the compiler from sinking each read next to its use, which would expose
// the LDS latency eight times).
__device__ __forceinline__ float tile_logits(const uint8_t* lds_k, const bf16x8 (&qf)[8], int rows, float scale_log2,
                                             int half, int col, f32x16& s) {
  bf16x8 a[8];
  tile_k_load(lds_k, half, col, a);
  __builtin_amdgcn_sched_barrier(0);
  tile_logits_mma(a, qf, s);
  return tile_mask_max(s, rows, scale_log2, half);
}

// Softmax numerators of one tile against a per-row reference m_ref that only moves when some row's
// tile max exceeds it by more than kRescaleSlack (log2 units): s becomes exp2(scale*s - m_ref), which
// is then at most 2^kRescaleSlack instead of at most 1.  Any common reference gives the same
// quotient sum(p v)/sum(p); moving it rarely saves rescaling the 64 accumulator registers on almost
// every tile.  l_run only covers the keys this half-lane holds; the halves are added at the end.
constexpr float kRescaleSlack = 8.f;

__device__ __forceinline__ void tile_softmax(f32x16& s, float m_loc, float scale_log2, float& m_ref, float& l_run,
                                             f32x16 (&acc)[4]) {
  // m_loc is per half-lane; the vote is over all 64 lanes, so either half exceeding moves both
  if (__ballot(m_loc > m_ref + kRescaleSlack) != 0) {   // wave-uniform; always taken on a wave's first tile
    const float m_row = fmaxf(m_loc, __shfl_xor(m_loc, 32));
    const float m_new = fmaxf(m_ref, m_row);
    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);   // exp2(-inf) = 0 on the first tile
    m_ref = m_new;
    l_run *= alpha;
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[e][i] *= alpha;
  }
  float l_loc = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    s[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], scale_log2, -m_ref));
    l_loc += s[i];
  }
  l_run += l_loc;
}

typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));

// O^T[column 32e + m, query] += V_tile^T P^T, 16 keys per MFMA step.  The A operand (V^T: 8 keys of
// one head-dim column per lane) comes straight out of the row-major V tile through gfx950's
// transposing LDS read (ds_read_b64_tr_b16): within each group of 16 lanes, lane i receives element
// i%4 of the 8-byte pieces addressed by lanes i/4, i/4+4, i/4+8, i/4+12.  Pointing lane s of a group
// at key row (s/4) and column piece (s%4) therefore hands lane i four consecutive keys of column
// (16 * group parity + i); two such reads make one operand, no register shuffling.
struct PvFrags { i16x8 av[2][4]; };

// The sixteen transposed reads of one V tile (all requested together; see tile_logits).
__device__ __forceinline__ void tile_pv_load(const uint8_t* lds_v, int lane, PvFrags& f) {
  typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
  const int half = lane >> 5, grp = (lane >> 4) & 1, s16 = lane & 15;
  const uint8_t* base = lds_v + (half * 4 + (s16 >> 2)) * kVRowBytes + (grp * 16 + (s16 & 3) * 4) * 2;
#pragma unroll
  for (int step = 0; step < 2; ++step)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(base + (step * 16) * kVRowBytes + e * 64));
      const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(base + (step * 16 + 8) * kVRowBytes + e * 64));
      f.av[step][e] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
}

__device__ __forceinline__ void tile_pv_mma(const PvFrags& f, const f32x16& s, f32x16 (&acc)[4]) {
  bf16x8 pb[2];
#pragma unroll
  for (int step = 0; step < 2; ++step)
#pragma unroll
    for (int j = 0; j < 8; ++j) pb[step][j] = (__bf16)s[step * 8 + j];
#pragma unroll
  for (int step = 0; step < 2; ++step)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      acc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.av[step][e]), pb[step], acc[e], 0, 0, 0);
}

__device__ __forceinline__ void tile_pv(const uint8_t* lds_v, const f32x16& s, int lane, f32x16 (&acc)[4]) {
  PvFrags f;
  tile_pv_load(lds_v, lane, f);
  __builtin_amdgcn_sched_barrier(0);
  tile_pv_mma(f, s, acc);
}

// ---- software-pipelined form (kernels whose tiles sit in shared LDS stages) ----
// One matrix-core block: the eight logits MFMAs of the NEXT tile (a dependent chain through sn) and the
// eight PV MFMAs of the CURRENT tile (four independent accumulators), issued alternately so that no
// MFMA waits for the one just before it.  A dependent MFMA stalls at the head of the SIMD's vector
// issue port until its predecessor retires, and nothing of any wave gets past it meanwhile; spaced
// two apart the sixteen run back to back and the other wave of the SIMD does its softmax under them.
__device__ __forceinline__ void mfma_block(const bf16x8 (&a)[8], const bf16x8 (&qf)[8], f32x16& sn, const PvFrags& f,
                                           const bf16x8 (&pb)[2], f32x16 (&acc)[4]) {
#pragma unroll
  for (int i = 0; i < 16; ++i) sn[i] = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], qf[i], sn, 0, 0, 0);
    acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.av[i >> 2][i & 3]), pb[i >> 2],
                                                         acc[i & 3], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);   // the scheduler would otherwise group the dependent chain
  }
}

// The PV product alone (last tile of a pipeline: no next tile's logits to pair it with).
__device__ __forceinline__ void pv_block(const PvFrags& f, const bf16x8 (&pb)[2], f32x16 (&acc)[4]) {
#pragma unroll
  for (int i = 0; i < 8; ++i)
    acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.av[i >> 2][i & 3]), pb[i >> 2],
                                                         acc[i & 3], 0, 0, 0);
}

// Softmax numerators of a tile's raw logits, packed to the bf16 B operands of its PV product.
__device__ __forceinline__ void softmax_block(f32x16& sn, int rows, float scale_log2, int half, float& m_ref, float& l_run,
                                              f32x16 (&acc)[4], bf16x8 (&pb)[2]) {
  const float m_loc = tile_mask_max(sn, rows, scale_log2, half);
  tile_softmax(sn, m_loc, scale_log2, m_ref, l_run, acc);
#pragma unroll
  for (int st = 0; st < 2; ++st)
#pragma unroll
    for (int j = 0; j < 8; ++j) pb[st][j] = (__bf16)sn[st * 8 + j];
}

// Register (e, i) of a lane is output column 32e + 8*(i/4) + 4*half + i%4 of query row lane%32: four
// consecutive registers are four consecutive columns.
__device__ __forceinline__ int out_col0(int e, int i4, int half) { return 32 * e + 8 * i4 + 4 * half; }

// One wave owns the complete result of a head (or of a key split of it): normalised bf16 rows to
// `out_row` (n_split == 1) or fp32 numerators + (max, sum) to the split-KV partial buffers.
__device__ __forceinline__ void write_wave_result(const f32x16 (&acc)[4], float m_run, float l_tot, int lane, int half,
                                                  bool final_out, char* out_row, float* part_o_row, float* part_ml_slot) {
  if (final_out) {
    const float inv = 1.f / l_tot;
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        bf16x4 o4;
#pragma unroll
        for (int r = 0; r < 4; ++r) o4[r] = (__bf16)(acc[e][i4 * 4 + r] * inv);
        *reinterpret_cast<bf16x4*>(out_row + out_col0(e, i4, half) * 2) = o4;
      }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 o4 = {acc[e][i4 * 4], acc[e][i4 * 4 + 1], acc[e][i4 * 4 + 2], acc[e][i4 * 4 + 3]};
        *reinterpret_cast<f32x4*>(part_o_row + out_col0(e, i4, half)) = o4;
      }
    if (lane < 32) {
      part_ml_slot[lane] = m_run;
      part_ml_slot[32 + lane] = l_tot;
    }
  }
}

// Two key segments, tiles never straddling them: segment 0 contributes ceil(n0/32) tiles, segment 1
// the rest.  A tile has one wave-uniform base pointer and row count, and K and V (which share
// strides) are addressed with the same per-lane 32-bit byte offsets.
struct TileSrc {
  const char* k;
  const char* v;
  int rows;        // valid keys in this tile (1..32)
};

struct SegPtrs {
  const char* k0; const char* v0; uint32_t r0;   // byte stride per row, segment 0
  const char* k1; const char* v1; uint32_t r1;
  int n0, n1, tiles0;
};

__device__ __forceinline__ SegPtrs seg_ptrs(const AttnParams& p, int b, int g, bool two_segments) {
  SegPtrs sp;
  sp.n0 = p.seg[0].n;
  sp.n1 = two_segments ? p.seg[1].n : 0;
  sp.tiles0 = (sp.n0 + kTileKeys - 1) / kTileKeys;
  sp.r0 = (uint32_t)(p.seg[0].sr * 2);
  sp.r1 = (uint32_t)(p.seg[1].sr * 2);
  sp.k0 = (const char*)p.seg[0].k + 2 * (b * p.seg[0].sb + g * p.seg[0].sh);
  sp.v0 = (const char*)p.seg[0].v + 2 * (b * p.seg[0].sb + g * p.seg[0].sh);
  sp.k1 = (const char*)p.seg[1].k + 2 * (b * p.seg[1].sb + g * p.seg[1].sh);
  sp.v1 = (const char*)p.seg[1].v + 2 * (b * p.seg[1].sb + g * p.seg[1].sh);
  return sp;
}

__device__ __forceinline__ TileSrc tile_src(const SegPtrs& sp, int tile, uint32_t& row_stride) {
  TileSrc ts;
  if (tile < sp.tiles0) {
    const int first = tile * kTileKeys;
    ts.k = sp.k0 + (size_t)first * sp.r0;
    ts.v = sp.v0 + (size_t)first * sp.r0;
    ts.rows = min(kTileKeys, sp.n0 - first);
    row_stride = sp.r0;
  } else {
    const int first = (tile - sp.tiles0) * kTileKeys;
    ts.k = sp.k1 + (size_t)first * sp.r1;
    ts.v = sp.v1 + (size_t)first * sp.r1;
    ts.rows = min(kTileKeys, sp.n1 - first);
    row_stride = sp.r1;
  }
  return ts;
}

}  // namespace sdllm
