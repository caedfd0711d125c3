// Merging the split-KV partials of one query row (Alg. 3, cache_state == 2: the softmax runs over
// Concat(K_c, K_n) as a whole, so the (max, sum, numerator) triples that the key splits of a head
// leave behind are folded with the usual rescaling).
#pragma once

#include <type_traits>

#include "sdllm_internal.h"

namespace sdllm {

typedef __attribute__((ext_vector_type(4))) float mf32x4;
typedef __attribute__((ext_vector_type(4))) __bf16 mbf16x4;

// Running (max, sum, numerators) of one query row's four output columns.
struct RowPiece {
  float m = -INFINITY, l = 0.f;
  mf32x4 o = {0.f, 0.f, 0.f, 0.f};
};

__device__ __forceinline__ void merge_pieces(RowPiece& a, const RowPiece& b) {
  const float m_new = fmaxf(a.m, b.m);
  const float fa = a.m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(a.m - m_new);
  const float fb = b.m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(b.m - m_new);
  a.l = a.l * fa + b.l * fb;
  a.o = a.o * fa + b.o * fb;
  a.m = m_new;
}

// One thread folds the splits first, first + step, ... of one query row's four output columns.  ml
// points at the row's max of split 0 (split stride ml_ss floats, the sum nq floats further on), po at the
// row's four numerators of split 0 (split stride po_ss floats).  One sweep in batches of eight (then
// four) splits: all loads of a batch (max, sum, numerators) are requested before any is used, then folded
// into the running piece.  The partials were written a moment ago and mostly sit in L2; what a merge
// pays for is dependent round trips, and a separate pass for the overall max plus batches of four cost
// five or six of them.
__device__ __forceinline__ RowPiece fold_splits(const float* ml, int ml_ss, int nq, const float* po, size_t po_ss, int n_split,
                                                int first, int step) {
  RowPiece r;
  const int n_mine = first < n_split ? (n_split - first + step - 1) / step : 0;
  auto fold = [&](auto batch, int j0) {
    constexpr int NB = decltype(batch)::value;
    float m_s[NB], l_s[NB];
    mf32x4 o_s[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int s = first + min(j0 + u, n_mine - 1) * step;   // past the end (last batch only): re-read the last one, weight 0 below
      m_s[u] = ml[s * ml_ss];
      l_s[u] = ml[s * ml_ss + nq];
      o_s[u] = *reinterpret_cast<const mf32x4*>(po + s * po_ss);
    }
    float m_new = r.m;
#pragma unroll
    for (int u = 0; u < NB; ++u) m_new = fmaxf(m_new, m_s[u]);   // the re-read duplicates change nothing
    if (m_new == -INFINITY) return;                              // nothing but empty splits so far
    const float f_old = __builtin_amdgcn_exp2f(r.m - m_new);    // 0 on the first batch
    r.l *= f_old;
    r.o *= f_old;
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const float f = (j0 + u < n_mine && m_s[u] != -INFINITY) ? __builtin_amdgcn_exp2f(m_s[u] - m_new) : 0.f;
      r.l += f * l_s[u];
      r.o += f * o_s[u];
    }
    r.m = m_new;
  };
  int j0 = 0;
  for (; j0 + 4 < n_mine; j0 += 8) fold(std::integral_constant<int, 8>{}, j0);   // five or more left
  if (j0 < n_mine) fold(std::integral_constant<int, 4>{}, j0);
  return r;
}

// Normalised output of a merged piece: four consecutive columns of one row.
template <typename T>
__device__ __forceinline__ void store_piece(const RowPiece& r, T* out) {
  const float inv = 1.f / r.l;
  if constexpr (sizeof(T) == 2) {
    mbf16x4 v;
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = (__bf16)(r.o[c] * inv);
    *reinterpret_cast<mbf16x4*>(out) = v;      // rows and row strides are 16-byte aligned, the column a multiple of 4
  } else {
    *reinterpret_cast<mf32x4*>(out) = r.o * inv;
  }
}

// Merge the n_split partial (max, sum, numerator) triples of each query row: TPI threads per (row, four
// output columns), 16-byte loads, eight splits' loads in flight per thread (the partials mostly sit in
// L2 / MALL, so the merge is bound by dependent round trips).  TPI = 1 for a few splits; with 16 and more
// (long rows on few KV heads: 64 splits at the batch-1 32k-prompt grouped-query shape) four adjacent lanes
// take every fourth split each and merge their pieces with two shuffles, which cuts the dependent batches
// of loads from eight to two.
// One block of kCombineThreads threads = kCombineThreads / TPI items of the [B*Hq, nq] x (d/4) item list.
constexpr int kCombineThreads = 256;

__host__ __device__ inline int combine_tpi(int n_split) { return n_split >= 16 ? 4 : 1; }

// blocks of kCombineThreads threads that cover every item
inline int64_t combine_blocks(const AttnParams& p) {
  const int64_t threads = (int64_t)p.batch * p.hq * p.nq * (p.d >> 2) * combine_tpi(p.n_split);
  return (threads + kCombineThreads - 1) / kCombineThreads;
}

template <typename T, int TPI>
__device__ __forceinline__ void combine_block(const AttnParams& p, int block_id) {
  const int total_rows = p.batch * p.hq * p.nq;
  const int per_row = p.d >> 2;                                   // items per row
  const int tid = block_id * kCombineThreads + threadIdx.x;
  const int item = tid / TPI, sub = tid - item * TPI;
  const int grow = item / per_row;                                // index into the [B*Hq, nq] row list
  const bool valid = grow < total_rows;                           // whole groups of TPI lanes are valid or not
  const int growc = valid ? grow : total_rows - 1;
  const int c4 = valid ? (item - grow * per_row) << 2 : 0;
  const int head = growc / p.nq;
  const int row = growc - head * p.nq;
  const int b = head / p.hq;
  const int h = head - b * p.hq;
  const float* ml = p.part_ml + (size_t)head * p.n_split * 2 * p.nq + row;        // split stride 2*nq
  const float* po = p.part_o + ((size_t)head * p.n_split * p.nq + row) * p.d + c4;   // split stride nq*d
  RowPiece r = fold_splits(ml, 2 * p.nq, p.nq, po, (size_t)p.nq * p.d, p.n_split, sub, TPI);
#pragma unroll
  for (int o = 1; o < TPI; o <<= 1) {
    RowPiece other;
    other.m = __shfl_xor(r.m, o);
    other.l = __shfl_xor(r.l, o);
#pragma unroll
    for (int c = 0; c < 4; ++c) other.o[c] = __shfl_xor(r.o[c], o);
    merge_pieces(r, other);
  }
  if (valid && sub == 0) store_piece<T>(r, (T*)p.out + b * p.o_sb + h * p.o_sh + row * p.o_sr + c4);
}

}  // namespace sdllm
