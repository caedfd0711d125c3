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

}  // namespace sdllm
