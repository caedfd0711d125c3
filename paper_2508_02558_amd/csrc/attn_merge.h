// Merging the split-KV partials of one query row (Alg. 3, cache_state == 2: the softmax runs over
// Concat(K_c, K_n) as a whole, so the (max, sum, numerator) triples that the key splits of a head
// leave behind are folded with the usual rescaling).  Shared by the stand-alone combine kernel and by
// the attention kernels that merge their own splits (last workgroup to arrive).
#pragma once

#include <type_traits>

#include "sdllm_internal.h"

namespace sdllm {

typedef __attribute__((ext_vector_type(4))) float mf32x4;
typedef __attribute__((ext_vector_type(4))) __bf16 mbf16x4;

// One thread, one query row, four output columns.  ml points at the row's max of split 0 (split
// stride ml_ss floats, the sum nq floats further on), po at the row's four numerators of split 0 (split
// stride po_ss floats).  One sweep in batches of eight (then four) splits: all loads of a batch (max,
// sum, numerators) are requested before any is used, then folded into the running (max, sum,
// numerator).  The partials were written a moment ago and mostly sit in L2; what a merge pays for is
// dependent round trips, and a separate pass for the overall max plus batches of four cost five or
// six of them.
template <typename T>
__device__ __forceinline__ void merge_row_piece(const float* ml, int ml_ss, int nq, const float* po, size_t po_ss,
                                                int n_split, T* out) {
  float m_tot = -INFINITY, l_tot = 0.f;
  mf32x4 o = {0.f, 0.f, 0.f, 0.f};
  auto fold = [&](auto batch, int s0) {
    constexpr int NB = decltype(batch)::value;
    float m_s[NB], l_s[NB];
    mf32x4 o_s[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int s = min(s0 + u, n_split - 1);   // past the end (last batch only): re-read the last split, weight 0 below
      m_s[u] = ml[s * ml_ss];
      l_s[u] = ml[s * ml_ss + nq];
      o_s[u] = *reinterpret_cast<const mf32x4*>(po + s * po_ss);
    }
    float m_new = m_tot;
#pragma unroll
    for (int u = 0; u < NB; ++u) m_new = fmaxf(m_new, m_s[u]);   // the re-read duplicates change nothing
    if (m_new == -INFINITY) return;                              // nothing but empty splits so far
    const float f_old = __builtin_amdgcn_exp2f(m_tot - m_new);  // 0 on the first batch
    l_tot *= f_old;
    o *= f_old;
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const float f = (s0 + u < n_split && m_s[u] != -INFINITY) ? __builtin_amdgcn_exp2f(m_s[u] - m_new) : 0.f;
      l_tot += f * l_s[u];
      o += f * o_s[u];
    }
    m_tot = m_new;
  };
  int s0 = 0;
  for (; s0 + 4 < n_split; s0 += 8) fold(std::integral_constant<int, 8>{}, s0);   // five or more left
  if (s0 < n_split) fold(std::integral_constant<int, 4>{}, s0);
  const float inv = 1.f / l_tot;
  if constexpr (sizeof(T) == 2) {
    mbf16x4 v;
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = (__bf16)(o[r] * inv);
    *reinterpret_cast<mbf16x4*>(out) = v;      // rows and row strides are 16-byte aligned, the column a multiple of 4
  } else {
    *reinterpret_cast<mf32x4*>(out) = o * inv;
  }
}

}  // namespace sdllm
