// Generic saliency scoring (Sec. 3.3 second equation + the query/head aggregation of Alg. 1):
// fp32 or bf16 storage, head_dim 64/128, any block length.  Two small kernels:
//   row_stats  : for SOFTMAX_MEAN, the max and sum-of-exponentials of every query row over all
//                candidates (one wavefront per row);
//   col_reduce : one thread per candidate key, summing that key's weight over the block's query
//                rows and the query heads of its KV group.
#include "sdllm_internal.h"

namespace sdllm {

__device__ __forceinline__ int cand_to_pos(int c, int block_off, int block_len) {
  return c < block_off ? c : c + block_len;   // K_f = Concat[K_{:o}, K_{o+b:}]
}

template <typename T, int D>
__global__ __launch_bounds__(64) void score_row_stats_kernel(const ScoreParams p) {
  __shared__ float q_s[D];
  const int lane = threadIdx.x;
  const int row = blockIdx.x;
  const int head = blockIdx.y;
  const int b = head / p.hq;
  const int h = head - b * p.hq;
  const int g = h / p.group;
  const T* q = (const T*)p.q + b * p.q_sb + h * p.q_sh + row * p.q_sr;
  for (int t = lane; t < D; t += 64) q_s[t] = (float)q[t];
  __syncthreads();
  const T* kbase = (const T*)p.k + b * p.k_sb + g * p.k_sh;
  float m = -INFINITY, l = 0.f;
  for (int c = lane; c < p.n_cand; c += 64) {
    const T* kr = kbase + (int64_t)cand_to_pos(c, p.block_off, p.block_len) * p.k_sr;
    float s = 0.f;
#pragma unroll 8
    for (int t = 0; t < D; ++t) s = fmaf(q_s[t], (float)kr[t], s);
    s *= p.scale_log2;
    const float m_new = fmaxf(m, s);
    l = l * __builtin_amdgcn_exp2f(m - m_new) + __builtin_amdgcn_exp2f(s - m_new);
    m = m_new;
  }
  float m_tot = m;
  for (int o = 32; o > 0; o >>= 1) m_tot = fmaxf(m_tot, __shfl_xor(m_tot, o));
  float l_tot = (m == -INFINITY) ? 0.f : l * __builtin_amdgcn_exp2f(m - m_tot);
  for (int o = 32; o > 0; o >>= 1) l_tot += __shfl_xor(l_tot, o);
  if (lane == 0) {
    // one partial per row: layout [B*Hq][n_part = 1][2][nq]
    p.part_ml[(size_t)head * 2 * p.nq + row] = m_tot;
    p.part_ml[(size_t)head * 2 * p.nq + p.nq + row] = l_tot;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void score_col_reduce_kernel(const ScoreParams p) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  const int bg = blockIdx.y;               // b * Hkv + g
  if (c >= p.n_cand) return;
  const int b = bg / p.hkv;
  const int g = bg - b * p.hkv;
  const T* kr = (const T*)p.k + b * p.k_sb + g * p.k_sh + (int64_t)cand_to_pos(c, p.block_off, p.block_len) * p.k_sr;
  float kf[D];
#pragma unroll
  for (int t = 0; t < D; ++t) kf[t] = (float)kr[t];
  float sum = 0.f;
  for (int hh = 0; hh < p.group; ++hh) {
    const int h = g * p.group + hh;
    const size_t head = (size_t)b * p.hq + h;
    for (int i = 0; i < p.nq; ++i) {
      const T* q = (const T*)p.q + b * p.q_sb + h * p.q_sh + i * p.q_sr;
      float s = 0.f;
#pragma unroll
      for (int t = 0; t < D; ++t) s = fmaf((float)q[t], kf[t], s);
      if (p.softmax) {
        const float m = p.part_ml[head * 2 * p.nq + i];
        const float l = p.part_ml[head * 2 * p.nq + p.nq + i];
        sum += __builtin_amdgcn_exp2f(s * p.scale_log2 - m) / l;
      } else {
        sum += s * p.scale;
      }
    }
  }
  p.score[(size_t)bg * p.score_stride + c] = sum / (float)(p.group * p.nq);
}

template <typename T, int D>
static hipError_t launch_t(const ScoreParams& p, hipStream_t s) {
  if (p.n_cand <= 0) return hipSuccess;
  if (p.softmax)
    hipLaunchKernelGGL((score_row_stats_kernel<T, D>), dim3(p.nq, p.batch * p.hq), dim3(64), 0, s, p);
  hipLaunchKernelGGL((score_col_reduce_kernel<T, D>), dim3((p.n_cand + 255) / 256, p.batch * p.hkv), dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_score_simple(const ScoreParams& p, int dtype, hipStream_t s) {
  if (dtype == 0) return p.d == 128 ? launch_t<__bf16, 128>(p, s) : launch_t<__bf16, 64>(p, s);
  return p.d == 128 ? launch_t<float, 128>(p, s) : launch_t<float, 64>(p, s);
}

}  // namespace sdllm
