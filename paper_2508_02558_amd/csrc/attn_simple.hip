// Generic attention kernels: any query-row count, head_dim 64/128, fp32 or bf16 storage, plus the
// split-KV combine used by the MFMA kernel.  One wavefront per (head, query row); each lane keeps
// a private online softmax over the keys it strides through and the 64 partial states are merged
// at the end.  This is the path for shapes the MFMA kernel does not cover (fp32 tensors, head_dim
// 64, block lengths other than 32); it favours simplicity over speed.
#include <type_traits>

#include "attn_merge.h"
#include "sdllm_internal.h"

namespace sdllm {

template <typename T> __device__ __forceinline__ float to_f32(T x) { return (float)x; }

template <typename T, int D>
__global__ __launch_bounds__(64) void attn_simple_kernel(const AttnParams p) {
  __shared__ float q_s[D];
  __shared__ float red[64][D + 1];
  const int lane = threadIdx.x;
  const int row = blockIdx.x;
  const int head = blockIdx.y;
  const int b = head / p.hq;
  const int h = head - b * p.hq;
  const int g = h / p.group;

  const T* q = (const T*)p.q + b * p.q_sb + h * p.q_sh + row * p.q_sr;
  for (int t = lane; t < D; t += 64) q_s[t] = to_f32(q[t]);
  __syncthreads();

  float acc[D];
#pragma unroll
  for (int t = 0; t < D; ++t) acc[t] = 0.f;
  float m = -INFINITY, l = 0.f;
  const int n0 = p.seg[0].n, M = p.seg[0].n + p.seg[1].n;
  for (int j = lane; j < M; j += 64) {
    const T* kr; const T* vr;
    if (j < n0) {
      const int64_t off = b * p.seg[0].sb + g * p.seg[0].sh + (int64_t)j * p.seg[0].sr;
      kr = (const T*)p.seg[0].k + off; vr = (const T*)p.seg[0].v + off;
    } else {
      const int64_t off = b * p.seg[1].sb + g * p.seg[1].sh + (int64_t)(j - n0) * p.seg[1].sr;
      kr = (const T*)p.seg[1].k + off; vr = (const T*)p.seg[1].v + off;
    }
    float s = 0.f;
#pragma unroll 8
    for (int t = 0; t < D; ++t) s = fmaf(q_s[t], to_f32(kr[t]), s);
    s *= p.scale_log2;
    const float m_new = fmaxf(m, s);
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    const float pj = __builtin_amdgcn_exp2f(s - m_new);
    l = l * alpha + pj;
    m = m_new;
#pragma unroll
    for (int t = 0; t < D; ++t) acc[t] = fmaf(pj, to_f32(vr[t]), acc[t] * alpha);
  }
  float m_tot = m;
  for (int o = 32; o > 0; o >>= 1) m_tot = fmaxf(m_tot, __shfl_xor(m_tot, o));
  const float f = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - m_tot);
  float l_tot = l * f;
  for (int o = 32; o > 0; o >>= 1) l_tot += __shfl_xor(l_tot, o);
#pragma unroll
  for (int t = 0; t < D; ++t) red[lane][t] = acc[t] * f;
  __syncthreads();
  T* out = (T*)p.out + b * p.o_sb + h * p.o_sh + row * p.o_sr;
  for (int t = lane; t < D; t += 64) {
    float sum = 0.f;
    for (int w = 0; w < 64; ++w) sum += red[w][t];
    out[t] = (T)(sum / l_tot);
  }
}

// The split-KV merge as a launch of its own (combine_block in attn_merge.h does the work).
template <typename T, int TPI>
__global__ __launch_bounds__(kCombineThreads) void attn_combine_kernel(const AttnParams p) {
  combine_block<T, TPI>(p, blockIdx.x);
}

hipError_t launch_attn_simple(const AttnParams& p, int dtype, hipStream_t s) {
  const dim3 grid(p.nq, p.batch * p.hq);
  if (dtype == 0) {
    if (p.d == 128) hipLaunchKernelGGL((attn_simple_kernel<__bf16, 128>), grid, dim3(64), 0, s, p);
    else hipLaunchKernelGGL((attn_simple_kernel<__bf16, 64>), grid, dim3(64), 0, s, p);
  } else {
    if (p.d == 128) hipLaunchKernelGGL((attn_simple_kernel<float, 128>), grid, dim3(64), 0, s, p);
    else hipLaunchKernelGGL((attn_simple_kernel<float, 64>), grid, dim3(64), 0, s, p);
  }
  return hipGetLastError();
}

hipError_t launch_attn_combine(const AttnParams& p, int dtype, hipStream_t s) {
  const int tpi = combine_tpi(p.n_split);
  const dim3 grid((unsigned)combine_blocks(p)), block(kCombineThreads);
  if (dtype == 0) {
    if (tpi == 4) hipLaunchKernelGGL((attn_combine_kernel<__bf16, 4>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((attn_combine_kernel<__bf16, 1>), grid, block, 0, s, p);
  } else {
    if (tpi == 4) hipLaunchKernelGGL((attn_combine_kernel<float, 4>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((attn_combine_kernel<float, 1>), grid, block, 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace sdllm
