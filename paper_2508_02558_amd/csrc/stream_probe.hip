// Measurement aid, not part of the method: a bare streaming read with the load pattern of the
// block-attention kernel (256-byte rows fetched with non-temporal 16-byte loads, one workgroup of 512
// threads per contiguous chunk, four loads in flight per thread - the depth that measured fastest on
// MI355X).  The benchmark times it over a buffer of the sparse step's size to report how far the
// attention kernel is from what the memory system delivers for this access pattern.
#include "sdllm_internal.h"

namespace sdllm {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__global__ __launch_bounds__(512) void stream_read_kernel(const u32x4* __restrict__ src, size_t vec_per_wg, size_t n_vec,
                                                          uint32_t* sink) {
  const size_t begin = (size_t)blockIdx.x * vec_per_wg;
  const size_t end = begin + vec_per_wg < n_vec ? begin + vec_per_wg : n_vec;
  u32x4 acc = {0u, 0u, 0u, 0u};
  size_t i = begin + threadIdx.x;
  for (; i + 3 * 512 < end; i += 4 * 512) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(&src[i + u * 512]);
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u];
  }
  for (; i < end; i += 512) acc ^= __builtin_nontemporal_load(&src[i]);
  const uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (r == 0x9e3779b9u && sink) sink[0] = r;   // keeps the loads alive; practically never taken
}

hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s) {
  const size_t n_vec = bytes / 16;
  if (n_vec == 0) return hipSuccess;
  const size_t vec_per_wg = (n_vec + kNumCUs - 1) / kNumCUs;
  hipLaunchKernelGGL(stream_read_kernel, dim3(kNumCUs), dim3(512), 0, s, (const u32x4*)src, vec_per_wg, n_vec, sink);
  return hipGetLastError();
}

}  // namespace sdllm
