// Gather-compaction of the retained K/V rows into the dense sparse cache (Sec. 3.3 fourth
// equation; Alg. 1 steps 12-14).  Pure byte movement: each thread copies one 16-byte chunk of two
// consecutive cache rows of K and of V, so a wavefront reads and writes whole rows with 16-byte
// non-temporal accesses and has 4 loads in flight per lane (more in flight measured slower).
//
// At the cache-update step of a shape whose dense attention was split over the keys, the merge of those
// splits has nothing to do with the gather and is only needed once the step returns: one launch then
// runs both (compact_combine_kernel: the first blocks merge, the rest copy), which saves a launch
// boundary and hides the merge under the copy.
#include "attn_merge.h"
#include "sdllm_internal.h"

namespace sdllm {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kRowsPerThread = 2;
constexpr int kCompactThreads = 256;
static_assert(kCompactThreads == kCombineThreads, "the fused launch runs both bodies with one block size");

__device__ __forceinline__ void compact_block(const CompactParams& p, int64_t block_id) {
  const int chunks = p.row_bytes >> 4;
  const int64_t gid = block_id * kCompactThreads + threadIdx.x;
  const int64_t rgroup = gid / chunks;
  const int c16 = (int)(gid - rgroup * chunks) << 4;
  const int64_t total_rows = (int64_t)p.batch * p.hkv * p.k_total;
  const int64_t r0 = rgroup * kRowsPerThread;
  if (r0 >= total_rows) return;

  const char* src_k[kRowsPerThread]; const char* src_v[kRowsPerThread];
  char* dst_k[kRowsPerThread]; char* dst_v[kRowsPerThread];
  bool ok[kRowsPerThread];
#pragma unroll
  for (int u = 0; u < kRowsPerThread; ++u) {
    const int64_t r = r0 + u;
    ok[u] = r < total_rows;
    const int64_t rr = ok[u] ? r : total_rows - 1;
    const int bg = (int)(rr / p.k_total);
    const int j = (int)(rr - (int64_t)bg * p.k_total);
    const int b = bg / p.hkv;
    const int g = bg - b * p.hkv;
    int pos = p.idx[rr];
    pos = min(max(pos, 0), p.seq_len - 1);   // never leave the source tensor, whatever idx holds
    const int64_t so = b * p.s_sb + g * p.s_sh + (int64_t)pos * p.s_sr + c16;
    const int64_t co = b * p.c_sb + g * p.c_sh + (int64_t)j * p.c_sr + c16;
    src_k[u] = (const char*)p.k + so; src_v[u] = (const char*)p.v + so;
    dst_k[u] = (char*)p.kc + co; dst_v[u] = (char*)p.vc + co;
  }
  u32x4 kv[kRowsPerThread], vv[kRowsPerThread];
#pragma unroll
  for (int u = 0; u < kRowsPerThread; ++u) {
    kv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src_k[u]));
    vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src_v[u]));
  }
#pragma unroll
  for (int u = 0; u < kRowsPerThread; ++u) {
    if (ok[u]) {
      __builtin_nontemporal_store(kv[u], reinterpret_cast<u32x4*>(dst_k[u]));
      __builtin_nontemporal_store(vv[u], reinterpret_cast<u32x4*>(dst_v[u]));
    }
  }
}

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(const CompactParams p) { compact_block(p, blockIdx.x); }

// blocks [0, n_combine): split-KV merge of the attention described by `a` (bf16 output); the rest: the gather
template <int TPI>
__global__ __launch_bounds__(kCompactThreads) void compact_combine_kernel(const CompactParams p, const AttnParams a,
                                                                          const int n_combine) {
  if ((int)blockIdx.x < n_combine) combine_block<__bf16, TPI>(a, blockIdx.x);
  else compact_block(p, (int64_t)blockIdx.x - n_combine);
}

static int64_t compact_blocks(const CompactParams& p) {
  const int64_t total_rows = (int64_t)p.batch * p.hkv * p.k_total;
  const int chunks = p.row_bytes >> 4;
  const int64_t threads = ((total_rows + kRowsPerThread - 1) / kRowsPerThread) * chunks;
  return (threads + kCompactThreads - 1) / kCompactThreads;
}

hipError_t launch_compact(const CompactParams& p, hipStream_t s) {
  const int64_t blocks = compact_blocks(p);
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(compact_kernel, dim3((unsigned)blocks), dim3(kCompactThreads), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_compact_combine(const CompactParams& p, const AttnParams& a, hipStream_t s) {
  const int64_t n_combine = combine_blocks(a);
  const int64_t blocks = n_combine + compact_blocks(p);
  if (combine_tpi(a.n_split) == 4)
    hipLaunchKernelGGL(compact_combine_kernel<4>, dim3((unsigned)blocks), dim3(kCompactThreads), 0, s, p, a, (int)n_combine);
  else
    hipLaunchKernelGGL(compact_combine_kernel<1>, dim3((unsigned)blocks), dim3(kCompactThreads), 0, s, p, a, (int)n_combine);
  return hipGetLastError();
}

}  // namespace sdllm
