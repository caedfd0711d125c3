// Gather-compaction of the retained K/V rows into the dense sparse cache (Sec. 3.3 fourth
// equation; Alg. 1 steps 12-14).  Pure byte movement: each thread copies one 16-byte chunk of two
// consecutive cache rows of K and of V, so a wavefront reads and writes whole rows with 16-byte
// non-temporal accesses and has 4 loads in flight per lane (more in flight measured slower).
#include "sdllm_internal.h"

namespace sdllm {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kRowsPerThread = 2;

__global__ __launch_bounds__(256) void compact_kernel(const CompactParams p) {
  const int chunks = p.row_bytes >> 4;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
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

hipError_t launch_compact(const CompactParams& p, hipStream_t s) {
  const int64_t total_rows = (int64_t)p.batch * p.hkv * p.k_total;
  if (total_rows == 0) return hipSuccess;
  const int chunks = p.row_bytes >> 4;
  const int64_t threads = ((total_rows + kRowsPerThread - 1) / kRowsPerThread) * chunks;
  const int64_t blocks = (threads + 255) / 256;
  hipLaunchKernelGGL(compact_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace sdllm
