// Device helpers shared by the bf16 MFMA kernels: vector types, the padded LDS tile layout and the
// coalesced 32-key tile load.
#pragma once

#include "sdllm_internal.h"

namespace sdllm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
// native vectors (not the HIP uint4 struct) so that register arrays of them are promoted to VGPRs
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kRowBytes = 256 + 16;               // 128 bf16 + one 16-byte pad: rows rotate over the banks
constexpr int kTileBytes = kTileKeys * kRowBytes; // one 32 x 128 bf16 tile in LDS

// V tiles use 320-byte rows: the transposing LDS read of the PV product touches four consecutive
// rows x 64 bytes per 32 lanes, and a row offset of 64 bytes (mod 256) puts those on 64 distinct banks.
constexpr int kVRowBytes = 256 + 64;
constexpr int kVTileBytes = kTileKeys * kVRowBytes;

__device__ __forceinline__ uint32_t vtile_off(int row, int chunk) { return (uint32_t)(row * kVRowBytes + (chunk << 4)); }

__device__ __forceinline__ uint32_t tile_off(int row, int chunk) {
  // padded rows: the sixteen lanes that read one chunk column of sixteen rows hit sixteen different
  // 16-byte bank groups, and every address is a per-lane base plus a compile-time constant
  return (uint32_t)(row * kRowBytes + (chunk << 4));
}

// Rows [0, rows) of a tile starting at `base` (wave-uniform), `stride` bytes apart: lane l loads the
// 16-byte chunk l%16 of rows l/16, l/16 + 4, ...  Rows past the end re-read the last valid row.
// NT: non-temporal loads for data that is streamed once per launch (they keep the tiles from
// displacing reusable lines in L2/MALL and measured ~12 % faster on MI355X); plain loads when sibling
// workgroups re-read the same rows (query heads of one KV group served by separate workgroups).
// A full tile (the common case, wave-uniform test) is addressed as base + j * (4 rows) (scalar) plus ONE
// per-lane offset, so the eight loads cost the vector ALU one multiply and eight adds instead of
// eight clamps, eight multiplies and eight adds (with two such calls per tile the address arithmetic
// was half of the vector-ALU time of an attention tile).
template <bool NT = true>
__device__ __forceinline__ void load_rows(const char* base, int rows, uint32_t stride, int lane, u32x4 (&reg)[8]) {
  const uint32_t c16 = (lane & 15) << 4;
  if (rows == kTileKeys) {
    const uint32_t lane_off = (uint32_t)(lane >> 4) * stride + c16;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const u32x4* src = reinterpret_cast<const u32x4*>(base + (size_t)(j * 4) * stride + lane_off);
      reg[j] = NT ? __builtin_nontemporal_load(src) : *src;
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    int r = j * 4 + (lane >> 4);
    r = r < rows ? r : rows - 1;
    const u32x4* src = reinterpret_cast<const u32x4*>(base + (uint32_t)r * stride + c16);
    reg[j] = NT ? __builtin_nontemporal_load(src) : *src;
  }
}

__device__ __forceinline__ void store_rows(uint8_t* lds_tile, int lane, const u32x4 (&reg)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j)
    *reinterpret_cast<u32x4*>(lds_tile + tile_off(j * 4 + (lane >> 4), lane & 15)) = reg[j];
}

__device__ __forceinline__ void store_rows_v(uint8_t* lds_tile, int lane, const u32x4 (&reg)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j)
    *reinterpret_cast<u32x4*>(lds_tile + vtile_off(j * 4 + (lane >> 4), lane & 15)) = reg[j];
}

// make this wave's LDS writes visible to its own later reads (wave-private tiles need no s_barrier)
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace sdllm
