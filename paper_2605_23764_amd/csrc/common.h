// Shared device-side types and small helpers for the gfx950 MoE-FFN kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kChunk = 64;       // tokens per rank group (one wave, lane = token)
constexpr int kSub = 32;         // tokens per routing sub-chunk (one histogram row); two per rank group
constexpr int kMaxK = 16;        // max experts per token
constexpr int kMaxE = 256;       // max global experts (4 logits per lane)
constexpr int kMaskWords = 4;    // 64-bit words of a local-expert bitmask (E_local <= 256)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16-byte staging register
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Workspace header words (int32) shared by all kernels of one layer call.
enum MetaWord {
  kMetaMTiles = 0,   // number of M tiles in the tile map
  kMetaRows = 1,     // R: rows in expert-contiguous order
  kMetaStatus = 2,   // scheduler status (0 ok, MOE_ERR_SCHED_TIMEOUT)
  kMetaMaxRows = 3,  // rows of the largest expert
  kMetaWords = 16
};

// Tile map over the expert-contiguous rows: M tile i covers rows
// [row0[i], row0[i]+rows[i]) of local expert expert[i]; rows[i] <= BM.
struct TileMap {
  int32_t* expert;
  int32_t* row0;
  int32_t* rows;
  int32_t* meta;   // MetaWord
};

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ float bf16_to_f32(__bf16 v) { return (float)v; }

// Two fp32 -> packed bf16 pair (round to nearest even, hardware convert on gfx950).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 p = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, p);
}

__device__ __forceinline__ float bf16_lo(uint32_t p) { return __builtin_bit_cast(float, p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return __builtin_bit_cast(float, p & 0xFFFF0000u); }

__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + expf(-z)); }
// For results that are rounded to bf16 anyway: hardware exp2 and reciprocal (about 1 ulp each, and the scaling by
// log2(e) adds |z| * 2^-24 relative), a fifth of the instructions of the version above.
__device__ __forceinline__ float sigmoid_bf16_(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * z));
}

}  // namespace moe
