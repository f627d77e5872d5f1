// Dispatch permute and weighted Combine (paper Section 2.2): HBM-bound row
// movers.  One wave moves one row with 16-byte accesses, several loads in
// flight per lane.  Combine accumulates in fp32 in slot order j = 0..k-1, so the
// result is deterministic; no atomics.
#pragma once
#include "common.h"

namespace moe {

struct PermuteParams {
  const void* x;            // [T,H]
  void* Xp;                 // [R_max,H]
  const int32_t* token_of;  // [R_max]
  const int32_t* meta;      // MetaWord (R on device)
  int H;                    // elements per row
  int elem_bytes;
};

// Copy rows [r_begin, r_end) of the expert-contiguous order: Xp[r] = x[token_of[r]].
// Called by every wave of the workgroup; waves split the rows.
__device__ __forceinline__ void permute_rows(const PermuteParams& p, int r_begin, int r_end,
                                             int wave, int n_waves) {
  const int lane = lane_id();
  const int vec_per_row = (p.H * p.elem_bytes) / 16;
  for (int r = r_begin + wave; r < r_end; r += n_waves) {
    const int t = p.token_of[r];
    const uint4* src = reinterpret_cast<const uint4*>(static_cast<const char*>(p.x) + (size_t)t * p.H * p.elem_bytes);
    uint4* dst = reinterpret_cast<uint4*>(static_cast<char*>(p.Xp) + (size_t)r * p.H * p.elem_bytes);
    int v = lane;
    for (; v + 3 * kWave < vec_per_row; v += 4 * kWave) {
      uint4 a = src[v], b = src[v + kWave], c = src[v + 2 * kWave], d = src[v + 3 * kWave];
      dst[v] = a; dst[v + kWave] = b; dst[v + 2 * kWave] = c; dst[v + 3 * kWave] = d;
    }
    for (; v < vec_per_row; v += kWave) dst[v] = src[v];
  }
}

__global__ __launch_bounds__(256) void permute_kernel(PermuteParams p) {
  const int R = p.meta[kMetaRows];
  const int n_waves = blockDim.x / kWave;
  const int wave = threadIdx.x / kWave;
  // workgroup b takes rows b*n_waves .. in a grid-stride loop, one row per wave
  for (int r0 = blockIdx.x * n_waves; r0 < R; r0 += gridDim.x * n_waves)
    permute_rows(p, r0, min(R, r0 + n_waves), wave, n_waves);
}

struct CombineParams {
  const void* Yp;          // [R_max,H]
  void* out;               // [T,H]
  const int32_t* row_of;   // [T,k]
  const float* topk_w;     // [T,k]; nullptr = unit weights (backward Combine)
  int T, H, k;
};

// out[t,:] = sum_j w[t,j] * Yp[row_of[t,j],:] (local slots only), one wave per token.
template <bool BF16>
__device__ __forceinline__ void combine_token(const CombineParams& p, int t) {
  const int lane = lane_id();
  // statically indexed slot arrays (stay in registers); row < 0 = slot not local
  int rows[kMaxK];
  float w[kMaxK];
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) {
    rows[j] = j < p.k ? p.row_of[(size_t)t * p.k + j] : -1;
    w[j] = j < p.k ? (p.topk_w ? p.topk_w[(size_t)t * p.k + j] : 1.f) : 0.f;
  }
  if (BF16) {
    const int vec_per_row = p.H / 8;
    uint4* dst = reinterpret_cast<uint4*>(static_cast<__bf16*>(p.out) + (size_t)t * p.H);
    // four column chunks per lane per pass: the loads of one slot are issued together
    // (memory-level parallelism inside the wave); each element still accumulates its
    // slots in order j = 0..k-1
    constexpr int U = 4;
    for (int v0 = lane; v0 < vec_per_row; v0 += U * kWave) {
      float acc[U][8];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int x = 0; x < 8; ++x) acc[u][x] = 0.f;
#pragma unroll
      for (int i = 0; i < kMaxK; ++i) {
        if (rows[i] < 0) continue;
        const uint4* yrow = reinterpret_cast<const uint4*>(static_cast<const __bf16*>(p.Yp) + (size_t)rows[i] * p.H);
        uint4 y[U];
#pragma unroll
        for (int u = 0; u < U; ++u) y[u] = (v0 + u * kWave < vec_per_row) ? yrow[v0 + u * kWave] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          acc[u][0] += w[i] * bf16_lo(y[u].x); acc[u][1] += w[i] * bf16_hi(y[u].x);
          acc[u][2] += w[i] * bf16_lo(y[u].y); acc[u][3] += w[i] * bf16_hi(y[u].y);
          acc[u][4] += w[i] * bf16_lo(y[u].z); acc[u][5] += w[i] * bf16_hi(y[u].z);
          acc[u][6] += w[i] * bf16_lo(y[u].w); acc[u][7] += w[i] * bf16_hi(y[u].w);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (v0 + u * kWave >= vec_per_row) break;
        uint4 o;
        o.x = pack_bf16(acc[u][0], acc[u][1]); o.y = pack_bf16(acc[u][2], acc[u][3]);
        o.z = pack_bf16(acc[u][4], acc[u][5]); o.w = pack_bf16(acc[u][6], acc[u][7]);
        dst[v0 + u * kWave] = o;
      }
    }
  } else {
    const int vec_per_row = p.H / 4;
    float4* dst = reinterpret_cast<float4*>(static_cast<float*>(p.out) + (size_t)t * p.H);
    for (int v = lane; v < vec_per_row; v += kWave) {
      float4 acc = {0, 0, 0, 0};
#pragma unroll
      for (int i = 0; i < kMaxK; ++i) {
        if (rows[i] < 0) continue;
        float4 y = reinterpret_cast<const float4*>(static_cast<const float*>(p.Yp) + (size_t)rows[i] * p.H)[v];
        acc.x += w[i] * y.x; acc.y += w[i] * y.y; acc.z += w[i] * y.z; acc.w += w[i] * y.w;
      }
      dst[v] = acc;
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(CombineParams p) {
  const int n_waves = blockDim.x / kWave;
  const int wave = threadIdx.x / kWave;
  for (int t = blockIdx.x * n_waves + wave; t < p.T; t += gridDim.x * n_waves) combine_token<BF16>(p, t);
}

}  // namespace moe
