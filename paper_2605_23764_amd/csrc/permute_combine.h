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
// Called by every wave of the workgroup; waves split the rows.  U = 16-byte loads a
// lane keeps in flight: 4 is enough when a CU holds dozens of waves; a worker of the
// persistent kernel has four waves on its CU and needs the memory-level parallelism
// inside the wave (a whole row in flight).  The copies are non-temporal: every byte is
// touched once, and with ordinary loads more than four in flight per lane made the
// persistent tasks slower (53 / 82 / 117 us per task at 4 / 7 / 14), not faster.
template <int U>
__device__ __forceinline__ void permute_rows(const PermuteParams& p, int r_begin, int r_end,
                                             int wave, int n_waves) {
  const int lane = lane_id();
  const int vec_per_row = (p.H * p.elem_bytes) / 16;
  const size_t row_bytes = (size_t)p.H * p.elem_bytes;
  // This wave's rows are r_begin + wave + i * n_waves.  Their tokens are fetched with one load (lane i: row i; 64
  // rows at a time) instead of one dependent load per row, and two rows are copied per pass, the loads of both in
  // flight before the first store: with only a few waves per CU the copy is latency bound otherwise.
  for (int base = r_begin + wave; base < r_end; base += kWave * n_waves) {
    const int n_rows = min(kWave, (r_end - base + n_waves - 1) / n_waves);   // wave-uniform
    const int tok_lane = lane < n_rows ? p.token_of[base + lane * n_waves] : 0;
    for (int i = 0; i < n_rows; i += 2) {
      const bool two = i + 1 < n_rows;
      const int t0 = __builtin_amdgcn_readlane(tok_lane, i), t1 = __builtin_amdgcn_readlane(tok_lane, two ? i + 1 : i);
      const int r0 = base + i * n_waves, r1 = r0 + n_waves;
      const uint4* src0 = reinterpret_cast<const uint4*>(static_cast<const char*>(p.x) + (size_t)t0 * row_bytes);
      const uint4* src1 = reinterpret_cast<const uint4*>(static_cast<const char*>(p.x) + (size_t)t1 * row_bytes);
      uint4* dst0 = reinterpret_cast<uint4*>(static_cast<char*>(p.Xp) + (size_t)r0 * row_bytes);
      uint4* dst1 = reinterpret_cast<uint4*>(static_cast<char*>(p.Xp) + (size_t)r1 * row_bytes);
      int v = lane;
      for (; v + (U - 1) * kWave < vec_per_row; v += U * kWave) {
        u32x4 q0[U], q1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) q0[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src0 + v + u * kWave));
        if (two) {
#pragma unroll
          for (int u = 0; u < U; ++u) q1[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src1 + v + u * kWave));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) __builtin_nontemporal_store(q0[u], reinterpret_cast<u32x4*>(dst0 + v + u * kWave));
        if (two) {
#pragma unroll
          for (int u = 0; u < U; ++u) __builtin_nontemporal_store(q1[u], reinterpret_cast<u32x4*>(dst1 + v + u * kWave));
        }
      }
      for (; v < vec_per_row; v += kWave) {
        dst0[v] = src0[v];
        if (two) dst1[v] = src1[v];
      }
    }
  }
}

__global__ __launch_bounds__(256) void permute_kernel(PermuteParams p) {
  const int R = p.meta[kMetaRows];
  const int n_waves = blockDim.x / kWave;
  const int wave = threadIdx.x / kWave;
  // workgroup b takes rows b*n_waves .. in a grid-stride loop, one row per wave
  for (int r0 = blockIdx.x * n_waves; r0 < R; r0 += gridDim.x * n_waves)
    permute_rows<4>(p, r0, min(R, r0 + n_waves), wave, n_waves);
}

// The same copy for the rows of experts with at least k_lo rows only (offsets: E_local + 1 prefix sums of
// the rows per expert).  Used by the backward when the forward kept no permuted copy: the register-
// stationary weight-gradient kernel reads x through the permutation itself, the general kernel (experts
// above its row limit) reads this partial copy.
__global__ __launch_bounds__(256) void permute_large_experts_kernel(PermuteParams p, const int32_t* offsets, int E_local,
                                                                    int k_lo) {
  const int n_waves = blockDim.x / kWave;
  const int wave = threadIdx.x / kWave;
  for (int e = 0; e < E_local; ++e) {
    const int seg0 = offsets[e], seg1 = offsets[e + 1];
    if (seg1 - seg0 < k_lo) continue;
    for (int r0 = seg0 + blockIdx.x * n_waves; r0 < seg1; r0 += gridDim.x * n_waves)
      permute_rows<4>(p, r0, min(seg1, r0 + n_waves), wave, n_waves);
  }
}

struct CombineParams {
  const void* Yp;          // [R_max,H]
  void* out;               // [T,H]
  const int32_t* row_of;   // [T,k]
  const float* topk_w;     // [T,k]; nullptr = unit weights (backward Combine)
  int T, H, k;
};

// acc[0..EPV) += w * (the elements of one 16-byte vector)
template <bool BF16>
__device__ __forceinline__ void accumulate(float (&acc)[BF16 ? 8 : 4], float w, const uint4& y) {
  if constexpr (BF16) {
    acc[0] += w * bf16_lo(y.x); acc[1] += w * bf16_hi(y.x);
    acc[2] += w * bf16_lo(y.y); acc[3] += w * bf16_hi(y.y);
    acc[4] += w * bf16_lo(y.z); acc[5] += w * bf16_hi(y.z);
    acc[6] += w * bf16_lo(y.w); acc[7] += w * bf16_hi(y.w);
  } else {
    acc[0] += w * __builtin_bit_cast(float, y.x); acc[1] += w * __builtin_bit_cast(float, y.y);
    acc[2] += w * __builtin_bit_cast(float, y.z); acc[3] += w * __builtin_bit_cast(float, y.w);
  }
}

// out[t,:] = sum_j w[t,j] * Yp[row_of[t,j],:] (local slots only), one wave per token.
// Lane j < k holds slot j; the local slots are walked in ascending j through the
// ballot of "row >= 0", two at a time, rows and weights as wave-uniform scalars, so
// the loads of both rows are in flight together and no per-slot branch breaks up the
// load batches.  Each element still accumulates its slots in order j = 0..k-1.
// UV = 16-byte vectors per lane per pass: 7 (4 for fp32) when a CU holds dozens of waves; a worker of the
// persistent kernel has four waves on its CU and takes a whole 7168-element row per pass (14), i.e. up to 28
// loads in flight per lane.  The arithmetic per element is the same for every UV.
// combine_token_rows: the token's slots are already in registers (lane j: row of slot j or -1, its score), G rows
// in flight at a time; the sum runs in slot order whatever G is, so every G gives the same bits.
template <bool BF16, int UV, int G>
__device__ __forceinline__ void combine_token_rows(const CombineParams& p, int t, int rowv, float wv) {
  const int lane = lane_id();
  const uint64_t local = __ballot(rowv >= 0);
  constexpr int EPV = BF16 ? 8 : 4;                 // elements per 16-byte vector
  constexpr int U = UV;                             // vectors per lane per pass
  const int vec_per_row = p.H / EPV;
  const size_t row_bytes = (size_t)p.H * (BF16 ? 2 : 4);
  uint4* dst = reinterpret_cast<uint4*>(static_cast<char*>(p.out) + (size_t)t * row_bytes);
  for (int v0 = lane; v0 < vec_per_row; v0 += U * kWave) {
    float acc[U][EPV];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int x = 0; x < EPV; ++x) acc[u][x] = 0.f;
    uint64_t m = local;
    while (m != 0) {
      const uint4* yp[G];
      float w[G];
      int n = 0;                                    // wave-uniform: rows of this round
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const bool have = m != 0;
        const int j = have ? __builtin_amdgcn_readfirstlane(__builtin_ctzll(m)) : 0;
        if (have) { m &= m - 1; n = g + 1; }
        const int r = __builtin_amdgcn_readlane(rowv, j);
        w[g] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv), j));
        yp[g] = reinterpret_cast<const uint4*>(static_cast<const char*>(p.Yp) + (size_t)(have ? r : 0) * row_bytes);
      }
      uint4 y[G][U];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (g >= n) break;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const bool ok = v0 + u * kWave < vec_per_row;
          y[g][u] = ok ? yp[g][v0 + u * kWave] : make_uint4(0, 0, 0, 0);
        }
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (g >= n) break;
#pragma unroll
        for (int u = 0; u < U; ++u) accumulate<BF16>(acc[u], w[g], y[g][u]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (v0 + u * kWave >= vec_per_row) break;
      uint4 o;
      if constexpr (BF16) {
        o.x = pack_bf16(acc[u][0], acc[u][1]); o.y = pack_bf16(acc[u][2], acc[u][3]);
        o.z = pack_bf16(acc[u][4], acc[u][5]); o.w = pack_bf16(acc[u][6], acc[u][7]);
      } else {
        o.x = __builtin_bit_cast(uint32_t, acc[u][0]); o.y = __builtin_bit_cast(uint32_t, acc[u][1]);
        o.z = __builtin_bit_cast(uint32_t, acc[u][2]); o.w = __builtin_bit_cast(uint32_t, acc[u][3]);
      }
      dst[v0 + u * kWave] = o;
    }
  }
}

// The token's slots as the lanes hold them: lane j < k the row of slot j (-1: not on this GPU) and its score.
__device__ __forceinline__ void combine_load_slots(const CombineParams& p, int t, int& rowv, float& wv) {
  const int lane = lane_id();
  rowv = -1;
  wv = 0.f;
  if (lane < p.k) {
    rowv = p.row_of[(size_t)t * p.k + lane];
    wv = p.topk_w ? p.topk_w[(size_t)t * p.k + lane] : 1.f;
  }
}

template <bool BF16, int UV = (BF16 ? 7 : 4), int G = 2>
__device__ __forceinline__ void combine_token(const CombineParams& p, int t) {
  int rowv;
  float wv;
  combine_load_slots(p, t, rowv, wv);
  combine_token_rows<BF16, UV, G>(p, t, rowv, wv);
}

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(CombineParams p) {
  const int n_waves = blockDim.x / kWave;
  const int wave = threadIdx.x / kWave;
  for (int t = blockIdx.x * n_waves + wave; t < p.T; t += gridDim.x * n_waves) combine_token<BF16>(p, t);
}

// Zeroes n16 16-byte vectors at dst: the layer output ahead of a GEMM-2 whose epilogue adds its rows into it
// (a kernel, not a memset node, so that the sequence can be captured in a graph).
__global__ __launch_bounds__(256) void zero_fill_kernel(uint4* dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace moe
