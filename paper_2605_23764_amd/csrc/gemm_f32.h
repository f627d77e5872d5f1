// Grouped fp32 GEMM (same operators as gemm_bf16.h, for the fp32 storage type).
// True fp32 multiply-add on the vector ALU, LDS-tiled 64 x 64 x 16, each thread a
// 4 x 4 block; K never split.  This path exists for exactness (the fp32
// workload's tolerance is 1e-5), not for throughput.
#pragma once
#include "common.h"
#include "gemm_bf16.h"  // GemmEpilogue, xcd_tile_id

namespace moe {

constexpr int kFBM = 64, kFBN = 64, kFBK = 16;

struct GemmParamsF32 {
  const float* A;   // [rows, lda]
  const float* B;   // per expert [K, ldb]
  float* C;         // [rows, ldc]
  float* C2;        // SwiGLU only: optional pre-activation [rows, 2N]
  long strideB;
  int K, N;         // N = output columns (SwiGLU: I)
  int lda, ldb, ldc;
  int n_ntiles;     // N / 64
  TileMap tiles;
};

template <int EPI>
__device__ __forceinline__ void gemm_tile_f32(const GemmParamsF32& p, int mtile, int ntile, float* smem) {
  constexpr int NB = (EPI == kEpiSwiglu) ? 2 : 1;   // weight column blocks per tile (gate, up)
  float(*As)[kFBM] = reinterpret_cast<float(*)[kFBM]>(smem);                       // [k][m]
  float(*Bs)[NB * kFBN] = reinterpret_cast<float(*)[NB * kFBN]>(smem + kFBK * kFBM);  // [k][n]
  const int tid = threadIdx.x;
  const int ty = tid >> 4, tx = tid & 15;
  const int e = p.tiles.expert[mtile];
  const int row0 = p.tiles.row0[mtile];
  const int rows = p.tiles.rows[mtile];
  if (rows <= 0) return;   // the empty half of a pair slot (block-uniform)
  const int n0 = ntile * kFBN;

  const int a_r = tid >> 2, a_k = (tid & 3) * 4;
  const float* a_ptr = p.A + (size_t)(row0 + min(a_r, rows - 1)) * p.lda + a_k;
  const int b_k = tid >> 4, b_n = (tid & 15) * 4;
  const float* b_ptr = p.B + (size_t)e * p.strideB + (size_t)b_k * p.ldb + n0 + b_n;

  float acc[NB][4][4];
#pragma unroll
  for (int h = 0; h < NB; ++h)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[h][i][j] = 0.f;

  for (int k0 = 0; k0 < p.K; k0 += kFBK) {
    float4 av = *reinterpret_cast<const float4*>(a_ptr + k0);
    float4 bv[NB];
#pragma unroll
    for (int h = 0; h < NB; ++h)
      bv[h] = *reinterpret_cast<const float4*>(b_ptr + (size_t)k0 * p.ldb + h * p.N);
    __syncthreads();   // previous step's reads are done
    As[a_k + 0][a_r] = av.x; As[a_k + 1][a_r] = av.y; As[a_k + 2][a_r] = av.z; As[a_k + 3][a_r] = av.w;
#pragma unroll
    for (int h = 0; h < NB; ++h) *reinterpret_cast<float4*>(&Bs[b_k][h * kFBN + b_n]) = bv[h];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kFBK; ++k) {
      float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
      const float ar[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
      for (int h = 0; h < NB; ++h) {
        float4 b = *reinterpret_cast<const float4*>(&Bs[k][h * kFBN + tx * 4]);
        const float br[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[h][i][j] = fmaf(ar[i], br[j], acc[h][i][j]);
      }
    }
  }
  __syncthreads();   // LDS free for the next tile

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = ty * 4 + i;
    if (m >= rows) continue;
    const size_t grow = (size_t)(row0 + m);
    const int c = n0 + tx * 4;
    if (EPI == kEpiSwiglu) {
      float a[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) a[j] = acc[0][i][j] * sigmoidf_(acc[0][i][j]) * acc[NB - 1][i][j];
      *reinterpret_cast<float4*>(p.C + grow * p.ldc + c) = make_float4(a[0], a[1], a[2], a[3]);
      if (p.C2) {
        float* h = p.C2 + grow * (size_t)(2 * p.N);
        *reinterpret_cast<float4*>(h + c) = make_float4(acc[0][i][0], acc[0][i][1], acc[0][i][2], acc[0][i][3]);
        *reinterpret_cast<float4*>(h + p.N + c) =
            make_float4(acc[NB - 1][i][0], acc[NB - 1][i][1], acc[NB - 1][i][2], acc[NB - 1][i][3]);
      }
    } else {
      *reinterpret_cast<float4*>(p.C + grow * p.ldc + c) = make_float4(acc[0][i][0], acc[0][i][1], acc[0][i][2], acc[0][i][3]);
    }
  }
}

template <int EPI>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(GemmParamsF32 p) {
  __shared__ __attribute__((aligned(16))) float smem[kFBK * kFBM + kFBK * 2 * kFBN];
  const int total = p.tiles.meta[kMetaMTiles] * p.n_ntiles;
  const int G = gridDim.x;
  for (int it = 0; it * G < total; ++it) {
    const int tile = xcd_tile_id(it, blockIdx.x, G);
    if (tile >= total) continue;
    gemm_tile_f32<EPI>(p, tile / p.n_ntiles, tile % p.n_ntiles, smem);
  }
}

}  // namespace moe
