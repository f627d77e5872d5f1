// Backward-only operators (paper Section 2.2, Figure 2b): backward Dispatch (the
// gradient of the forward Combine) and the fp32 versions of the four backward
// GEMMs.  The bf16 GEMMs are the NT / TN layouts of gemm_bf16.h; backward Combine
// (the gradient of the forward Dispatch) is combine_token with unit weights.
#pragma once
#include "common.h"
#include "gemm_f32.h"
#include "route.h"

namespace moe {

struct BwdDispatchParams {
  const void* dY;          // [T,H]
  const void* Yp;          // [R_max,H] saved GEMM-2 output
  void* dYp;               // [R_max,H]
  const int32_t* row_of;   // [T,k]
  const float* topk_w;     // [T,k]
  float* d_topk_w;         // [T,k]
  int T, H, k;
  // The backward's M-tile map, rebuilt from the saved rows per expert, and the counters the later kernels draw
  // tickets from: nothing in this kernel needs them, so its last workgroup makes them on the side (one wave).
  const int32_t* counts;   // [E_local]
  int E_local, wide_max, granule, tall;
  TileMap tiles;
  uint32_t* zero;
  int n_zero;
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// One wave per token t: for every local slot j with row r = row_of[t,j]
//   dYp[r,:] = topk_w[t,j] * dY[t,:],   d_topk_w[t,j] = <dY[t,:], Yp[r,:]>  (fp32),
// and d_topk_w[t,j] = 0 for slots whose expert is not local.
// Lane j < k holds slot j; the local slots are walked through the ballot of "row >= 0" with rows and
// weights as wave-uniform scalars.  A pass covers 7 x 64 16-byte vectors of the row: dY[t] is fetched
// once per pass and reused by every local slot, the Yp vectors of a slot are all in flight together.
template <bool BF16>
__device__ __forceinline__ void bwd_dispatch_token(const BwdDispatchParams& p, int t) {
  const int lane = lane_id();
  int rowv = -1;
  float wv = 0.f;
  if (lane < p.k) {
    rowv = p.row_of[(size_t)t * p.k + lane];
    wv = p.topk_w[(size_t)t * p.k + lane];
    if (rowv < 0) p.d_topk_w[(size_t)t * p.k + lane] = 0.f;
  }
  const uint64_t local = __ballot(rowv >= 0);
  if (local == 0) return;
  constexpr int EPV = BF16 ? 8 : 4;                 // elements per 16-byte vector
  constexpr int U = BF16 ? 7 : 4;                   // vectors per lane per pass
  const int vec = p.H / EPV;
  const size_t row_bytes = (size_t)p.H * (BF16 ? 2 : 4);
  const uint4* dy = reinterpret_cast<const uint4*>(static_cast<const char*>(p.dY) + (size_t)t * row_bytes);
  float dot[kMaxK];
#pragma unroll
  for (int n = 0; n < kMaxK; ++n) dot[n] = 0.f;
  for (int v0 = lane; v0 < vec; v0 += U * kWave) {
    uint4 a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = v0 + u * kWave < vec ? dy[v0 + u * kWave] : make_uint4(0, 0, 0, 0);
    uint64_t m = local;
#pragma unroll
    for (int n = 0; n < kMaxK; ++n) {
      if (m == 0) break;
      const int j = __builtin_amdgcn_readfirstlane(__builtin_ctzll(m));
      m &= m - 1;
      const int r = __builtin_amdgcn_readlane(rowv, j);
      const float w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv), j));
      const uint4* yp = reinterpret_cast<const uint4*>(static_cast<const char*>(p.Yp) + (size_t)r * row_bytes);
      uint4* o = reinterpret_cast<uint4*>(static_cast<char*>(p.dYp) + (size_t)r * row_bytes);
      uint4 b[U];
#pragma unroll
      for (int u = 0; u < U; ++u) b[u] = v0 + u * kWave < vec ? yp[v0 + u * kWave] : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (v0 + u * kWave >= vec) break;
        const uint32_t aw[4] = {a[u].x, a[u].y, a[u].z, a[u].w};
        const uint32_t bw[4] = {b[u].x, b[u].y, b[u].z, b[u].w};
        uint32_t ow[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          if constexpr (BF16) {
            const float lo = bf16_lo(aw[x]), hi = bf16_hi(aw[x]);
            dot[n] = fmaf(lo, bf16_lo(bw[x]), dot[n]);
            dot[n] = fmaf(hi, bf16_hi(bw[x]), dot[n]);
            ow[x] = pack_bf16(w * lo, w * hi);
          } else {
            const float av = __builtin_bit_cast(float, aw[x]);
            dot[n] = fmaf(av, __builtin_bit_cast(float, bw[x]), dot[n]);
            ow[x] = __builtin_bit_cast(uint32_t, w * av);
          }
        }
        o[v0 + u * kWave] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
      }
    }
  }
  uint64_t m = local;
#pragma unroll
  for (int n = 0; n < kMaxK; ++n) {
    if (m == 0) break;
    const int j = __builtin_amdgcn_readfirstlane(__builtin_ctzll(m));
    m &= m - 1;
    const float d = wave_sum(dot[n]);
    if (lane == 0) p.d_topk_w[(size_t)t * p.k + j] = d;
  }
}

template <bool BF16>
__global__ __launch_bounds__(256) void bwd_dispatch_kernel(BwdDispatchParams p) {
  const int n_waves = blockDim.x / kWave;
  const int wave = threadIdx.x / kWave;
  const int n_blocks = (int)gridDim.x - 1;
  if ((int)blockIdx.x == n_blocks) {
    if (wave == 0) {
      for (int i = threadIdx.x; i < p.n_zero; i += kWave) p.zero[i] = 0;
      build_tile_map(p.E_local, p.counts, p.wide_max, p.granule, p.tall, nullptr, nullptr, p.tiles);
    }
    return;
  }
  for (int t = blockIdx.x * n_waves + wave; t < p.T; t += n_blocks * n_waves) bwd_dispatch_token<BF16>(p, t);
}

// ---- fp32 backward GEMMs: one 64 x 64 x 16 LDS-tiled kernel with element strides,
// every bound checked, K zero-padded.  Exactness path, not a throughput path. ----
struct GemmBwdParamsF32 {
  const float* A;     // dgrad: [rows, lda]; wgrad: [rows, lda] read transposed
  const float* B;     // dgrad: per expert [N, ldb] (weights, read transposed); wgrad: [rows, ldb]
  float* C;           // dgrad: [rows, ldc]; wgrad: per expert [M, ldc]
  const float* G;     // SwiGLU-grad: saved pre-activations [rows, 2N]
  long strideB, strideC;
  int K, N, M;
  int lda, ldb, ldc;
  int n_ntiles, n_mtiles, E_local;
  const int32_t* offsets;
  TileMap tiles;
};

// acc[i][j] += sum_k A(m0 + ty*4 + i, k) * B(k, n0 + tx*4 + j); A(m,k) = A[m*sam + k*sak], B(k,n) = B[k*sbk + n*sbn];
// m < M, n < N, k < K else 0.
__device__ __forceinline__ void gemm_tile_f32_strided(const float* A, long sam, long sak, const float* B, long sbk,
                                                      long sbn, int M, int N, int K, float* smem,
                                                      float (&acc)[4][4]) {
  float(*As)[kFBM] = reinterpret_cast<float(*)[kFBM]>(smem);                  // [k][m]
  float(*Bs)[kFBN] = reinterpret_cast<float(*)[kFBN]>(smem + kFBK * kFBM);    // [k][n]
  const int tid = threadIdx.x;
  const int ty = tid >> 4, tx = tid & 15;
  for (int k0 = 0; k0 < K; k0 += kFBK) {
    float av[4], bv[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int idx = tid + q * 256;              // 1024 elements of each 64 x 16 operand tile
      const int k = idx & 15, x = idx >> 4;       // x = m (A) or n (B)
      av[q] = (x < M && k0 + k < K) ? A[(long)x * sam + (long)(k0 + k) * sak] : 0.f;
      bv[q] = (x < N && k0 + k < K) ? B[(long)(k0 + k) * sbk + (long)x * sbn] : 0.f;
    }
    __syncthreads();   // previous step's reads are done
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int idx = tid + q * 256;
      As[idx & 15][idx >> 4] = av[q];
      Bs[idx & 15][idx >> 4] = bv[q];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kFBK; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
      const float ar[4] = {a.x, a.y, a.z, a.w};
      const float br[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(ar[i], br[j], acc[i][j]);
    }
  }
  __syncthreads();   // LDS free for the next tile
}

// act_grad (+ SwiGLU_grad) and gate_grad: C[rows, N] = A[rows, K] * W_e[N, K]^T per M tile.
template <int EPI>
__global__ __launch_bounds__(256) void grouped_dgrad_f32_kernel(GemmBwdParamsF32 p) {
  __shared__ __attribute__((aligned(16))) float smem[kFBK * kFBM + kFBK * kFBN];
  const int total = p.tiles.meta[kMetaMTiles] * p.n_ntiles;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
    const int mtile = tile / p.n_ntiles, n0 = (tile % p.n_ntiles) * kFBN;
    const int e = p.tiles.expert[mtile], row0 = p.tiles.row0[mtile], rows = p.tiles.rows[mtile];
    if (rows <= 0) continue;   // the empty half of a pair slot (block-uniform)
    float acc[4][4] = {};
    gemm_tile_f32_strided(p.A + (size_t)row0 * p.lda, p.lda, 1, p.B + (size_t)e * p.strideB + (size_t)n0 * p.ldb, 1,
                          p.ldb, rows, p.N - n0, p.K, smem, acc);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = ty * 4 + i;
      if (m >= rows) continue;
      const size_t grow = (size_t)(row0 + m);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = n0 + tx * 4 + j;
        if (c >= p.N) continue;
        if (EPI == kEpiSwigluGrad) {
          const float g = p.G[grow * (size_t)(2 * p.N) + c], u = p.G[grow * (size_t)(2 * p.N) + p.N + c];
          const float s = sigmoidf_(g), da = acc[i][j];
          p.C[grow * p.ldc + c] = da * u * s * (1.f + g * (1.f - s));
          p.C[grow * p.ldc + p.N + c] = da * g * s;
        } else {
          p.C[grow * p.ldc + c] = acc[i][j];
        }
      }
    }
  }
}

// w2_grad and w1_grad: C_e[M, N] = A_e[rows_e, M]^T * B_e[rows_e, N]; zeros for experts without rows.
__global__ __launch_bounds__(256) void grouped_wgrad_f32_kernel(GemmBwdParamsF32 p) {
  __shared__ __attribute__((aligned(16))) float smem[kFBK * kFBM + kFBK * kFBN];
  const int per_e = p.n_mtiles * p.n_ntiles;
  const int total = p.E_local * per_e;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
    const int e = tile / per_e, rem = tile % per_e;
    const int m0 = (rem / p.n_ntiles) * kFBM, n0 = (rem % p.n_ntiles) * kFBN;
    const int seg0 = p.offsets[e], cnt = p.offsets[e + 1] - seg0;
    float acc[4][4] = {};
    gemm_tile_f32_strided(p.A + (size_t)seg0 * p.lda + m0, 1, p.lda, p.B + (size_t)seg0 * p.ldb + n0, p.ldb, 1,
                          p.M - m0, p.N - n0, cnt, smem, acc);
    float* c_base = p.C + (size_t)e * p.strideC;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int m = m0 + ty * 4 + i, c = n0 + tx * 4 + j;
        if (m < p.M && c < p.N) c_base[(size_t)m * p.ldc + c] = acc[i][j];
      }
  }
}

}  // namespace moe
