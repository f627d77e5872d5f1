// Grouped bf16 GEMM on gfx950 MFMA (paper Section 2.2: GMM-1 gate/up projections
// with the SwiGLU activation, GMM-2 down projection).
//
// One workgroup (256 threads = 4 waves, 2x2) computes a 256 x 256 tile of
// C[rows_e, N] = A[rows_e, K] * W_e[K, N] with v_mfma_f32_32x32x16_bf16, fp32
// accumulation, K never split (Section 4.2: reduction dimensions stay intact).
// Rows come from the M-tile map built by the routing scan, so a tile never
// crosses an expert boundary.
//
// Data path per K step of 64:
//   global -> registers (prefetch of step s+1 while step s computes)
//   registers -> LDS, both operands stored k-contiguous, 16-byte chunks XOR-swizzled
//     * activations are already k-contiguous: straight copy
//     * weights are n-contiguous in memory ([K, N] row-major): each thread loads
//       an 8(k) x 8(n) block and transposes it in registers (32 permutes) so the
//       MFMA operand fetch is one ds_read_b128 per lane
//   LDS -> MFMA operands; two LDS stages, one barrier per K step.
// The MFMA is issued as D^T = W^T-fragment x X-fragment so that a lane ends up
// with 4 consecutive output columns of one row (8-byte bf16 stores).
//
// SwiGLU epilogue: the tile's 256 weight columns are 128 gate columns and the 128
// matching up columns, placed so each wave owns both halves of its columns and
// applies A = g*sigmoid(g)*u to the fp32 accumulators in registers.
#pragma once
#include "common.h"

namespace moe {

enum GemmEpilogue { kEpiStore = 0, kEpiSwiglu = 1 };

constexpr int kBM = 256;   // tile rows
constexpr int kBN = 256;   // weight columns staged per tile
constexpr int kBK = 64;    // K step
constexpr int kGemmThreads = 256;
// LDS stage of one operand: 256 rows of 64 bf16 (128 B) padded to 144 B, plus 16 B
// more per group of 8 rows.  All addresses are affine (thread base + immediates).
constexpr int kLdsRow = kBK * 2 + 16;
constexpr int kLdsGroup = 8 * kLdsRow + 16;             // 8 rows
constexpr int kStageBytes = (kBM / 8) * kLdsGroup;      // 37376 B per operand per stage
constexpr int kGemmLdsBytes = 4 * kStageBytes;          // A0 A1 B0 B1 = 146 KB

struct GemmParams {
  const __bf16* A;    // [rows, lda] activations, expert-contiguous rows, k-contiguous
  const __bf16* B;    // per expert [K, ldb] row-major weights
  __bf16* C;          // [rows, ldc]
  __bf16* C2;         // SwiGLU only: optional pre-activation [rows, 2N] (gate|up), else null
  long strideB;       // elements between consecutive experts' weights
  int K, N;           // N = output columns (SwiGLU: I, weights have 2N columns)
  int lda, ldb, ldc;
  int n_ntiles;       // ceil(N / 256) (SwiGLU: ceil(N / 128))
  TileMap tiles;
};

// Byte offset of 16-byte chunk `chunk` (0..7) of LDS row `row`.  Padding instead of
// an XOR swizzle: 8 consecutive rows at one chunk fall in 8 distinct 16-byte bank
// groups (operand fetch), and so do rows 8 apart (the transposed weight store).
__device__ __forceinline__ int lds_off(int row, int chunk) {
  return (row >> 3) * kLdsGroup + (row & 7) * kLdsRow + chunk * 16;
}

// Global -> register prefetch of one K step: 8 x 16 bytes of each operand per thread.
__device__ __forceinline__ void gemm_load_global(u32x4 (&ra)[8], u32x4 (&rb)[8], const __bf16* a_base,
                                                 const uint32_t (&a_off)[8], const __bf16* b_base, uint32_t b_off,
                                                 int ldb, int k0) {
  const __bf16* a_k = a_base + k0;                  // wave-uniform parts stay in scalar registers
#pragma unroll
  for (int i = 0; i < 8; ++i) ra[i] = *reinterpret_cast<const u32x4*>(a_k + a_off[i]);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const __bf16* b_k = b_base + (size_t)(k0 + i) * ldb;
    rb[i] = *reinterpret_cast<const u32x4*>(b_k + b_off);
  }
}

// Registers -> LDS stage.  Activations: straight copy.  Weights: the thread's
// 8(k) x 8(n) block is transposed so each column becomes one k-contiguous chunk.
__device__ __forceinline__ void gemm_store_lds(char* As, char* Bs, const u32x4 (&ra)[8], const u32x4 (&rb)[8],
                                               int ar, int ac, int bn, int bk) {
#pragma unroll
  for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(As + lds_off(ar + 32 * i, ac)) = ra[i];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    uint32_t o[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const uint32_t lo = rb[2 * m][j >> 1], hi = rb[2 * m + 1][j >> 1];
      o[m] = (j & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
    }
    *reinterpret_cast<u32x4*>(Bs + lds_off(bn + j, bk)) = u32x4{o[0], o[1], o[2], o[3]};
  }
}

// One K step (64) of MFMA work for a wave's 128 x 128 block from an LDS stage.
template <int EPI>
__device__ __forceinline__ void gemm_compute_stage(f32x16 (&acc)[4][4], const char* As, const char* Bs, int wm,
                                                   int wn, int l32, int lh) {
#pragma unroll
  for (int ks = 0; ks < kBK / 16; ++ks) {
    const int chunk = ks * 2 + lh;
    bf16x8 af[4], bfr[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
      af[mt] = *reinterpret_cast<const bf16x8*>(As + lds_off(wm * 128 + mt * 32 + l32, chunk));
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      // LDS row of weight sub-tile nt: SwiGLU keeps gate rows 0..127 and up rows 128..255
      const int brow = (EPI == kEpiSwiglu) ? ((nt >> 1) * (kBN / 2) + wn * 64 + (nt & 1) * 32) : (wn * 128 + nt * 32);
      bfr[nt] = *reinterpret_cast<const bf16x8*>(Bs + lds_off(brow + l32, chunk));
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[nt], af[mt], acc[mt][nt], 0, 0, 0);
  }
}

template <int EPI>
__device__ __forceinline__ void gemm_tile_bf16(const GemmParams& p, int mtile, int ntile, char* smem) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  const int e = p.tiles.expert[mtile];
  const int row0 = p.tiles.row0[mtile];
  const int rows = p.tiles.rows[mtile];

  // ---- global load mapping ----
  // A: thread -> chunk ac (8 k) of rows ar + 32*i; uniform tile base + 32-bit lane offsets
  const int ac = tid & 7, ar = tid >> 3;
  const __bf16* a_base = p.A + (size_t)row0 * p.lda;
  uint32_t a_off[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int r = min(ar + 32 * i, rows - 1);   // rows past the tile end re-read its last row; never stored
    a_off[i] = (uint32_t)(r * p.lda + ac * 8);
  }
  // B: thread -> 8 columns starting at LDS row bn, k rows bk*8 .. bk*8+7
  const int bn = (tid & 31) * 8, bk = tid >> 5;
  int gcol;
  if (EPI == kEpiSwiglu) {
    int c = min(ntile * (kBN / 2) + (bn & (kBN / 2 - 1)), p.N - 8);
    gcol = (bn >= kBN / 2) ? p.N + c : c;
  } else {
    gcol = min(ntile * kBN + bn, p.N - 8);
  }
  const __bf16* b_base = p.B + (size_t)e * p.strideB;
  const uint32_t b_off = (uint32_t)(bk * 8 * p.ldb + gcol);

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Two LDS stages; stage s&1 is written at the top of step s, one barrier per step:
  // a wave can only reach the write of step s+2 after every wave left compute(s).
  u32x4 ra[8], rb[8];
  const int n_steps = p.K / kBK;
  gemm_load_global(ra, rb, a_base, a_off, b_base, b_off, p.ldb, 0);
  for (int s = 0; s < n_steps - 1; ++s) {
    char* As = smem + (s & 1) * kStageBytes;
    char* Bs = smem + 2 * kStageBytes + (s & 1) * kStageBytes;
    gemm_store_lds(As, Bs, ra, rb, ar, ac, bn, bk);
    __syncthreads();
    gemm_load_global(ra, rb, a_base, a_off, b_base, b_off, p.ldb, (s + 1) * kBK);
    gemm_compute_stage<EPI>(acc, As, Bs, wm, wn, l32, lh);
  }
  {
    const int s = n_steps - 1;
    char* As = smem + (s & 1) * kStageBytes;
    char* Bs = smem + 2 * kStageBytes + (s & 1) * kStageBytes;
    gemm_store_lds(As, Bs, ra, rb, ar, ac, bn, bk);
    __syncthreads();
    gemm_compute_stage<EPI>(acc, As, Bs, wm, wn, l32, lh);
  }
  __syncthreads();   // both stages free before the next tile's first write

  // ---- epilogue: lane holds row m = l32 of each 32x32 block and, per register
  // group q, the 4 consecutive columns q*8 + lh*4 .. +3 ----
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    const int m = wm * 128 + mt * 32 + l32;
    if (m >= rows) continue;
    const size_t grow = (size_t)(row0 + m);
    if (EPI == kEpiSwiglu) {
#pragma unroll
      for (int ng = 0; ng < 2; ++ng)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = ntile * (kBN / 2) + wn * 64 + ng * 32 + q * 8 + lh * 4;
          if (c >= p.N) continue;
          float g[4], u[4], a[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            g[x] = acc[mt][ng][q * 4 + x];
            u[x] = acc[mt][ng + 2][q * 4 + x];
            a[x] = g[x] * sigmoidf_(g[x]) * u[x];
          }
          *reinterpret_cast<u32x2*>(p.C + grow * p.ldc + c) = u32x2{pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3])};
          if (p.C2) {
            __bf16* h = p.C2 + grow * (size_t)(2 * p.N);
            *reinterpret_cast<u32x2*>(h + c) = u32x2{pack_bf16(g[0], g[1]), pack_bf16(g[2], g[3])};
            *reinterpret_cast<u32x2*>(h + p.N + c) = u32x2{pack_bf16(u[0], u[1]), pack_bf16(u[2], u[3])};
          }
        }
    } else {
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = ntile * kBN + wn * 128 + nt * 32 + q * 8 + lh * 4;
          if (c >= p.N) continue;
          *reinterpret_cast<u32x2*>(p.C + grow * p.ldc + c) =
              u32x2{pack_bf16(acc[mt][nt][q * 4 + 0], acc[mt][nt][q * 4 + 1]),
                    pack_bf16(acc[mt][nt][q * 4 + 2], acc[mt][nt][q * 4 + 3])};
        }
    }
  }
}

// Tile id for workgroup b in sweep `it` of a grid of G workgroups (G % 8 == 0).
// Workgroups are dealt to the 8 XCDs round-robin by id, so giving XCD x the
// contiguous ids [x*G/8, (x+1)*G/8) keeps tiles that share an operand panel
// (same M tile, neighbouring N tiles) behind the same L2.
__device__ __forceinline__ int xcd_tile_id(int it, int b, int G) {
  return it * G + (b & 7) * (G >> 3) + (b >> 3);
}

template <int EPI>
__global__ __launch_bounds__(kGemmThreads) void grouped_gemm_bf16_kernel(GemmParams p) {
  __shared__ __attribute__((aligned(16))) char smem[kGemmLdsBytes];
  const int total = p.tiles.meta[kMetaMTiles] * p.n_ntiles;
  const int G = gridDim.x;
  for (int it = 0; it * G < total; ++it) {
    const int tile = xcd_tile_id(it, blockIdx.x, G);
    if (tile >= total) continue;
    gemm_tile_bf16<EPI>(p, tile / p.n_ntiles, tile % p.n_ntiles, smem);
  }
}

}  // namespace moe
