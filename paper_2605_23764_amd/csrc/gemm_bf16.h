// Grouped bf16 GEMM on gfx950 MFMA (paper Section 2.2: GMM-1 gate/up projections
// with the SwiGLU activation, GMM-2 down projection).
//
// One workgroup (256 threads = 4 waves, 2 x 2) computes a tile of up to 512 rows x
// 128 weight columns of C[rows_e, N] = A[rows_e, K] * W_e[K, N] with
// v_mfma_f32_32x32x16_bf16, fp32 accumulation, K never split (Section 4.2:
// reduction dimensions stay intact).  Rows come from the M-tile map built by the
// routing scan, so a tile never crosses an expert boundary and an expert with up
// to 512 rows streams each weight element from HBM exactly once.  The two wave
// rows split the tile's rows evenly in units of 32, so MFMA work follows the real
// row count instead of the tile capacity.
//
// Data path per K step of 32, three LDS stages (one computing, two in flight):
//   * global -> LDS directly (global_load_lds_dwordx4: 64 lanes x 16 B land in
//     1 KB of consecutive LDS, no registers involved).  Which global chunk a lane
//     fetches is chosen so that the later operand reads are bank-conflict free.
//   * activations (k-contiguous): a 1 KB line holds 16 rows x 32 k, chunk-major;
//     operand fetch is one ds_read_b128 per lane.
//   * weights ([K, N] row-major, n-contiguous): a 1 KB line holds 4 k-rows x 128 n,
//     each k-row rotated by 64 B; the k-contiguous MFMA operand is fetched with
//     the LDS transpose read ds_read_b64_tr_b16 (two per operand).
//   * s_waitcnt vmcnt(n) + one s_barrier per K step order the pipeline.
// The MFMA is issued as D^T = W^T-fragment x X-fragment so that a lane ends up
// with 4 consecutive output columns of one row (8-byte bf16 stores).
//
// SwiGLU epilogue: the tile's 128 weight columns are 64 gate columns and the 64
// matching up columns, placed so each wave owns both halves of its columns and
// applies A = g*sigmoid(g)*u to the fp32 accumulators in registers.
#pragma once
#include "common.h"

namespace moe {

enum GemmEpilogue { kEpiStore = 0, kEpiSwiglu = 1 };

#ifndef MOE_GEMM_BM
#define MOE_GEMM_BM 512
#endif
#ifndef MOE_GEMM_STAGES
#define MOE_GEMM_STAGES 3
#endif
constexpr int kBM = MOE_GEMM_BM;    // tile row capacity (one M tile of the tile map)
constexpr int kBN = 128;            // weight columns staged per tile
constexpr int kBK = 32;             // K step
constexpr int kStages = MOE_GEMM_STAGES;
constexpr int kGemmThreads = 256;
constexpr int kLine = 1024;                          // bytes moved by one wave-wide 16-byte load
constexpr int kALines = kBM / 16;                    // 16 rows x 32 k per line
constexpr int kBLines = kBK / 4;                     // 4 k-rows x 128 n per line
constexpr int kStageBytes = (kALines + kBLines) * kLine;   // 40 KB
constexpr int kGemmLdsBytes = kStages * kStageBytes;       // 120 KB
constexpr int kMaxMT = kBM / 64;                     // 32-row MFMA sub-tiles per wave row (8)

struct GemmParams {
  const __bf16* A;    // [rows, lda] activations, expert-contiguous rows, k-contiguous
  const __bf16* B;    // per expert [K, ldb] row-major weights
  __bf16* C;          // [rows, ldc]
  __bf16* C2;         // SwiGLU only: optional pre-activation [rows, 2N] (gate|up), else null
  long strideB;       // elements between consecutive experts' weights
  int K, N;           // N = output columns (SwiGLU: I, weights have 2N columns)
  int lda, ldb, ldc;
  int n_ntiles;       // ceil(N / 128) (SwiGLU: N / 64)
  TileMap tiles;
};

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

// s_waitcnt vmcnt(n) only (expcnt/lgkmcnt left at "don't wait"); n is wave-uniform, 0..63.
// The count is an instruction immediate, so a runtime n goes through a jump table.
__device__ __forceinline__ void wait_vmcnt(int n) {
#define MOE_WAIT_CASE(i) case i: __builtin_amdgcn_s_waitcnt(0x0F70 | ((i) & 15) | (((i) >> 4) << 14)); break;
#define MOE_WAIT_CASE8(b) MOE_WAIT_CASE(b) MOE_WAIT_CASE(b + 1) MOE_WAIT_CASE(b + 2) MOE_WAIT_CASE(b + 3) \
                          MOE_WAIT_CASE(b + 4) MOE_WAIT_CASE(b + 5) MOE_WAIT_CASE(b + 6) MOE_WAIT_CASE(b + 7)
  switch (n) {
    MOE_WAIT_CASE(1) MOE_WAIT_CASE(2) MOE_WAIT_CASE(3) MOE_WAIT_CASE(4) MOE_WAIT_CASE(5) MOE_WAIT_CASE(6) MOE_WAIT_CASE(7)
    MOE_WAIT_CASE8(8) MOE_WAIT_CASE8(16) MOE_WAIT_CASE8(24) MOE_WAIT_CASE8(32) MOE_WAIT_CASE8(40) MOE_WAIT_CASE8(48)
    MOE_WAIT_CASE8(56)
    default: __builtin_amdgcn_s_waitcnt(0x0F70); break;   // vmcnt(0)
  }
#undef MOE_WAIT_CASE8
#undef MOE_WAIT_CASE
}

// Per-tile, per-lane addressing state shared by the load and compute phases.
struct GemmTileCtx {
  const char* a_base;          // uniform: first row of the tile, byte address
  const char* b_base;          // uniform: expert's weights, byte address
  uint32_t a_off[kMaxMT];      // per lane: byte offset of the chunk this lane fetches for its i-th A line
  uint32_t b_off;              // per lane: byte offset inside a 4-row weight line
  int nA;                      // A lines per wave per step (1..8)
  int ldb_bytes;
  int wave;
};

// Issue the loads of K step `step` into LDS stage `stage`: nA + 2 wave-wide loads.
__device__ __forceinline__ void gemm_issue_loads(const GemmTileCtx& t, char* smem, int stage, int step) {
  char* st = smem + stage * kStageBytes;
  const char* a_k = t.a_base + (size_t)step * (kBK * 2);
#pragma unroll
  for (int i = 0; i < kMaxMT; ++i) {
    if (i < t.nA)
      __builtin_amdgcn_global_load_lds(a_k + t.a_off[i], (lds_void_ptr)(st + (t.wave + 4 * i) * kLine), 16, 0, 0);
  }
  const char* b_k = t.b_base + (size_t)(step * kBK + t.wave * 8) * t.ldb_bytes;
  char* bs = st + kALines * kLine + t.wave * 2 * kLine;
  __builtin_amdgcn_global_load_lds(b_k + t.b_off, (lds_void_ptr)bs, 16, 0, 0);
  __builtin_amdgcn_global_load_lds(b_k + (size_t)4 * t.ldb_bytes + t.b_off, (lds_void_ptr)(bs + kLine), 16, 0, 0);
}

// One K step (32) of MFMA work for a wave: NMT row sub-tiles x 2 column sub-tiles.
template <int NMT>
__device__ __forceinline__ void gemm_compute_stage(f32x16 (&acc)[kMaxMT][2], const char* st, uint32_t a_rd,
                                                   const uint32_t (&b_rd)[2]) {
  if (NMT == 0) return;
#pragma unroll
  for (int ks = 0; ks < kBK / 16; ++ks) {
    bf16x8 wf[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const char* bp = st + kALines * kLine + b_rd[nt] + ks * 4 * kLine;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(bp));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(bp + kLine));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      s16x8 both = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      wf[nt] = __builtin_bit_cast(bf16x8, both);
    }
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
      bf16x8 xf = *reinterpret_cast<const bf16x8*>(st + a_rd + mt * 2 * kLine + ks * 512);
      acc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[0], xf, acc[mt][0], 0, 0, 0);
      acc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1], xf, acc[mt][1], 0, 0, 0);
    }
  }
}

// K loop of one tile for a wave with NMT active row sub-tiles.  With S stages, at
// the top of step s the loads of steps s .. s+S-2 are outstanding; after the
// wait + barrier every wave's step-s data is in LDS and every wave has left
// compute(s-1), whose stage is then refilled with step s+S-1.
template <int NMT>
__device__ __forceinline__ void gemm_k_loop(f32x16 (&acc)[kMaxMT][2], const GemmTileCtx& t, char* smem, int n_steps,
                                            uint32_t a_rd, const uint32_t (&b_rd)[2]) {
  const int per_step = t.nA + 2;
#pragma unroll
  for (int i = 0; i < kStages - 1; ++i)
    if (i < n_steps) gemm_issue_loads(t, smem, i, i);
  int stage = 0;
  for (int s = 0; s < n_steps; ++s) {
    wait_vmcnt(min(kStages - 2, n_steps - 1 - s) * per_step);   // younger steps may stay in flight
    __builtin_amdgcn_s_barrier();
    if (s + kStages - 1 < n_steps) gemm_issue_loads(t, smem, stage == 0 ? kStages - 1 : stage - 1, s + kStages - 1);
#if !defined(MOE_DBG_NOCOMPUTE)
    gemm_compute_stage<NMT>(acc, smem + stage * kStageBytes, a_rd, b_rd);
#endif
    stage = stage == kStages - 1 ? 0 : stage + 1;
  }
  __builtin_amdgcn_s_barrier();   // all stages free before the next tile's first loads
}

template <int EPI>
__device__ __forceinline__ void gemm_tile_bf16(const GemmParams& p, int mtile, int ntile, char* smem) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps branches and LDS bases scalar
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  const int e = p.tiles.expert[mtile];
  const int row0 = p.tiles.row0[mtile];
  const int rows = p.tiles.rows[mtile];
  const int half = ((rows + 63) >> 6) << 5;                 // rows per wave row, multiple of 32
  const int my_rows = wm == 0 ? min(rows, half) : max(0, rows - half);
  const int n_mt = (my_rows + 31) >> 5;
  const int n_lines = ((rows + 31) >> 5) << 1;              // 16-row lines that any operand read touches

  GemmTileCtx t;
  t.wave = wave;
  t.nA = (n_lines + 3) >> 2;
  t.ldb_bytes = p.ldb * 2;
  t.a_base = reinterpret_cast<const char*>(p.A + (size_t)row0 * p.lda);
  t.b_base = reinterpret_cast<const char*>(p.B + (size_t)e * p.strideB);
  {
    // A line L = wave + 4*i holds rows 16L..16L+15; lane -> (chunk c = lane/16, row r = lane%16)
    const int c = lane >> 4, r = lane & 15;
#pragma unroll
    for (int i = 0; i < kMaxMT; ++i) {
      int row = min((wave + 4 * i) * 16 + r, rows - 1);     // rows past the end re-read the last row; never stored
      t.a_off[i] = (uint32_t)((row * p.lda + c * 8) * 2);
    }
    // B line: lane -> (k-row kk = lane/16, LDS chunk position pos = lane%16) holds weight chunk j = pos - 4*kk
    const int kk = lane >> 4, pos = lane & 15;
    const int nl = ((pos - 4 * kk) & 15) * 8;               // column inside the tile's 128
    int gcol;
    if (EPI == kEpiSwiglu) {
      gcol = (nl < kBN / 2) ? ntile * (kBN / 2) + nl : p.N + ntile * (kBN / 2) + (nl - kBN / 2);
    } else {
      gcol = min(ntile * kBN + nl, p.N - 8);
    }
    t.b_off = (uint32_t)((kk * p.ldb + gcol) * 2);
  }

  // operand read offsets inside a stage
  const uint32_t a_rd = (uint32_t)(((wm * half) >> 4) * kLine + (l32 >> 4) * kLine + lh * 256 + (l32 & 15) * 16);
  uint32_t b_rd[2];
  {
    const int g = lane >> 4, i = lane & 15;
    const int kk = i >> 2;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const int nbase = (EPI == kEpiSwiglu) ? nt * 64 + wn * 32 : wn * 64 + nt * 32;   // column block of 32 in the tile
      const int j = (nbase >> 3) + (g & 1) * 2 + ((i & 3) >> 1);
      b_rd[nt] = (uint32_t)((g >> 1) * 2 * kLine + kk * 256 + ((j + 4 * kk) & 15) * 16 + (i & 1) * 8);
    }
  }

  f32x16 acc[kMaxMT][2];
#pragma unroll
  for (int i = 0; i < kMaxMT; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int n_steps = p.K / kBK;
  switch (n_mt) {
    case 0: gemm_k_loop<0>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 1: gemm_k_loop<1>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 2: gemm_k_loop<2>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 3: gemm_k_loop<3>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 4: gemm_k_loop<4>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 5: gemm_k_loop<5>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 6: gemm_k_loop<6>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 7: gemm_k_loop<7>(acc, t, smem, n_steps, a_rd, b_rd); break;
    default: gemm_k_loop<8>(acc, t, smem, n_steps, a_rd, b_rd); break;
  }

  // ---- epilogue: lane holds row l32 of each 32 x 32 block and, per register group q,
  // the 4 consecutive columns q*8 + lh*4 .. +3 ----
#pragma unroll
  for (int mt = 0; mt < kMaxMT; ++mt) {
    const int m = wm * half + mt * 32 + l32;
    if (mt >= n_mt || m >= rows) continue;
    const size_t grow = (size_t)(row0 + m);
    if (EPI == kEpiSwiglu) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = ntile * (kBN / 2) + wn * 32 + q * 8 + lh * 4;
        float g[4], u[4], a[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          g[x] = acc[mt][0][q * 4 + x];
          u[x] = acc[mt][1][q * 4 + x];
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
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = ntile * kBN + wn * 64 + nt * 32 + q * 8 + lh * 4;
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
  __shared__ __attribute__((aligned(1024))) char smem[kGemmLdsBytes];
  const int total = p.tiles.meta[kMetaMTiles] * p.n_ntiles;
  const int G = gridDim.x;
  for (int it = 0; it * G < total; ++it) {
    const int tile = xcd_tile_id(it, blockIdx.x, G);
    if (tile >= total) continue;
    gemm_tile_bf16<EPI>(p, tile / p.n_ntiles, tile % p.n_ntiles, smem);
  }
}

}  // namespace moe
