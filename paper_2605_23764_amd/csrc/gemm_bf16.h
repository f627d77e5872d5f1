// Grouped bf16 GEMM on gfx950 MFMA (paper Section 2.2: GMM-1 gate/up projections
// with the SwiGLU activation, GMM-2 down projection).
//
// One workgroup (256 threads = 4 waves, 2 x 2, 128 x 128 per wave) computes a tile
// of up to 256 rows x 256 weight columns of C[rows_e, N] = A[rows_e, K] * W_e[K, N]
// with v_mfma_f32_32x32x16_bf16, fp32 accumulation, K never split (Section 4.2:
// reduction dimensions stay intact).  256 x 256 is the largest tile the register
// file holds and the only shape whose operand traffic (32 B/clk at MFMA peak) fits
// the ~40 B/clk a CU can pull through its vector memory path.  Rows come from the
// M-tile map built by the routing scan, so a tile never crosses an expert
// boundary; the two wave rows split the tile's rows in units of 32, so MFMA work
// follows the real row count.
//
// Data path per K step of 64:
//   * global -> LDS directly (global_load_lds_dwordx4: 64 lanes x 16 B land in
//     1 KB of consecutive LDS, no registers involved).  Lanes that are neighbours
//     fetch neighbouring addresses (full 128 B or 256 B segments per row: anything
//     less halves the load rate); WHICH chunk of its segment a lane fetches is
//     permuted so that the later operand reads are bank-conflict free.
//   * activations (k-contiguous): a 1 KB line holds 8 rows x 64 k, the eight 16 B
//     chunks of a row XOR-swizzled by (row/2)%8; operand fetch is one ds_read_b128.
//   * weights ([K, N] row-major, n-contiguous): a 1 KB line holds 4 k-rows x 128 n,
//     each k-row rotated by 64 B; the k-contiguous MFMA operand is fetched with
//     the LDS transpose read ds_read_b64_tr_b16 (two per operand).
//   * weights come from HBM (long latency): three LDS stages, two steps in flight;
//     activations come from L2: two stages.  160 KB of LDS in total.
//   * s_waitcnt vmcnt(n) + one s_barrier per K step order the pipeline.
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

constexpr int kBM = 256;            // tile row capacity (one M tile of the tile map)
constexpr int kBN = 256;            // weight columns staged per tile
constexpr int kBK = 64;             // K step
constexpr int kRowGranule = 32;     // M tiles of one expert are equal multiples of this
constexpr int kAStages = 2;
constexpr int kBStages = 3;
constexpr int kGemmThreads = 256;
constexpr int kLine = 1024;                          // bytes moved by one wave-wide 16-byte load
constexpr int kALines = kBM / 8;                     // 8 rows x 64 k per line (32)
constexpr int kBLines = (kBK / 4) * (kBN / 128);     // 4 k-rows x 128 n per line (32)
constexpr int kAStageBytes = kALines * kLine;        // 32 KB
constexpr int kBStageBytes = kBLines * kLine;        // 32 KB
constexpr int kBRegion = kAStages * kAStageBytes;    // weights stages start here
constexpr int kGemmLdsBytes = kBRegion + kBStages * kBStageBytes;   // 160 KB
constexpr int kMaxMT = kBM / 64;                     // 32-row MFMA sub-tiles per wave row (4)
constexpr int kBLinesPerWave = kBLines / 4;          // 8

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

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

// s_waitcnt vmcnt(n) only (expcnt/lgkmcnt left at "don't wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// One wave-wide global -> LDS copy: lane l moves 16 bytes from sbase + voff to LDS
// byte address lds_addr + 16*l.  Issued as inline assembly so that the compiler's
// own wait-count pass does not see an LDS write and force vmcnt(0) before every
// operand read (which would serialise the pipeline); ordering is done by hand with
// wait_vmcnt + s_barrier.  The "memory" clobber keeps LDS reads from moving across.
__device__ __forceinline__ void lds_dma16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(sbase)
               : "memory", "m0");
}

__device__ __forceinline__ uint32_t lds_addr_of(const char* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// Per-tile, per-lane addressing state shared by the load and compute phases.
struct GemmTileCtx {
  const char* a_base;          // uniform: first row of the tile, byte address
  const char* b_base;          // uniform: expert's weights, byte address
  uint32_t a_off[8];           // per lane: byte offset of the chunk this lane fetches for its i-th A line
  uint32_t b_off[2];           // per lane: byte offset inside a 4-row weight line, column halves 0 / 1
  int nA;                      // A lines per wave per step (1..8)
  int ldb_bytes;
  int wave;
};

// Quarter `part` (0..3) of the loads a K step issues: parts 0-1 fetch the
// activation lines of step `a_step` into A stage `a_stage` (nA wave-wide loads in
// all), parts 2-3 the weight lines of step `b_step` into B stage `b_stage` (8
// loads: this wave's 16 k-rows x both 128-column halves).  A negative step skips.
// Activation loads always precede weight loads, which the vmcnt waits rely on.
__device__ __forceinline__ void gemm_issue_part(const GemmTileCtx& t, uint32_t lds0, int part, int a_stage, int a_step,
                                                int b_stage, int b_step) {
  if (part < 2) {
    if (a_step < 0) return;
    const uint32_t st = lds0 + a_stage * kAStageBytes + t.wave * kLine;
    const char* a_k = t.a_base + (size_t)a_step * (kBK * 2);
#pragma unroll
    for (int i = part * 4; i < part * 4 + 4; ++i)
      if (i < t.nA) lds_dma16(a_k, t.a_off[i], st + 4 * i * kLine);
  } else {
    if (b_step < 0) return;
    const uint32_t st = lds0 + kBRegion + b_stage * kBStageBytes + t.wave * kBLinesPerWave * kLine;
    const char* b_k = t.b_base + (size_t)(b_step * kBK + t.wave * 16) * t.ldb_bytes;
#pragma unroll
    for (int i = (part - 2) * 4; i < (part - 2) * 4 + 4; ++i)
      lds_dma16(b_k + (size_t)((i >> 1) * 4) * t.ldb_bytes, t.b_off[i & 1], st + i * kLine);
  }
}

// MFMA operands of one 16-wide k slice: 4 weight fragments (transpose reads) and
// NMT activation fragments.
template <int NMT>
struct GemmFrags {
  bf16x8 wf[4];
  bf16x8 xf[NMT > 0 ? NMT : 1];
};

template <int NMT>
__device__ __forceinline__ void gemm_load_frags(GemmFrags<NMT>& f, const char* as, const char* bs, int ks,
                                                const uint32_t (&a_rd)[4], const uint32_t (&b_rd)[4]) {
#pragma unroll
  for (int nt = 0; nt < 4; ++nt) {
    const char* bp = bs + b_rd[nt] + ks * 8 * kLine;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(bp));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(bp + 2 * kLine));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    s16x8 both = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    f.wf[nt] = __builtin_bit_cast(bf16x8, both);
  }
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt)
    f.xf[mt] = *reinterpret_cast<const bf16x8*>(as + a_rd[ks] + mt * 4 * kLine);
}

// One K step (64) for a wave: NMT x 4 MFMAs per 16-wide k slice.  The operand
// reads of slice ks+1 and a quarter of the step's global->LDS loads are issued
// before the MFMAs of slice ks, so LDS latency and load issue hide under MFMA time.
template <int NMT>
__device__ __forceinline__ void gemm_step(f32x16 (&acc)[kMaxMT][4], const GemmTileCtx& t, uint32_t lds0, const char* as,
                                          const char* bs, const uint32_t (&a_rd)[4], const uint32_t (&b_rd)[4],
                                          int a_stage, int a_step, int b_stage, int b_step) {
  GemmFrags<NMT> cur, nxt;
  if (NMT > 0) gemm_load_frags<NMT>(cur, as, bs, 0, a_rd, b_rd);
#pragma unroll
  for (int ks = 0; ks < kBK / 16; ++ks) {
    if (NMT > 0 && ks + 1 < kBK / 16) gemm_load_frags<NMT>(nxt, as, bs, ks + 1, a_rd, b_rd);
    gemm_issue_part(t, lds0, ks, a_stage, a_step, b_stage, b_step);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.wf[nt], cur.xf[mt], acc[mt][nt], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (ks + 1 < kBK / 16) cur = nxt;
  }
}

// K loop of one tile for a wave with NMT active row sub-tiles.
// Issue order is A(s+1) then B(s+2) during step s, so at the top of step s+1 the
// only loads allowed to be outstanding are the 8 of B(s+2).  After the wait +
// barrier every wave's A(s) and B(s) are in LDS and every wave has left step s-1,
// whose A stage and B stage are refilled during step s.
template <int NMT>
__device__ __forceinline__ void gemm_k_loop(f32x16 (&acc)[kMaxMT][4], const GemmTileCtx& t, char* smem, int n_steps,
                                            const uint32_t (&a_rd)[4], const uint32_t (&b_rd)[4]) {
  const uint32_t lds0 = lds_addr_of(smem);
#pragma unroll
  for (int part = 0; part < 4; ++part) gemm_issue_part(t, lds0, part, 0, 0, 0, 0);            // A(0), B(0)
  if (n_steps > 1) {
    gemm_issue_part(t, lds0, 2, 0, -1, 1, 1);                                                  // B(1)
    gemm_issue_part(t, lds0, 3, 0, -1, 1, 1);
  }
  int bstage = 0;
  for (int s = 0; s < n_steps; ++s) {
    if (s + 1 < n_steps) wait_vmcnt<kBLinesPerWave>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    gemm_step<NMT>(acc, t, lds0, smem + (s & 1) * kAStageBytes, smem + kBRegion + bstage * kBStageBytes, a_rd, b_rd,
                   (s + 1) & 1, s + 1 < n_steps ? s + 1 : -1, bstage == 0 ? 2 : bstage - 1, s + 2 < n_steps ? s + 2 : -1);
    bstage = bstage == kBStages - 1 ? 0 : bstage + 1;
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

  GemmTileCtx t;
  t.wave = wave;
  t.nA = (rows + 31) >> 5;            // (8-row lines any operand read touches = 4*ceil(rows/32)) / 4 waves
  t.ldb_bytes = p.ldb * 2;
  t.a_base = reinterpret_cast<const char*>(p.A + (size_t)row0 * p.lda);
  t.b_base = reinterpret_cast<const char*>(p.B + (size_t)e * p.strideB);
  {
    // A line L = wave + 4*i holds rows 8L..8L+7; lane -> (row r = lane/8, LDS chunk position pos = lane%8),
    // which holds k chunk pos ^ ((row/2)%8)
    const int r = lane >> 3, pos = lane & 7;
    const int c = pos ^ ((4 * (wave & 1) + (r >> 1)) & 7);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int row = min((wave + 4 * i) * 8 + r, rows - 1);      // rows past the end re-read the last row; never stored
      t.a_off[i] = (uint32_t)((row * p.lda + c * 8) * 2);
    }
    // B line: lane -> (k-row kk = lane/16, LDS chunk position pos = lane%16) holds weight chunk j = pos - 4*kk
    const int kk = lane >> 4, bpos = lane & 15;
    const int nl = ((bpos - 4 * kk) & 15) * 8;              // column inside a 128-column half
#pragma unroll
    for (int nh = 0; nh < 2; ++nh) {
      int gcol;
      if (EPI == kEpiSwiglu) gcol = nh * p.N + min(ntile * (kBN / 2) + nl, p.N - 8);   // half 0 = gate, 1 = up
      else gcol = min(ntile * kBN + nh * 128 + nl, p.N - 8);
      t.b_off[nh] = (uint32_t)((kk * p.ldb + gcol) * 2);
    }
  }

  // operand read offsets inside a stage
  uint32_t a_rd[4], b_rd[4];
  {
    const uint32_t a0 = (uint32_t)(((wm * half) >> 3) * kLine + (l32 >> 3) * kLine + (l32 & 7) * 128);
    const int f = (l32 >> 1) & 7;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) a_rd[ks] = a0 + (uint32_t)((((ks * 2 + lh) ^ f) & 7) << 4);
    const int g = lane >> 4, i = lane & 15;
    const int kk = i >> 2;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      // column block of 32 inside the tile's 256 staged columns
      const int nb = (EPI == kEpiSwiglu) ? (nt >> 1) * 128 + wn * 64 + (nt & 1) * 32 : wn * 128 + nt * 32;
      const int j = ((nb & 127) >> 3) + (g & 1) * 2 + ((i & 3) >> 1);
      b_rd[nt] = (uint32_t)((g >> 1) * 4 * kLine + (nb >> 7) * kLine + kk * 256 + ((j + 4 * kk) & 15) * 16 + (i & 1) * 8);
    }
  }

  f32x16 acc[kMaxMT][4];
#pragma unroll
  for (int i = 0; i < kMaxMT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int n_steps = p.K / kBK;
  switch (n_mt) {
    case 0: gemm_k_loop<0>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 1: gemm_k_loop<1>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 2: gemm_k_loop<2>(acc, t, smem, n_steps, a_rd, b_rd); break;
    case 3: gemm_k_loop<3>(acc, t, smem, n_steps, a_rd, b_rd); break;
    default: gemm_k_loop<4>(acc, t, smem, n_steps, a_rd, b_rd); break;
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
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void grouped_gemm_bf16_kernel(GemmParams p) {
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
