// Weight gradients of the grouped GEMMs (paper Section 2.2, Figure 2b: w2_grad, w1_grad):
//   C_e[M, N] = A_e[rows_e, M]^T * B_e[rows_e, N]      for every local expert e,
// bf16 operands, fp32 accumulation, bf16 result.  The reduction runs over the expert's rows
// only (a few hundred at the paper's shapes), while the result is the size of the weights:
// the kernel writes far more than it reads and its K loop is a handful of steps, so what
// matters is that stores, operand loads and MFMAs of DIFFERENT tiles overlap.  Inside one
// wave they cannot (loads and stores retire in order behind one counter), therefore two
// workgroups share a CU: 128 x 256 tiles (4 waves, 2 x 2, 64 x 128 per wave, 128 accumulator
// registers), K step 32, three LDS stages of 24 KB (72 KB per workgroup), one barrier per
// step, loads two steps ahead.  While one workgroup drains its epilogue the other computes.
//
// Both operands are k-rows of contiguous m / n: they are staged as lines of 4 k-rows x 128
// columns (each k-row rotated by 64 bytes) and fetched with the LDS transpose read, exactly
// like the weight operand of the forward GEMMs.  k-rows past the segment are clamped when
// loaded and zeroed in LDS before the last step.
#pragma once
#include "gemm_bf16.h"

namespace moe {

constexpr int kWgBM = 128, kWgBN = 256, kWgBK = 32, kWgStages = 3;
constexpr int kWgALines = kWgBK / 4;                                 // 8 lines: 4 k-rows x 128 m
constexpr int kWgBLines = (kWgBK / 4) * 2;                           // 16 lines: 4 k-rows x 128 n, two column halves
constexpr int kWgStageBytes = (kWgALines + kWgBLines) * kLine;       // 24 KB
constexpr int kWgLdsBytes = kWgStages * kWgStageBytes;               // 72 KB
constexpr int kWgLoads = (kWgALines + kWgBLines) / 4;                // wave-wide loads per wave per step (6)
static_assert(4 * kEpiWaveBytes <= kWgLdsBytes, "epilogue staging aliases the stages");

struct WgradCtx {
  const char* a_base;      // uniform: first row of the expert's segment in A, byte address
  const char* b_base;      // uniform: same for B
  uint32_t a_col;          // per lane: byte offset of the column chunk it fetches from an A k-row
  uint32_t b_col[2];       // per lane: same for the two 128-column halves of B
  uint32_t a_rd[2];        // transpose-read offset of 32-row block mt inside the A part of a stage
  uint32_t b_rd[4];        // same for 32-column block nt inside the B part
  uint32_t lds0;
  int lda_bytes, ldb_bytes;
  int k_rows;              // rows of the segment (reduction length)
  int kk;                  // k-row of this lane inside a line (lane / 16)
  int wave;
};

// Offset of this lane's transpose read for the 32-column block starting at staged column nb;
// a 4-k-row group spans `halves` lines.  Lanes 0..31 cover k-rows 0..3 of the slice (the second
// read, `halves` lines further, rows 4..7), lanes 32..63 rows 8..11 (12..15).
__device__ __forceinline__ uint32_t wgrad_tr_off(int lane, int nb, int halves) {
  const int g = lane >> 4, i = lane & 15, kk = i >> 2;
  const int j = ((nb & 127) >> 3) + (g & 1) * 2 + ((i & 3) >> 1);
  return (uint32_t)((g >> 1) * 2 * halves * kLine + (nb >> 7) * kLine + kk * 256 + ((j + 4 * kk) & 15) * 16 + (i & 1) * 8);
}

// The 6 loads of this wave for K step `step` into stage `stage`: the 24 lines of a stage are
// dealt to the waves in order, A lines first.
__device__ __forceinline__ void wgrad_issue_step(const WgradCtx& t, int step, int stage) {
  const uint32_t st = uniform_u32(t.lds0 + (uint32_t)stage * kWgStageBytes);
  const int k0 = step * kWgBK;
#pragma unroll
  for (int i = 0; i < kWgLoads; ++i) {
    const int L = t.wave * kWgLoads + i;                     // wave-uniform
    if (L < kWgALines) {
      const int krow = min(k0 + L * 4 + t.kk, t.k_rows - 1); // rows past the segment: re-read, zeroed later
      lds_dma16(t.a_base, (uint32_t)(krow * t.lda_bytes) + t.a_col, st + L * kLine);
    } else {
      const int j = L - kWgALines;
      const int krow = min(k0 + (j >> 1) * 4 + t.kk, t.k_rows - 1);
      const uint32_t col = (j & 1) ? t.b_col[1] : t.b_col[0];
      lds_dma16(t.b_base, (uint32_t)(krow * t.ldb_bytes) + col, st + L * kLine);
    }
  }
}

// Zero the k-rows >= k_valid of a stage (A: one 256-byte row per line, B: one per half).
__device__ __forceinline__ void wgrad_zero_k_tail(char* stage, int k_valid) {
  typedef __attribute__((address_space(3))) u32x4* lds_u32x4_ptr;
  const lds_cptr lds = (lds_cptr)stage;
  const u32x4 z = {0u, 0u, 0u, 0u};
  // 48 sixteen-byte chunks per k-row: 16 of A, 32 of B
  for (int idx = threadIdx.x; idx < (kWgBK - k_valid) * 48; idx += kGemmThreads) {
    const int kr = k_valid + idx / 48, c = idx % 48;
    int off;
    if (c < 16) off = (kr >> 2) * kLine + (kr & 3) * 256 + c * 16;
    else off = kWgALines * kLine + ((kr >> 2) * 2 + ((c - 16) >> 4)) * kLine + (kr & 3) * 256 + ((c - 16) & 15) * 16;
    *(lds_u32x4_ptr)(lds + off) = z;
  }
}

// One K step for a wave with NMT active 32-row blocks: two 16-wide slices, each 4 weight-side
// and NMT activation-side fragments (two transpose reads per fragment), NMT x 4 MFMAs.
template <int NMT>
__device__ __forceinline__ void wgrad_compute_step(f32x16 (&acc)[2][4], const WgradCtx& t, lds_cptr stage) {
  if (NMT == 0) return;
  const lds_cptr as = stage, bs = stage + kWgALines * kLine;
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    bf16x8 wf[4], xf[NMT > 0 ? NMT : 1];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      const lds_cptr q = bs + t.b_rd[nt] + ks * 8 * kLine;
      wf[nt] = join_tr(__builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)q),
                       __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(q + 2 * kLine)));
    }
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
      const lds_cptr q = as + t.a_rd[mt] + ks * 4 * kLine;
      xf[mt] = join_tr(__builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)q),
                       __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(q + kLine)));
    }
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nt], xf[mt], acc[mt][nt], 0, 0, 0);
  }
}

template <int NMT>
__device__ __forceinline__ void wgrad_k_loop(f32x16 (&acc)[2][4], const WgradCtx& t, char* smem, int n_steps, int k_tail) {
  if (n_steps <= 0) return;
  wgrad_issue_step(t, 0, 0);
  if (n_steps > 1) wgrad_issue_step(t, 1, 1);
  int st = 0;                                   // stage of step s
  for (int s = 0; s < n_steps; ++s) {
    if (s + 1 < n_steps) wait_vmcnt<kWgLoads>(); else wait_vmcnt<0>();   // this wave's part of step s has landed
    __builtin_amdgcn_s_barrier();               // ... and everybody's; stage (s + 2) % 3 has been read out by all
    const int st2 = st == 0 ? 2 : st - 1;       // (s + 2) % 3
    if (s + 2 < n_steps) wgrad_issue_step(t, s + 2, st2);
    if (s + 1 == n_steps && k_tail) {
      wgrad_zero_k_tail(smem + st * kWgStageBytes, k_tail);
      wait_lgkmcnt0();
      __builtin_amdgcn_s_barrier();
    }
    wgrad_compute_step<NMT>(acc, t, (lds_cptr)smem + st * kWgStageBytes);
    st = st == 2 ? 0 : st + 1;
  }
}

// Tile (mt, nt) of expert e's gradient.
__device__ __forceinline__ void wgrad_tile_bf16(const GemmParams& p, int e, int mtile, int ntile, char* smem) {
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));                // per-lane setup stays inside the tile loop
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31;
  const int row0 = mtile * kWgBM;               // first output row
  const int rows = min(kWgBM, p.M - row0);
  const int row_base = wm * 64;
  const int n_mt = min(2, max(0, (rows - row_base + 31) >> 5));
  const int seg0 = __builtin_amdgcn_readfirstlane(p.offsets[e]);
  const int cnt = __builtin_amdgcn_readfirstlane(p.offsets[e + 1]) - seg0;
  const int n_steps = (cnt + kWgBK - 1) / kWgBK, k_tail = cnt % kWgBK;

  WgradCtx t;
  t.wave = wave;
  t.kk = lane >> 4;
  t.k_rows = cnt;
  t.lda_bytes = p.lda * 2;
  t.ldb_bytes = p.ldb * 2;
  t.a_base = uniform_ptr(reinterpret_cast<const char*>(p.A + (size_t)seg0 * p.lda));
  t.b_base = uniform_ptr(reinterpret_cast<const char*>(p.B + (size_t)seg0 * p.ldb));
  // lane -> (k-row kk, position pos = lane % 16) holds column chunk pos - 4*kk of the line's 128 columns
  const int tr_nl = (((lane & 15) - 4 * t.kk) & 15) * 8;
  t.a_col = (uint32_t)(min(row0 + tr_nl, p.M - 8) * 2);             // columns past the end: re-read, never stored
#pragma unroll
  for (int h = 0; h < 2; ++h) t.b_col[h] = (uint32_t)(min(ntile * kWgBN + h * 128 + tr_nl, p.N - 8) * 2);
  t.lds0 = lds_addr_of(smem);
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) t.a_rd[mt] = wgrad_tr_off(lane, wm * 64 + mt * 32, 1);
#pragma unroll
  for (int nt = 0; nt < 4; ++nt) t.b_rd[nt] = wgrad_tr_off(lane, wn * 128 + nt * 32, 2);

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  switch (n_mt) {
    case 0: wgrad_k_loop<0>(acc, t, smem, n_steps, k_tail); break;
    case 1: wgrad_k_loop<1>(acc, t, smem, n_steps, k_tail); break;
    default: wgrad_k_loop<2>(acc, t, smem, n_steps, k_tail); break;
  }
  __builtin_amdgcn_s_barrier();                 // every wave has read its last operands: the stages become staging space

  // lane holds row l32 of each 32 x 32 block and, per register group q, 4 consecutive columns
  __bf16* c_base = p.C + (size_t)e * p.strideC;
  char* region = smem + wave * kEpiWaveBytes;
  const int c0 = ntile * kWgBN + wn * 128;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    const int m0 = row_base + mt * 32;
    const int rows_valid = min(32, rows - m0);
    if (mt >= n_mt || rows_valid <= 0) continue;             // wave-uniform
    u32x2 pk[4][4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        pk[nt][q] = u32x2{pack_bf16(acc[mt][nt][q * 4 + 0], acc[mt][nt][q * 4 + 1]),
                          pack_bf16(acc[mt][nt][q * 4 + 2], acc[mt][nt][q * 4 + 3])};
    store_block_via_lds<4, true>(region, pk, c_base + (size_t)(row0 + m0) * p.ldc + c0, p.ldc, rows_valid, p.N - c0);
  }
  (void)l32;
  wait_lgkmcnt0();
  __builtin_amdgcn_s_barrier();                 // staging space is read out before the next tile's loads land in it
}

// Tile number r of an expert -> (M tile, N tile).  The tiles that run at the same time behind one L2 (64
// consecutive numbers) should share as many operand panels as possible: a k step of an a x b block of tiles
// reads a A-panels of 8 KB and b B-panels of 16 KB, which for 64 tiles is least around 8 x 8 (192 KB; a whole
// row of N tiles at a time would be 288 KB at 16 N tiles and 466 KB at 28).  So the numbering runs block by
// block: bands of 8 M tiles, inside a band blocks of 8 N tiles (the last block of a band narrower, the last
// band lower), inside a block N-tile-major; no gaps.
constexpr int kWgBlock = 8;
__device__ __forceinline__ void wgrad_tile_of(int r, int n_mt, int n_nt, int& mt, int& nt) {
  const int band = r / (kWgBlock * n_nt), rr = r - band * kWgBlock * n_nt;
  const int h = min(kWgBlock, n_mt - kWgBlock * band);
  const int full = n_nt / kWgBlock;
  if (rr < h * kWgBlock * full) {
    const int sbn = rr / (h * kWgBlock), i = rr - sbn * h * kWgBlock;
    mt = band * kWgBlock + i / kWgBlock;
    nt = sbn * kWgBlock + i % kWgBlock;
  } else {
    const int rem = rr - h * kWgBlock * full, w = n_nt - full * kWgBlock;
    mt = band * kWgBlock + rem / w;
    nt = full * kWgBlock + rem % w;
  }
}

// Experts without rows get zeros (unless k_lo > 0 leaves them, like every expert with fewer than
// k_lo rows, to the register-stationary kernel).
//
// Work distribution.  A tile costs as much as its expert has rows, and with skewed routing the experts this
// kernel takes differ by an order of magnitude while others are not its business at all.  Every workgroup
// therefore first ranks the experts it has to do by rows, largest first, which gives one list of tiles,
// expert by expert (wgrad_tile_of inside an expert), without gaps and with neighbours of equal cost: a sweep of
// G consecutive tiles over the G workgroups is then balanced by construction (all tiles of a sweep belong to
// one expert or to two of neighbouring size), and the last, partly filled sweep holds the cheapest tiles.  An
// XCD takes a contiguous range of every sweep, so the CUs that share operand panels sit behind one L2.
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void grouped_wgrad2_bf16_kernel(GemmParams p) {
  __shared__ __attribute__((aligned(1024))) char smem[kWgLdsBytes];
  __shared__ int s_rows[kMaxE];      // rows of expert e if this kernel takes it, else -1
  __shared__ int s_order[kMaxE];     // the experts it takes, most rows first
  __shared__ int s_box[1];           // number of such experts
  const int n_mt = (p.M + kWgBM - 1) / kWgBM, n_nt = (p.N + kWgBN - 1) / kWgBN;
  const int per_e = n_mt * n_nt;
  // nothing to do when the other kernel takes every expert (p.tiles.meta: the M-tile map's header, or nullptr)
  if (p.k_lo > 0 && p.tiles.meta && __builtin_amdgcn_readfirstlane(p.tiles.meta[kMetaMaxRows]) < p.k_lo) return;
  for (int e = threadIdx.x; e < p.E_local; e += kGemmThreads) {
    const int cnt = p.offsets[e + 1] - p.offsets[e];
    s_rows[e] = cnt >= p.k_lo ? cnt : -1;
  }
  __syncthreads();
  int n_mine = 0;
  for (int e = threadIdx.x; e < p.E_local; e += kGemmThreads) {
    const int cnt = s_rows[e];
    int rank = 0;    // experts ahead of e: more rows, or as many and a lower id
    for (int o = 0; o < p.E_local; ++o) {
      const int c = s_rows[o];
      rank += c >= 0 && (c > cnt || (c == cnt && o < e));
    }
    if (cnt >= 0) s_order[rank] = e;
    n_mine += cnt >= 0;
  }
  if (threadIdx.x == 0) s_box[0] = 0;
  __syncthreads();
  if (n_mine) atomicAdd(&s_box[0], n_mine);
  __syncthreads();
  const int total = s_box[0] * per_e;
  const int G = gridDim.x;
  for (int it = 0; it * G < total; ++it) {
    const int tile = xcd_tile_id(it, blockIdx.x, G);
    if (tile >= total) continue;
    const int r = tile / per_e;
    const int e = __builtin_amdgcn_readfirstlane(s_order[r]);
    int mt, nt;
    wgrad_tile_of(tile - r * per_e, n_mt, n_nt, mt, nt);
    wgrad_tile_bf16(p, e, __builtin_amdgcn_readfirstlane(mt), __builtin_amdgcn_readfirstlane(nt), smem);
  }
}

}  // namespace moe
