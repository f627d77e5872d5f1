// Weight gradients, register-stationary form (paper Section 2.2, Figure 2b: w2_grad, w1_grad):
//   C_e[M, N] = A_e[rows_e, M]^T * B_e[rows_e, N],   rows_e <= 384.
// At the paper's shapes an expert has a few hundred rows, so the whole reduction extent of a
// 256-row panel of A_e^T fits in registers as MFMA operands (16 registers per 64 k-rows and
// wave).  A workgroup (8 waves, 32 output rows each) loads its panel once and then sweeps N
// tiles of 128 columns: per tile only B_e[:, 128 columns] has to be fetched (64 KB at 256
// rows), about one operand byte per result byte, where a tile-by-tile kernel fetches three.
// That matters because the operand stream is latency bound: what a CU can keep in flight is
// fixed by its LDS.
//
// Everything a workgroup consumes is one stream of "entries" of 64 k-rows x 128 columns
// (16 KB, staged as lines of 4 k-rows x 128 columns for the LDS transpose read, as in the
// forward GEMMs): first the panel (two entries per 64 k-rows, one per 128-column half), then
// the B chunks of tile 0, tile 1, ...  A ring of 5 slots holds them; entry g + 4 is requested
// as soon as the barrier of entry g has shown that the slot of entry g - 1 is free.  One
// barrier per entry; the epilogue of a tile (through a wave-private LDS region, whole lines,
// non-temporal) needs none: the packed block is parked in the region at the end of its tile and
// read back and stored one row group per MFMA under the first slices of the next tile (the last
// tile of an item is written out at once).
//
// Loads and stores of a wave retire in order behind one counter, so the wait for entry g has
// to allow for everything issued after its loads: the loads of the following entries (2 per
// entry and wave) and the 8 stores of every epilogue in between.  Tiles are always full
// here (M % 256 == 0, N % 128 == 0 is a launch condition), so those counts are exact.
#pragma once
#include "gemm_bf16.h"
#include "wave_sync.h"

namespace moe {

// Tracing variant only (-DMOE_SCHED_TRACE): shader-clock cycles that waves 0 and 5 of every workgroup spend per
// phase of the tile sweep, summed over all items.  Per wave 8 words: vmcnt wait, barrier, next request (the three
// steps of an entry hand-over), everything between two hand-overs (16 MFMAs and their operand reads), epilogues,
// number of hand-overs, number of tiles, unused.
#if defined(MOE_SCHED_TRACE)
__device__ unsigned long long g_wgrad_cycles[16];
#define MOE_WG_CLOCK() ((long long)__builtin_amdgcn_s_memtime())
#endif

constexpr int kWpM = 256;                          // output rows per panel
constexpr int kWpN = 128;                          // output columns per tile
constexpr int kWpBK = 64;                          // k-rows per entry
constexpr int kWpSlot = 16 * kLine;                // 16 KB
constexpr int kWpThreads = 512;                    // 8 waves, two per SIMD: one wave's waits and VALU work hide under the other's MFMAs
constexpr int kWpWaves = kWpThreads / kWave;
constexpr int kWpDepth = 5;                        // ring slots
constexpr int kWpAhead = kWpDepth - 1;             // entries requested ahead of the one being consumed
constexpr int kWpMaxKC = 6;                        // 64-row chunks: rows_e <= 384 (16 registers per chunk; 256 per wave in all)
constexpr int kWpMaxRows = kWpMaxKC * kWpBK;
constexpr int kWpLoads = 16 / kWpWaves;            // wave-wide loads per wave per entry (2)
constexpr int kWpEpiStores = 8;                    // store instructions per wave per epilogue
constexpr int kWpTokBytes = 2048;                  // gathered A: byte offset of every row of the expert's segment (<= 384 x 4 B)
constexpr int kWpTokOff = kWpDepth * kWpSlot + kWpWaves * kEpiWaveBytes;
constexpr int kWpLdsBytes = kWpTokOff + kWpTokBytes;                          // 150 KB
static_assert(kWpMaxRows * 4 <= kWpTokBytes, "row-offset table");
static_assert(kWpLdsBytes <= kGemmLdsBytes, "LDS budget");

struct WpCtx {
  const char* a_base;      // uniform: first row of the expert's segment in A / B, byte addresses
  const char* b_base;      //          (gathered A: row 0 of the whole matrix, rows found through a_rows)
  const __attribute__((address_space(3))) uint32_t* a_rows;   // gathered A: byte offset of segment row k, else unused
  int gathered;
  uint32_t lane_col;       // per lane: byte offset of the column chunk it fetches inside a 128-column line
  uint32_t a_rd;           // transpose-read offset of this wave's 32-row block inside a panel entry
  uint32_t b_rd[4];        // ... of the four 32-column blocks inside a B entry
  uint32_t lds0;
  int a_col0, b_col0;      // first column (elements) of the panel in A, of tile 0 in B
  int lda_bytes, ldb_bytes;
  int k_rows, kk, wave;
  int NT;                  // tiles of this item
  __bf16* c_base;          // the expert's output
  int ldc;
};

// s_waitcnt vmcnt(n) for a wave-uniform even n; anything above 22 waits for 22 (stricter).
__device__ __forceinline__ void wait_vmcnt_uniform(int n) {
  switch (n >> 1) {
    case 0: wait_vmcnt<0>(); break;   case 1: wait_vmcnt<2>(); break;   case 2: wait_vmcnt<4>(); break;
    case 3: wait_vmcnt<6>(); break;   case 4: wait_vmcnt<8>(); break;   case 5: wait_vmcnt<10>(); break;
    case 6: wait_vmcnt<12>(); break;  case 7: wait_vmcnt<14>(); break;  case 8: wait_vmcnt<16>(); break;
    case 9: wait_vmcnt<18>(); break;  case 10: wait_vmcnt<20>(); break;
    default: wait_vmcnt<22>(); break;
  }
}

// Request entry g of the item's stream into its ring slot: this wave's 2 lines (8 k-rows).
template <int KC>
__device__ __forceinline__ void wp_issue_entry(const WpCtx& t, int g) {
  const uint32_t slot = uniform_u32(t.lds0 + (uint32_t)(g % kWpDepth) * kWpSlot);
  const char* base;
  int kc, col, ld_bytes;
  const bool a_rows = g < 2 * KC && t.gathered;   // uniform
  if (g < 2 * KC) {
    kc = g >> 1;
    col = t.a_col0 + (g & 1) * 128;
    base = t.a_base;
    ld_bytes = t.lda_bytes;
  } else {
    const int h = g - 2 * KC;
    const int tile = h / (KC > 0 ? KC : 1);
    kc = h - tile * KC;
    col = t.b_col0 + tile * kWpN;
    base = t.b_base;
    ld_bytes = t.ldb_bytes;
  }
  const uint32_t col_bytes = (uint32_t)col * 2 + t.lane_col;
#pragma unroll
  for (int i = 0; i < kWpLoads; ++i) {
    const int L = t.wave * kWpLoads + i;                                   // line = group of 4 k-rows
    const int krow = min(kc * kWpBK + L * 4 + t.kk, t.k_rows - 1);         // rows past the segment: re-read; masked in the panel
    const uint32_t row_bytes = a_rows ? t.a_rows[krow] : (uint32_t)(krow * ld_bytes);
    lds_dma16(base, row_bytes + col_bytes, slot + L * kLine);
  }
}

// Wait until this wave's loads of entry g have landed.  Issued after them: the loads of up to
// kWpAhead - 1 further entries and the stores of the epilogues of the last kWpAhead + 1 entries (bit i of
// epi_mask: an epilogue ran after entry g - 1 - i; entry g was requested while entry g - 1 - kWpAhead
// was the current one, ahead of that entry's epilogue, so exactly these epilogues are younger than
// the request).  Allowing for FEWER operations than were issued is always safe, for more never: more
// than two such epilogues are counted as two.
__device__ __forceinline__ void wp_wait_entry(int g, int n_entries, uint32_t epi_mask) {
  const int nl = min(kWpAhead - 1, n_entries - 1 - g);   // entries g + 1 .. g + kWpAhead - 1 have been requested by now
  const int ne = min(2, __builtin_popcount(epi_mask & ((1u << (kWpAhead + 1)) - 1)));
  wait_vmcnt_uniform(kWpLoads * nl + kWpEpiStores * ne);
}

// Full 32 x 128 block through the wave's staging region: like store_block_via_lds<4>, but without
// bounds (tiles are full here), so the eight row-contiguous reads are issued together and the
// eight stores follow without a branch in between.
__device__ __forceinline__ void wp_store_block(char* region, const u32x2 (&pk)[4][4], __bf16* gdst, long ld) {
  typedef __attribute__((address_space(3))) char* lds_ptr;
  typedef __attribute__((address_space(3))) u32x2* lds_u32x2_ptr;
  typedef __attribute__((address_space(3))) const u32x4* lds_u32x4_cptr;
  int lane = lane_id();
  asm volatile("" : "+v"(lane));
  const int l32 = lane & 31, lh = lane >> 5;
  const lds_ptr base = (lds_ptr)region;
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int q = 0; q < 4; ++q) *(lds_u32x2_ptr)(base + l32 * kEpiRowBytes + (nt * 32 + q * 8 + lh * 4) * 2) = pk[nt][q];
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const int row_l = lane >> 4, ch = lane & 15;              // 16 lanes x 16 bytes per row, 4 rows per access
  const lds_ptr lp = base + row_l * kEpiRowBytes + ch * 16;
  __bf16* gp = gdst + (size_t)row_l * ld + ch * 8;
  u32x4 v[8];
#pragma unroll
  for (int it = 0; it < 8; ++it) v[it] = *(lds_u32x4_cptr)(lp + it * 4 * kEpiRowBytes);
#pragma unroll
  for (int it = 0; it < 8; ++it) __builtin_nontemporal_store(v[it], reinterpret_cast<u32x4*>(gp + (size_t)(it * 4) * ld));
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// The same epilogue in two parts, for a tile that is followed by another one: the packed block is parked in the
// staging region at the end of its tile (wp_stage_write); the reads back and the eight stores are issued one per
// MFMA during the first slices of the NEXT tile (wp_stage_read / wp_stage_store), where they cost no matrix-pipe time.
__device__ __forceinline__ void wp_stage_write(char* region, const f32x16 (&acc)[4]) {
  typedef __attribute__((address_space(3))) char* lds_ptr;
  typedef __attribute__((address_space(3))) u32x2* lds_u32x2_ptr;
  int lane = lane_id();
  asm volatile("" : "+v"(lane));
  const int l32 = lane & 31, lh = lane >> 5;
  const lds_ptr base = (lds_ptr)region;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the previous block has been read out
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *(lds_u32x2_ptr)(base + l32 * kEpiRowBytes + (nt * 32 + q * 8 + lh * 4) * 2) =
          u32x2{pack_bf16(acc[nt][q * 4 + 0], acc[nt][q * 4 + 1]), pack_bf16(acc[nt][q * 4 + 2], acc[nt][q * 4 + 3])};
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// rows it*4 .. it*4+3 of the parked block: 16 lanes x 16 bytes per row
__device__ __forceinline__ u32x4 wp_stage_read(const char* region, int lane, int it) {
  typedef __attribute__((address_space(3))) const char* lds_cptr_;
  typedef __attribute__((address_space(3))) const u32x4* lds_u32x4_cptr;
  const lds_cptr_ lp = (lds_cptr_)region + (lane >> 4) * kEpiRowBytes + (lane & 15) * 16;
  return *(lds_u32x4_cptr)(lp + it * 4 * kEpiRowBytes);
}
__device__ __forceinline__ void wp_stage_store(const u32x4& v, __bf16* gdst, long ld, int lane, int it) {
  __bf16* gp = gdst + (size_t)(lane >> 4) * ld + (lane & 15) * 8;
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(gp + (size_t)(it * 4) * ld));
}

template <int KC>
__device__ __forceinline__ void wp_item(const WpCtx& t, int row0, char* smem) {
  constexpr int KS = KC * 4;                                   // 16-wide k slices of the panel
  const lds_cptr lds = (lds_cptr)smem;
  const int wm = t.wave;
  const int n_entries = 2 * KC + KC * t.NT;
  int lane = lane_id();
  asm volatile("" : "+v"(lane));
  const int lh = lane >> 5;

  bf16x8 xa[KS > 0 ? KS : 1];                                   // the panel: this wave's 32 rows, per k slice
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

#pragma unroll 1
  for (int g = 0; g < min(kWpAhead, n_entries); ++g) wp_issue_entry<KC>(t, g);
  uint32_t epi_mask = 0;
  int g = 0, slot = 0;
  auto next_entry = [&]() {
    wp_wait_entry(g, n_entries, epi_mask);
    __builtin_amdgcn_s_barrier();          // entry g is complete; everybody is done with entry g - 1
    if (g + kWpAhead < n_entries) wp_issue_entry<KC>(t, g + kWpAhead);
  };
  auto entry_done = [&]() {
    epi_mask <<= 1;
    ++g;
    slot = slot == kWpDepth - 1 ? 0 : slot + 1;
  };

  // ---- the panel: entry (kc, half) holds k-rows kc*64.. x columns half*128..; wave wm owns rows wm*32.. ----
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      next_entry();
      if ((wm >> 2) == half) {                                  // wave-uniform
        const lds_cptr s = lds + slot * kWpSlot;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const lds_cptr q = s + t.a_rd + ks * 4 * kLine;
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            s16x8 v = __builtin_bit_cast(s16x8, join_tr(__builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)q),
                                                        __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(q + kLine))));
            if (kc == KC - 1) {
              // this lane holds k = kc*64 + ks*16 + lh*8 + j, j = 0..7: blank what lies past the segment
              const int k0 = kc * kWpBK + ks * 16 + lh * 8;
#pragma unroll
              for (int j = 0; j < 8; ++j) v[j] = k0 + j < t.k_rows ? v[j] : (short)0;
            }
            xa[kc * 4 + ks] = __builtin_bit_cast(bf16x8, v);
          }
        // the next hand-over lets the other waves request into this slot: the panel has to be in registers first
        wait_lgkmcnt0();
      }
      entry_done();
    }
  }

  // ---- tiles ----
  __bf16* c_row = t.c_base + (size_t)(row0 + wm * 32) * t.ldc + t.b_col0;
  char* region = smem + kWpDepth * kWpSlot + wm * kEpiWaveBytes;
  // Fragments of one 16-wide slice of the current B entry.  While a slice is multiplied (4 MFMAs), the
  // 8 transpose reads of the next slice are issued two per MFMA, pinned there by sched_barrier; the
  // other wave of the SIMD covers what latency remains.  Before the LAST slice of an entry the wave already moves on
  // to the next entry (wait, barrier, next request): that, too, then hides under the last slice.
  s16x4 cur[4][2], nxt[4][2];
  auto read_one = [&](s16x4 (&f)[4][2], int sl, int ks, int j) {
    const lds_cptr q = lds + sl * kWpSlot + t.b_rd[j >> 1] + ks * 4 * kLine + (j & 1) * kLine;
    f[j >> 1][j & 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)q);
  };
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // `first`: the tile's first slice starts from zero (the MFMA takes the constant, nothing is cleared by hand)
  auto slice = [&](const bf16x8& x, bool first, bool read_next, int sl, int ks) {
    bf16x8 wf[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) wf[nt] = join_tr(cur[nt][0], cur[nt][1]);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], x, first ? zero : acc[j], 0, 0, 0);
      if (read_next) {
        read_one(nxt, sl, ks, 2 * j);
        read_one(nxt, sl, ks, 2 * j + 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (read_next) {
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) { cur[nt][0] = nxt[nt][0]; cur[nt][1] = nxt[nt][1]; }
    }
  };
  // The same slice with the parked epilogue of the previous tile riding along: MFMA m = m0 + j of the tile's first
  // twelve reads row group m back from the staging region and stores row group m - 1 (two buffers in turn).
  u32x4 ev[2];
  __bf16* pend_dst = c_row;
  auto slice_epi = [&](const bf16x8& x, bool first, int sl, int ks, int m0) {
    bf16x8 wf[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) wf[nt] = join_tr(cur[nt][0], cur[nt][1]);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], x, first ? zero : acc[j], 0, 0, 0);
      read_one(nxt, sl, ks, 2 * j);
      read_one(nxt, sl, ks, 2 * j + 1);
      const int m = m0 + j;
      if (m >= 1 && m <= 8) wp_stage_store(ev[(m - 1) & 1], pend_dst, t.ldc, lane, m - 1);
      if (m < 8) ev[m & 1] = wp_stage_read(region, lane, m);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) { cur[nt][0] = nxt[nt][0]; cur[nt][1] = nxt[nt][1]; }
  };
  if (g < n_entries) {
    next_entry();
#pragma unroll
    for (int j = 0; j < 8; ++j) read_one(cur, slot, 0, j);
  }
#if defined(MOE_SCHED_TRACE)
  long long cy[6] = {0, 0, 0, 0, 0, 0};
  long long c_prev = MOE_WG_CLOCK();
#endif
#pragma unroll 1
  for (int tile = 0; tile < t.NT; ++tile) {
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      if (kc == 0 && tile > 0) {              // wave-uniform: the previous tile's block is parked
#pragma unroll
        for (int ks = 0; ks < 3; ++ks) slice_epi(xa[kc * 4 + ks], ks == 0, slot, ks + 1, ks * 4);
      } else {
#pragma unroll
        for (int ks = 0; ks < 3; ++ks) slice(xa[kc * 4 + ks], kc == 0 && ks == 0, true, slot, ks + 1);
      }
      entry_done();
      const bool more = g < n_entries;
      if (more) {
        wait_lgkmcnt0();                   // this wave holds everything it needs from the entry it leaves
#if defined(MOE_SCHED_TRACE)
        const long long c0 = MOE_WG_CLOCK();
        wp_wait_entry(g, n_entries, epi_mask);
        const long long c1 = MOE_WG_CLOCK();
        __builtin_amdgcn_s_barrier();
        const long long c2 = MOE_WG_CLOCK();
        if (g + kWpAhead < n_entries) wp_issue_entry<KC>(t, g + kWpAhead);
        const long long c3 = MOE_WG_CLOCK();
        cy[0] += c1 - c0; cy[1] += c2 - c1; cy[2] += c3 - c2; cy[3] += c0 - c_prev; cy[5] += 1; c_prev = c3;
#else
        next_entry();
#endif
      }
      slice(xa[kc * 4 + 3], false, more, slot, 0);
    }
    // epilogue: lane holds row lane%32 of each 32 x 32 block and, per register group q, 4 consecutive columns
    if (KC > 0 && tile + 1 < t.NT) {
      wp_stage_write(region, acc);            // read back and stored under the next tile's first MFMAs
      pend_dst = c_row + tile * kWpN;
    } else {
      u32x2 pk[4][4];
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          // an expert without rows (KC = 0) has no slices: its tiles are the zeros acc starts with
          pk[nt][q] = u32x2{pack_bf16(acc[nt][q * 4 + 0], acc[nt][q * 4 + 1]),
                            pack_bf16(acc[nt][q * 4 + 2], acc[nt][q * 4 + 3])};
        }
      wp_store_block(region, pk, c_row + tile * kWpN, t.ldc);
    }
#if defined(MOE_SCHED_TRACE)
    { const long long ce = MOE_WG_CLOCK(); cy[4] += ce - c_prev; c_prev = ce; }
#endif
    epi_mask |= 1u;
  }
  wait_lgkmcnt0();
  __builtin_amdgcn_s_barrier();            // ring and staging space are quiet before the next item's first loads
#if defined(MOE_SCHED_TRACE)
  if (lane == 0 && (wm == 0 || wm == 5)) {
    unsigned long long* d = g_wgrad_cycles + (wm == 0 ? 0 : 8);
    for (int i = 0; i < 6; ++i) atomicAdd(d + i, (unsigned long long)cy[i]);
    atomicAdd(d + 6, (unsigned long long)t.NT);
  }
#endif
}

// Launch condition: p.M % 256 == 0, p.N % 128 == 0.  Experts with more than 384 rows are left alone (the
// general kernel takes them); experts without rows get zeros.  An item is (expert, one of n_split column
// ranges, row panel); n_split is the smallest divisor of the N-tile count that gives the experts this kernel
// really multiplies (1 .. 384 rows: counted here, the host never sees the counts) at least `want_items` items.
// p.gather != nullptr: row k of expert e's segment of A is row p.gather[offsets[e] + k] of p.A (the
// dispatch permutation applied while loading; the caller guarantees that p.A spans < 4 GB).
__global__ __launch_bounds__(kWpThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void grouped_wgrad_panel_bf16_kernel(GemmParams p, int want_items) {
  __shared__ __attribute__((aligned(1024))) char smem[kWpLdsBytes];
  const int n_mp = p.M / kWpM, n_nt = p.N / kWpN;
  int n_split = 1;
  {
    int mine = 0;   // every wave counts for itself: a wave-uniform result without a barrier
    for (int e = lane_id(); e < p.E_local; e += kWave) {
      const int cnt = p.offsets[e + 1] - p.offsets[e];
      mine += cnt > 0 && cnt <= kWpMaxRows;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mine += __shfl_xor(mine, off, kWave);
    // none to multiply (only zeros to write, or nothing): one range per expert, the fewest tickets
    const int per_split = __builtin_amdgcn_readfirstlane(mine) * n_mp;
    for (int d = 1; d <= (per_split > 0 ? n_nt : 1); ++d)
      if (n_nt % d == 0) {
        n_split = d;
        if (per_split * d >= want_items) break;
      }
  }
  const int NT = n_nt / n_split;
  const int per_e = n_split * n_mp;
  const int total = p.E_local * per_e;
  const int G = gridDim.x;
  int lane = lane_id();
  asm volatile("" : "+v"(lane));
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // The n_mp row panels of one (expert, column range) read the same B chunks: a "group".  With p.tickets,
  // group g belongs to XCD g % 8, so that B is fetched into one L2 only, and the workgroups of an XCD draw
  // its items from a shared counter (wave 0 draws, LDS broadcasts; the staging area is quiet between
  // items): items cost 4 to 6 chunks of work depending on the expert's rows, and a fixed assignment leaves
  // some workgroups 5-8 % more than the mean.  Without tickets: fixed round-robin assignment.
  const int xcd = blockIdx.x & 7;
  const int n_groups = p.E_local * n_split;
  const int groups_x = n_groups > xcd ? (n_groups - xcd + 7) >> 3 : 0;
  volatile int* s_box = reinterpret_cast<volatile int*>(smem);
  for (int it = 0;; ++it) {
    int e, sp, mp;
    if (p.tickets) {
      if (wave == 0) s_box[0] = (int)wave_atomic_add(&p.tickets[xcd], 1u);
      __syncthreads();
      const int ticket = __builtin_amdgcn_readfirstlane(s_box[0]);
      __syncthreads();
      const int k = ticket / n_mp;
      if (k >= groups_x) break;
      const int g = xcd + 8 * k;
      e = __builtin_amdgcn_readfirstlane(g / n_split);
      sp = g - e * n_split;
      mp = ticket - k * n_mp;
    } else {
      if (it * G >= total) break;
      const int id = xcd_tile_id(it, blockIdx.x, G);
      if (id >= total) continue;
      // items of one expert and column range are neighbours: they share the B chunks through the L2
      e = __builtin_amdgcn_readfirstlane(id / per_e);
      const int r = id - e * per_e;
      sp = __builtin_amdgcn_readfirstlane(r / n_mp);
      mp = r - sp * n_mp;
    }
    const int seg0 = __builtin_amdgcn_readfirstlane(p.offsets[e]);
    const int cnt = __builtin_amdgcn_readfirstlane(p.offsets[e + 1]) - seg0;
    if (cnt > kWpMaxRows) continue;

    WpCtx t;
    t.wave = wave;
    t.kk = lane >> 4;
    t.k_rows = cnt;
    t.NT = NT;
    t.lda_bytes = p.lda * 2;
    t.ldb_bytes = p.ldb * 2;
    t.gathered = p.gather != nullptr;
    t.a_base = uniform_ptr(reinterpret_cast<const char*>(t.gathered ? p.A : p.A + (size_t)seg0 * p.lda));
    t.b_base = uniform_ptr(reinterpret_cast<const char*>(p.B + (size_t)seg0 * p.ldb));
    t.a_rows = (const __attribute__((address_space(3))) uint32_t*)(smem + kWpTokOff);
    if (t.gathered) {
      // every item closes with a barrier, so nobody still reads the previous item's table
      if ((int)threadIdx.x < cnt)
        ((__attribute__((address_space(3))) uint32_t*)(smem + kWpTokOff))[threadIdx.x] =
            (uint32_t)p.gather[seg0 + threadIdx.x] * (uint32_t)(p.lda * 2);
      __syncthreads();
    }
    t.a_col0 = mp * kWpM;
    t.b_col0 = sp * NT * kWpN;
    // lane -> (k-row kk of the line, position lane % 16) holds column chunk (position - 4*kk) mod 16
    t.lane_col = (uint32_t)((((lane & 15) - 4 * t.kk) & 15) * 16);
    t.lds0 = lds_addr_of(smem);
    t.c_base = p.C + (size_t)e * p.strideC;
    t.ldc = p.ldc;
    {
      const int gq = lane >> 4, i = lane & 15, kk = i >> 2;
      auto tr_off = [&](int nb) {   // 32-column block starting at staged column nb of a 128-column entry
        const int j = (nb >> 3) + (gq & 1) * 2 + ((i & 3) >> 1);
        return (uint32_t)((gq >> 1) * 2 * kLine + kk * 256 + ((j + 4 * kk) & 15) * 16 + (i & 1) * 8);
      };
      t.a_rd = tr_off((wave & 3) * 32);
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) t.b_rd[nt] = tr_off(nt * 32);
    }
    const int row0 = mp * kWpM;
    switch ((cnt + kWpBK - 1) / kWpBK) {
      case 0: wp_item<0>(t, row0, smem); break;
      case 1: wp_item<1>(t, row0, smem); break;
      case 2: wp_item<2>(t, row0, smem); break;
      case 3: wp_item<3>(t, row0, smem); break;
      case 4: wp_item<4>(t, row0, smem); break;
      case 5: wp_item<5>(t, row0, smem); break;
      default: wp_item<6>(t, row0, smem); break;
    }
  }
}

}  // namespace moe
