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

// Operand layouts.  The forward GEMMs are "NN": activations [rows, K] k-contiguous,
// weights [K, N] n-contiguous.  The backward graph (Section 2.2, Figure 2b) adds
//   NT  act_grad / gate_grad: C[rows, N] = A[rows, K] * W_e[N, K]^T -- both operands
//       k-contiguous, so the weight tile is staged like an activation tile (8 rows x
//       64 k per line, XOR swizzle, plain 16-byte operand reads).
// The weight gradients (reduction over the expert's rows) have kernels of their own
// (wgrad_panel.h, wgrad_bf16.h); they share GemmParams and the epilogue staging.
enum GemmLayout { kLayNN = 0, kLayNT = 1 };
enum GemmEpilogue { kEpiStore = 0, kEpiSwiglu = 1, kEpiSwigluGrad = 2, kEpiScatter = 3 };

constexpr int kBM = 256;            // tile row capacity (one M tile of the tile map)
constexpr int kBN = 256;            // weight columns staged per tile
constexpr int kBK = 64;             // K step
constexpr int kRowGranule = 64;     // an expert's rows are dealt to its M tiles in units of this (two wave rows x 32)
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
// Rows a wide tile can take: 256 staged through LDS plus, per wave row, one more 32-row block whose operand
// fragments the waves fetch straight from global memory into registers (see gemm_k_loop, NX).  An expert with
// 257..320 rows is then ONE wide tile: its weights stream once, its staged activation bytes per K step stay
// those of a 256-row tile, and the MFMA work grows by the real rows only.
constexpr int kWideRows = kBM + 64;
constexpr int kBLinesPerWave = kBLines / 4;          // 8

struct GemmParams {
  const __bf16* A;    // [rows, lda] activations, expert-contiguous rows, k-contiguous
  const __bf16* B;    // per expert [K, ldb] row-major weights
  __bf16* C;          // [rows, ldc]
  __bf16* C2;         // SwiGLU only: optional pre-activation [rows, 2N] (gate|up), else null
  const __bf16* G;    // SwiGLU-grad only: pre-activations saved by the forward [rows, 2N]
  const int32_t* gather;   // NN, optional: row r of the tile map is row gather[r] of A (A = the unpermuted tokens:
                           // the Dispatch permutation applied while loading, no permuted copy needed)
  // kEpiScatter (GEMM-2 with Combine in its epilogue, Section 4.4): row r of the tile map is added, times
  // sc_w[sc_token[r] * sc_k + sc_slot[r]], to row sc_token[r] of C (the layer output, zeroed beforehand)
  const int32_t* sc_token;
  const int32_t* sc_slot;
  const int32_t* sc_row_of;   // [T, sc_k]: a token with one local slot (one entry >= 0) gets a plain store
  const float* sc_w;
  int sc_k;
  long strideB;       // elements between consecutive experts' weights (NN, NT)
  long strideC;       // weight gradients: elements between consecutive experts' outputs
  int K, N;           // N = output columns (SwiGLU: I, weights have 2N columns); weight gradients: K unused (rows of the expert)
  int M;              // weight gradients: output rows
  int lda, ldb, ldc;
  int n_ntiles;       // ceil(N / 256) (SwiGLU: ceil(N / 128))
  int E_local;        // weight gradients
  int k_lo;           // weight gradients, general kernel: experts with fewer rows are left to the register-stationary kernel
  const int32_t* offsets;   // weight gradients: [E_local + 1] segment boundaries
  uint32_t* tickets;        // weight gradients, register-stationary kernel: 8 zeroed counters (one per XCD) from which
                            // the workgroups draw their items; nullptr = fixed round-robin assignment
  TileMap tiles;      // NN, NT
};

typedef short s16x4 __attribute__((ext_vector_type(4)));
// LDS is addressed through explicit address-space-3 pointers: a generic pointer
// would turn the operand reads into FLAT loads, which count on vmcnt and would
// drain the global -> LDS pipeline at every read.
typedef __attribute__((address_space(3))) const char* lds_cptr;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
typedef __attribute__((address_space(3))) const bf16x8* lds_bf16x8_cptr;

// s_waitcnt vmcnt(n) only (expcnt/lgkmcnt left at "don't wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// One wave-wide global -> LDS copy: lane l moves 16 bytes from sbase + voff to LDS
// byte address lds_addr + 16*l.  sbase and lds_addr must be wave-uniform values held
// in scalar registers (see uniform_ptr / uniform_u32).  Issued as inline assembly so
// that the compiler's own wait-count pass does not see an LDS write and force
// vmcnt(0) before every operand read (which would serialise the pipeline); ordering
// is done by hand with wait_vmcnt + s_barrier.  The "memory" clobber keeps LDS reads
// from moving across.
__device__ __forceinline__ void lds_dma16(const char* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(sbase)
               : "memory", "m0");
}

// One slice of the register-fed row block: lane (row l32, half lh) fetches the 16 bytes that are its MFMA operand
// for k slice KS of a K step (k = 16*KS + 8*lh .. +7).  Plain global load in assembly, so that the hand-kept
// vmcnt accounting of the pipeline covers it; the value is valid once a later wait has retired it.
template <int KS>
__device__ __forceinline__ void load_xblock(bf16x8& dst, const char* sbase, uint32_t voff) {
  asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(dst) : "v"(voff), "s"(sbase), "n"(KS * 32) : "memory");
}
// Retires the four fragments of a K step, behind which at most N memory operations have been issued (see
// gemm_k_loop); names the registers so that no use can be scheduled ahead of the wait.
template <int N>
__device__ __forceinline__ void wait_xblock(bf16x8 (&f)[4]) {
  asm volatile("s_waitcnt vmcnt(%4)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : "n"(N) : "memory");
}

// Pin a wave-uniform value into scalar registers (readfirstlane returns a signed
// int: widen through uint32_t, or the low half sign-extends into the high half).
__device__ __forceinline__ uint32_t uniform_u32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ const char* uniform_ptr(const char* p) {
  const uint64_t b = reinterpret_cast<uint64_t>(p);
  return reinterpret_cast<const char*>((uint64_t)uniform_u32((uint32_t)b) | ((uint64_t)uniform_u32((uint32_t)(b >> 32)) << 32));
}

__device__ __forceinline__ uint32_t lds_addr_of(const char* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// Tile shapes.  "Wide" is the default 256 rows x 256 staged weight columns (waves
// 2 x 2).  "Tall" is 384 rows x 128 columns (waves 4 x 1, up to 96 rows each): an
// expert with 257..384 rows is covered by ONE tall M tile, so its weights stream
// from HBM once instead of once per 256-row tile (two sibling tiles on neighbouring
// CUs do not share through the L2: the in-flight footprint of 32 CUs is most of its
// 4 MB).  Both shapes issue 16 wave-wide loads per wave per K step (8 + 8 or
// 12 + 4), so the pipeline and its wait counts are the same.
template <bool TALL>
struct TileShape {
  static constexpr int kRows = TALL ? 384 : 256;
  static constexpr int kCols = TALL ? 128 : 256;
  static constexpr int kALoads = TALL ? 12 : 8;             // A lines per wave per K step
  static constexpr int kBLoads = TALL ? 4 : 8;              // B lines per wave per K step
  static constexpr int kAStage = kALoads * 4 * kLine;       // 48 KB : 32 KB
  static constexpr int kBStage = kBLoads * 4 * kLine;       // 16 KB : 32 KB
  static constexpr int kBReg = kAStages * kAStage;          // weight stages start here
  static constexpr int kHalves = TALL ? 1 : 2;              // 128-column halves per 4-k-row group
  static_assert(kBReg + kBStages * kBStage <= kGemmLdsBytes, "LDS budget");
};
constexpr int kTallRows = TileShape<true>::kRows;

// Per-tile addressing state shared by the load and compute phases.
struct GemmTileCtx {
  const char* a_base;          // uniform: first row of the tile, byte address
  const char* b_base;          // uniform: expert's weights, byte address
  uint32_t a_off[12];          // per lane byte offset of the chunk fetched for the i-th A line
  uint32_t b_off[8];           // NN: per lane byte offset inside a 4-row line per column half; NT: like a_off
  uint32_t a_rd[4];            // operand read offset inside an A stage, per k slice
  uint32_t b_rd[4];            // operand read offset inside a B stage (NN: per 32-column block; NT: per k slice)
  uint32_t x_off;              // register-fed row block: per lane byte offset of (row, k half) inside the K step
  uint32_t lds0;               // LDS byte address of the staging area
  int nA;                      // A lines per wave per step
  int lda_bytes, ldb_bytes;
  int wave;
};

// The 16 wave-wide loads issued between two barriers: the A lines of one K step
// (indices 0..kALoads-1, only nA of them real) followed by the B lines of a
// later K step.  A loads always precede B loads, which the vmcnt waits rely on.
struct GemmLoadGroup {
  const char* a_k;   // uniform source of the A lines, nullptr = none
  const char* b_k;   // uniform source of the B lines, nullptr = none
  uint32_t a_st;     // uniform LDS address of this wave's first A line
  uint32_t b_st;     // uniform LDS address of this wave's first B line
};

template <int LAY, bool TALL>
__device__ __forceinline__ GemmLoadGroup gemm_load_group(const GemmTileCtx& t, int a_step, int a_stage, int b_step,
                                                         int b_stage) {
  typedef TileShape<TALL> S;
  GemmLoadGroup g;
  g.a_k = a_step >= 0 ? uniform_ptr(t.a_base + (size_t)a_step * (kBK * 2)) : nullptr;
  g.a_st = uniform_u32(t.lds0 + a_stage * S::kAStage + t.wave * kLine);
  if (LAY == kLayNT) g.b_k = b_step >= 0 ? uniform_ptr(t.b_base + (size_t)b_step * (kBK * 2)) : nullptr;
  else g.b_k = b_step >= 0 ? uniform_ptr(t.b_base + (size_t)(b_step * kBK + t.wave * 16) * t.ldb_bytes) : nullptr;
  if (LAY == kLayNT) g.b_st = uniform_u32(t.lds0 + S::kBReg + b_stage * S::kBStage + t.wave * kLine);
  else g.b_st = uniform_u32(t.lds0 + S::kBReg + b_stage * S::kBStage + t.wave * S::kBLoads * kLine);
  return g;
}

template <int LAY, bool TALL>
__device__ __forceinline__ void gemm_issue_one(const GemmTileCtx& t, const GemmLoadGroup& g, int idx) {
  typedef TileShape<TALL> S;
  if (idx < S::kALoads) {
    if (g.a_k != nullptr && idx < t.nA) lds_dma16(g.a_k, t.a_off[idx], g.a_st + 4 * idx * kLine);
  } else {
    const int i = idx - S::kALoads;
    if (g.b_k == nullptr) return;
    if (LAY == kLayNN) {
      // line i of this wave: k-row group i / halves, column half i % halves
      lds_dma16(g.b_k + (size_t)((i / S::kHalves) * 4) * t.ldb_bytes, t.b_off[i % S::kHalves], g.b_st + i * kLine);
    } else {
      lds_dma16(g.b_k, t.b_off[i], g.b_st + 4 * i * kLine);
    }
  }
}

// MFMA operands of one 16-wide k slice: 4 weight-side fragments and NMT
// activation-side fragments.  An operand staged n-/m-contiguous takes two
// transpose reads per fragment, a k-contiguous one a single 16-byte read.
template <int LAY, int NMT>
struct GemmFrags {
  s16x4 w[4][2];                       // NN
  bf16x8 wk[4];                        // NT
  bf16x8 xf[NMT > 0 ? NMT : 1];
};

template <int LAY, int NMT>
struct GemmSliceShape {
  static constexpr int n_wreads = LAY == kLayNT ? 4 : 8;
  static constexpr int n_xreads = NMT;
  static constexpr int n_reads = n_wreads + n_xreads;
};

// Operand read number `a` of slice ks from the stages as / bs into f.
template <int LAY, int NMT, bool TALL>
__device__ __forceinline__ void gemm_read_one(GemmFrags<LAY, NMT>& f, int a, lds_cptr as, lds_cptr bs, int ks,
                                              const GemmTileCtx& t) {
  typedef GemmSliceShape<LAY, NMT> S;
  constexpr int H = TileShape<TALL>::kHalves;   // lines per 4-k-row group of the weight stage
  if (a < S::n_wreads) {
    if (LAY == kLayNT) f.wk[a] = *(lds_bf16x8_cptr)(bs + t.b_rd[ks] + a * 4 * kLine);
    else
      f.w[a >> 1][a & 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4_ptr)(bs + t.b_rd[a >> 1] + ks * 4 * H * kLine + (a & 1) * H * kLine));
  } else {
    const int i = a - S::n_wreads;
    f.xf[i] = *(lds_bf16x8_cptr)(as + t.a_rd[ks] + i * 4 * kLine);
  }
}

__device__ __forceinline__ bf16x8 join_tr(s16x4 lo, s16x4 hi) {
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  return __builtin_bit_cast(bf16x8, (s16x8){lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w});
}

// One 16-wide k slice for a wave: (NMT + NX) x 4 MFMAs on `cur` (NX = 1: the last row block's activation
// fragment is `xblk`, held in registers).  Behind the MFMAs, one per slot, go the operand reads that fill `nxt`
// (slice ks_n of the stages as_n / bs_n) and four of the load group's global -> LDS copies, so LDS latency
// and load issue hide under MFMA time.  sched_barrier pins that order.
// The accumulators of the register-fed block live in architectural VGPRs (the 256 accumulation registers hold the
// four staged blocks), which only an assembly statement with register-class constraints can pin: left to
// the register allocator the fifth block's accumulators wander between the two files, 64 moves per slice.
__device__ __forceinline__ void mfma_vgpr_acc(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

template <int LAY, int NMT, bool TALL, int NX = 0>
__device__ __forceinline__ void gemm_slice(f32x16 (&acc)[kMaxMT][4], const GemmFrags<LAY, NMT>& cur,
                                           GemmFrags<LAY, NMT>& nxt, bool read_next, lds_cptr as_n, lds_cptr bs_n,
                                           int ks_n, const GemmTileCtx& t, const GemmLoadGroup& g, int load0,
                                           f32x16 (&accx)[4], const bf16x8& xblk) {
  typedef GemmSliceShape<LAY, NMT> S;
  constexpr int n_mfma = (NMT + NX) * 4, n_act = S::n_reads + 4;
  bf16x8 wf[4], xf[NMT > 0 ? NMT : 1];
#pragma unroll
  for (int nt = 0; nt < 4; ++nt) wf[nt] = LAY == kLayNT ? cur.wk[nt] : join_tr(cur.w[nt][0], cur.w[nt][1]);
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt) xf[mt] = cur.xf[mt];
#pragma unroll
  for (int j = 0; j < n_mfma; ++j) {
    if (j < NMT * 4) acc[j >> 2][j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j & 3], xf[j >> 2], acc[j >> 2][j & 3], 0, 0, 0);
    else mfma_vgpr_acc(accx[j & 3], wf[j & 3], xblk);
#pragma unroll
    for (int a = 0; a < n_act; ++a) {
      if ((a * n_mfma) / n_act != j) continue;
      if (a < S::n_reads) {
        if (read_next) gemm_read_one<LAY, NMT, TALL>(nxt, a, as_n, bs_n, ks_n, t);
      } else {
        gemm_issue_one<LAY, TALL>(t, g, load0 + (a - S::n_reads));
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int LAY, int NMT, bool TALL>
__device__ __forceinline__ void gemm_read_frags(GemmFrags<LAY, NMT>& f, lds_cptr as, lds_cptr bs, int ks,
                                                const GemmTileCtx& t) {
#pragma unroll
  for (int a = 0; a < GemmSliceShape<LAY, NMT>::n_reads; ++a) gemm_read_one<LAY, NMT, TALL>(f, a, as, bs, ks, t);
}

// K loop of one tile for a wave with NMT active row sub-tiles.
//
// Step s computes from A stage s%2 and B stage s%3.  Its barrier sits in front of
// the LAST k slice: by then this wave has fetched all of step s's operands
// (lgkmcnt 0), and the wait allows only the B loads of B(s+2) to be outstanding,
// so A(s+1) and B(s+1) are in LDS.  After the barrier that holds for every wave:
// the stages of step s are free and are refilled by the next load group, A(s+2)
// then B(s+3), issued four at a time behind the MFMAs of the following four
// slices, while the first operands of step s+1 are already being read under the
// last slice of step s.
//
// NX = 1 (wide tiles of 257..320 rows, NMT = 4): this wave also owns a fifth 32-row block whose
// activation fragments bypass LDS: four 16-byte loads per lane and K step, straight into the MFMA operand
// layout.  The fragments of step s + 1 are requested at the top of step s, ahead of that step's copies in the
// wave's in-order stream of memory operations, so the barrier's wait of step s (which retires everything
// older than the last 8 copies) has retired them too: three slices of load-to-use distance and no change to
// the pipeline's wait counts.  The loads are assembly with register outputs, i.e. the registers are written
// behind the compiler's back until a wait has retired them; the window from request to retirement therefore
// lies inside ONE loop trip (a value carried around the loop may be copied by the compiler at the back
// edge, which must only happen to retired values) and ends, right behind the barrier's wait, in a statement
// that names the registers, so that the compiler can neither use nor copy them earlier.
template <int LAY, int NMT, bool TALL, int NX = 0>
__device__ __forceinline__ void gemm_k_loop(f32x16 (&acc)[kMaxMT][4], f32x16 (&accx)[4], const GemmTileCtx& t, char* smem,
                                            int n_steps) {
  typedef TileShape<TALL> S;
  static_assert(NX == 0 || (NMT == kMaxMT && !TALL), "the register-fed block extends a full wide tile");
  const lds_cptr lds = (lds_cptr)smem;
  if (n_steps <= 0) return;
  bf16x8 xb[4], xn[4];                           // register-fed block: one fragment per k slice; this step's, next step's
  auto load_x = [&](bf16x8 (&f)[4], int step) __attribute__((always_inline)) {
    const char* base = uniform_ptr(t.a_base + (size_t)step * (kBK * 2));
    load_xblock<0>(f[0], base, t.x_off); load_xblock<1>(f[1], base, t.x_off);
    load_xblock<2>(f[2], base, t.x_off); load_xblock<3>(f[3], base, t.x_off);
  };
  if (NX) load_x(xb, 0);
  {
    const GemmLoadGroup g0 = gemm_load_group<LAY, TALL>(t, 0, 0, 0, 0);                       // A(0), B(0)
#pragma unroll
    for (int i = 0; i < 16; ++i) gemm_issue_one<LAY, TALL>(t, g0, i);
    if (n_steps > 1) {
      const GemmLoadGroup g1 = gemm_load_group<LAY, TALL>(t, -1, 0, 1, 1);                    // B(1)
#pragma unroll
      for (int i = S::kALoads; i < 16; ++i) gemm_issue_one<LAY, TALL>(t, g1, i);
      wait_vmcnt<S::kBLoads>();
    } else {
      wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    if (NX) wait_xblock<S::kBLoads>(xb);   // already retired by the wait above: this one names the registers
  }
  GemmLoadGroup g = gemm_load_group<LAY, TALL>(t, n_steps > 1 ? 1 : -1, 1, n_steps > 2 ? 2 : -1, 2);   // A(1), B(2)
#pragma unroll
  for (int i = 0; i < 4; ++i) gemm_issue_one<LAY, TALL>(t, g, i);
  GemmFrags<LAY, NMT> cur, nxt;
  if (NMT > 0) gemm_read_frags<LAY, NMT, TALL>(cur, lds, lds + S::kBReg, 0, t);

  int bs_i = 0;
  for (int s = 0; s < n_steps; ++s) {
    const lds_cptr as = lds + (s & 1) * S::kAStage;
    const lds_cptr bs = lds + S::kBReg + bs_i * S::kBStage;
    const int bs_next = bs_i == kBStages - 1 ? 0 : bs_i + 1;
    const bool more = s + 1 < n_steps;
    if (NX && more) load_x(xn, s + 1);
#pragma unroll
    for (int ks = 0; ks < 3; ++ks) {
      if (NMT > 0) {
        gemm_slice<LAY, NMT, TALL, NX>(acc, cur, nxt, true, as, bs, ks + 1, t, g, 4 + 4 * ks, accx, xb[ks]);
        cur = nxt;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) gemm_issue_one<LAY, TALL>(t, g, 4 + 4 * ks + i);
      }
    }
    if (more) {
      wait_lgkmcnt0();
      if (s + 2 < n_steps) wait_vmcnt<S::kBLoads>(); else wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      // the next step's fragments are older than the copies the wait above lets pass: retired; from this
      // statement on (it names the registers) they are ordinary values
      if (NX) wait_xblock<S::kBLoads>(xn);
      g = gemm_load_group<LAY, TALL>(t, s + 2 < n_steps ? s + 2 : -1, s & 1, s + 3 < n_steps ? s + 3 : -1, bs_i);
    }
    if (NMT > 0) {
      // `more` false: no loads left (both sources null) and nothing further to read
      gemm_slice<LAY, NMT, TALL, NX>(acc, cur, nxt, more, lds + ((s + 1) & 1) * S::kAStage,
                                     lds + S::kBReg + bs_next * S::kBStage, 0, t, g, 0, accx, xb[3]);
      if (more) cur = nxt;
    } else if (more) {
#pragma unroll
      for (int i = 0; i < 4; ++i) gemm_issue_one<LAY, TALL>(t, g, i);
    }
    if (NX && more) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) xb[ks] = xn[ks];
    }
    bs_i = bs_next;
  }
  if (NX) asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");   // the last assembly MFMA's result before any read of it
  __builtin_amdgcn_s_barrier();   // all stages free before the next tile's first loads
}

// Epilogue staging.  The MFMA result layout gives a lane 4 consecutive columns of
// one row, so a direct store writes 16-byte pieces of 32 different rows: partial
// lines, which the L2 completes by fetching the rest of each line from HBM (seen as
// ~0.9 GB of extra fetches on a 1.4 GB weight-gradient write).  Instead each wave
// parks a 32-row block in its own LDS region and writes it back out row-contiguous,
// 16 bytes per lane, whole 128-byte lines.  No cross-wave synchronisation: a wave
// only touches its own region, and LDS operations of one wave complete in order.
// The regions lie at 128..154 KB and 48..57 KB of the staging area: the next tile's
// first loads (activation stage 0, weight stages 0 and 1: wide 0..32 KB and
// 64..128 KB, tall 0..48 KB and 96..128 KB) do not touch them before its first
// barrier, whichever shape it has.
constexpr int kEpiRowBytes = 256 + 16;                 // 128 columns + padding against bank alignment of the rows
constexpr int kEpiWaveBytes = 32 * kEpiRowBytes;       // 8704

__device__ __forceinline__ char* epilogue_region(char* smem, int wave) {
  return wave < 3 ? smem + 128 * 1024 + wave * kEpiWaveBytes : smem + 48 * 1024;
}

// pk[nt][q]: this lane's 4 packed columns nt*32 + q*8 + (lane/32)*4 .. +3 of row lane%32.
// Writes rows [0, rows_valid) x columns [0, cols_valid) of the block to gdst (row stride ld elements).
// SPLIT: the block is two half-blocks side by side (NB/2 groups of 32 columns each) that go to different places,
// the left half to gdst, the right half to gdst2, cols_valid columns of each (SwiGLU: the gate and the up half of
// the stored pre-activations, one LDS round trip for both).
// All reads back from the region are issued before the first store, and the stores are predicated, not branched
// around: one LDS latency per call instead of one per row group.
template <int NB, bool NT = false, bool SPLIT = false>
__device__ __forceinline__ void store_block_via_lds(char* region, const u32x2 (&pk)[NB][4], __bf16* gdst, long ld,
                                                    int rows_valid, int cols_valid, __bf16* gdst2 = nullptr) {
  typedef __attribute__((address_space(3))) char* lds_ptr;
  typedef __attribute__((address_space(3))) u32x2* lds_u32x2_ptr;
  typedef __attribute__((address_space(3))) const u32x4* lds_u32x4_cptr;
  constexpr int LPR = NB * 4;                           // lanes per row at 16 bytes each
  constexpr int RPI = kWave / LPR, NIT = 32 / RPI;      // rows per access, accesses
  // The lane id passes through an empty asm so that nothing derived from it here counts as
  // loop-invariant: hoisted out of the tile loop, the per-row addresses and bounds were spilled
  // and every reload (s_waitcnt vmcnt(0)) waited for all earlier global stores as well.
  int lane = lane_id();
  asm volatile("" : "+v"(lane));
  const int l32 = lane & 31, lh = lane >> 5;
  const lds_ptr base = (lds_ptr)region;
#pragma unroll
  for (int nt = 0; nt < NB; ++nt)
#pragma unroll
    for (int q = 0; q < 4; ++q) *(lds_u32x2_ptr)(base + l32 * kEpiRowBytes + (nt * 32 + q * 8 + lh * 4) * 2) = pk[nt][q];
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const int row_l = lane / LPR, ch = lane % LPR;
  const int chh = SPLIT ? ch % (LPR / 2) : ch;           // 16-byte chunk inside the (half-)block
  const bool col_ok = chh * 8 < cols_valid;
  __bf16* gp = (SPLIT && ch >= LPR / 2 ? gdst2 : gdst) + (size_t)row_l * ld + chh * 8;
  const lds_ptr lp = base + row_l * kEpiRowBytes + ch * 16;
  u32x4 v[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) v[it] = *(lds_u32x4_cptr)(lp + it * RPI * kEpiRowBytes);
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    if (it * RPI + row_l < rows_valid && col_ok) {
      u32x4* dst = reinterpret_cast<u32x4*>(gp + (size_t)(it * RPI) * ld);
      if (NT) __builtin_nontemporal_store(v[it], dst);
      else *dst = v[it];
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Combine in the epilogue (Section 4.4: the result rows never make the round trip through HBM as a permuted
// tensor).  The block is staged like a stored block; then each of its rows goes out as ONE wave-wide packed-bf16
// atomic add, lane l adding columns 2l, 2l + 1 of the row to the token's output row: whole 128-byte lines per
// instruction, device scope, no return value.  tok: the token of this lane's row l32 (lanes r and r + 32 agree).
// Several expert rows of one token may meet in any order, and every add rounds to bf16: results are equal to the
// fixed-order Combine only up to that rounding.
// one: bit r set = the token of row r has no other row on this GPU; the add into its zeroed output row is then
// a plain store (no read-modify-write, and bit-reproducible).
__device__ __forceinline__ void scatter_block_via_lds(char* region, const u32x2 (&pk)[4][4], __bf16* out, long ld,
                                                      int tok, uint32_t one, int rows_valid, int cols_valid) {
  typedef __attribute__((address_space(3))) char* lds_ptr;
  typedef __attribute__((address_space(3))) u32x2* lds_u32x2_ptr;
  typedef __attribute__((address_space(3))) const uint32_t* lds_u32_cptr;
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef __attribute__((address_space(1))) bf16x2* global_bf16x2_ptr;
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
  uint32_t v[32];
#pragma unroll
  for (int r = 0; r < 32; ++r) v[r] = *(lds_u32_cptr)(base + r * kEpiRowBytes + lane * 4);
  const bool col_ok = lane * 2 < cols_valid;
#pragma unroll
  for (int r = 0; r < 32; ++r) {
    if (r < rows_valid) {                                        // wave-uniform
      const int tr = __builtin_amdgcn_readlane(tok, r);
      __bf16* dst = out + (size_t)tr * ld + lane * 2;
      if (one >> r & 1) {                                          // wave-uniform
        if (col_ok) *reinterpret_cast<uint32_t*>(dst) = v[r];
      } else if (col_ok) {
        __builtin_amdgcn_global_atomic_fadd_v2bf16((global_bf16x2_ptr)dst, __builtin_bit_cast(bf16x2, v[r]));
      }
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// One output tile: (t0, t1) = (M tile of the tile map, N tile of TileShape<TALL>::kCols
// columns; SwiGLU: half as many output columns).  X5: a wide tile of 257..320 rows (rows past 256 go
// through the register-fed block of each wave row).
template <int LAY, int EPI, bool TALL, int X5 = 0>
__device__ __forceinline__ void gemm_tile_bf16(const GemmParams& p, int t0, int t1, char* smem) {
  typedef TileShape<TALL> S;
  static_assert(!(TALL && X5), "one shape at a time");
  const int tid = threadIdx.x;
  // opaque to the optimiser: per-lane setup is recomputed per tile instead of being hoisted out of
  // the tile loop and held (or spilled) across every K loop
  int lane = tid & 63;
  asm volatile("" : "+v"(lane));
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps branches and LDS bases scalar
  const int wm = wave >> 1, wn = TALL ? 0 : (wave & 1);
  const int l32 = lane & 31, lh = lane >> 5;

  // row_base: first tile row of this wave; n_mt: its 32-row blocks
  const int e = p.tiles.expert[t0], row0 = p.tiles.row0[t0], rows = p.tiles.rows[t0], ntile = t1;
  // rows per wave (row), a multiple of 32: tall = four wave rows, wide = two
  const int rows_lds = X5 ? kBM : rows;               // rows staged through LDS
  const int per = TALL ? ((((rows + 31) >> 5) + 3) >> 2) << 5 : ((rows_lds + 63) >> 6) << 5;
  const int row_base = (TALL ? wave : wm) * per;
  const int n_mt = (max(0, min(per, rows_lds - row_base)) + 31) >> 5;
  const int n_steps = p.K / kBK;
  const int x_row0 = kBM + wm * 32;                   // X5: first row of this wave row's register-fed block
  const bool has_x = X5 && rows > x_row0;             // wave-uniform

  GemmTileCtx t;
  t.wave = wave;
  const int kk4 = lane >> 4;          // k-row of this lane inside a 4-k-row line
  t.nA = (rows_lds + 31) >> 5;        // (8-row lines any operand read touches = 4*ceil(rows/32)) / 4 waves
  t.lda_bytes = p.lda * 2;
  t.ldb_bytes = p.ldb * 2;
  // chunk position -> k chunk of an 8-row x 64-k line: lane -> (row r = lane/8, position pos = lane%8) holds
  // k chunk pos ^ ((row/2)%8); line L = wave + 4*i, so (row/2)%8 = 4*(wave&1) + r/2
  const int kc_r = lane >> 3;
  const int kc_c = (lane & 7) ^ ((4 * (wave & 1) + (kc_r >> 1)) & 7);
  // 4-k-row x 128-column line: lane -> (k-row kk = lane/16, position pos = lane%16) holds column chunk pos - 4*kk
  const int tr_nl = (((lane & 15) - 4 * kk4) & 15) * 8;
  {
    const bool gathered = LAY == kLayNN && p.gather != nullptr;   // uniform
    t.a_base = uniform_ptr(reinterpret_cast<const char*>(gathered ? p.A : p.A + (size_t)row0 * p.lda));
    t.b_base = uniform_ptr(reinterpret_cast<const char*>(p.B + (size_t)e * p.strideB));
#pragma unroll
    for (int i = 0; i < S::kALoads; ++i) {
      const int row = min((wave + 4 * i) * 8 + kc_r, rows - 1);      // rows past the end re-read the last row; never stored
      // gathered: offsets are relative to the first token (the caller guarantees that A spans < 4 GB)
      const long arow = gathered ? (long)p.gather[row0 + row] : (long)row;
      t.a_off[i] = (uint32_t)((arow * p.lda + kc_c * 8) * 2);
    }
    if (X5) {
      const int row = min(x_row0 + l32, rows - 1);
      const long arow = gathered ? (long)p.gather[row0 + row] : (long)row;
      t.x_off = (uint32_t)((arow * p.lda + lh * 8) * 2);
    }
    if (LAY == kLayNT) {
#pragma unroll
      for (int i = 0; i < S::kBLoads; ++i) {
        const int n = min(ntile * S::kCols + (wave + 4 * i) * 8 + kc_r, p.N - 1);   // weight row = output column
        t.b_off[i] = (uint32_t)(((size_t)n * p.ldb + kc_c * 8) * 2);
      }
    } else if (TALL) {
      // one 128-column line per k-row group; SwiGLU: 64 gate columns then the 64 matching up columns
      int gcol;
      if (EPI == kEpiSwiglu) gcol = (tr_nl >> 6) * p.N + min(ntile * 64 + (tr_nl & 63), p.N - 8);
      else gcol = min(ntile * 128 + tr_nl, p.N - 8);
      t.b_off[0] = (uint32_t)((kk4 * p.ldb + gcol) * 2);
    } else {
#pragma unroll
      for (int nh = 0; nh < 2; ++nh) {
        int gcol;
        if (EPI == kEpiSwiglu) gcol = nh * p.N + min(ntile * (kBN / 2) + tr_nl, p.N - 8);   // half 0 = gate, 1 = up
        else gcol = min(ntile * kBN + nh * 128 + tr_nl, p.N - 8);
        t.b_off[nh] = (uint32_t)((kk4 * p.ldb + gcol) * 2);
      }
    }
  }

  // operand read offsets inside a stage
  t.lds0 = lds_addr_of(smem);
  {
    // k-contiguous stage: row m -> line m/8, 128 bytes per row, chunk swizzle by (m/2)%8
    const int f = (l32 >> 1) & 7;
    const uint32_t a0 = (uint32_t)((row_base >> 3) * kLine + (l32 >> 3) * kLine + (l32 & 7) * 128);
    const uint32_t w0 = (uint32_t)(((wn * 128) >> 3) * kLine + (l32 >> 3) * kLine + (l32 & 7) * 128);
    // transposing stage: 32-column block nb of the staged columns; a 4-k-row group is kHalves lines
    const int g = lane >> 4, i = lane & 15;
    const int kk = i >> 2;
    auto tr_off = [&](int nb, int halves) {
      const int j = ((nb & 127) >> 3) + (g & 1) * 2 + ((i & 3) >> 1);
      return (uint32_t)((g >> 1) * 2 * halves * kLine + (nb >> 7) * kLine + kk * 256 + ((j + 4 * kk) & 15) * 16 + (i & 1) * 8);
    };
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      t.a_rd[q] = a0 + (uint32_t)((((q * 2 + lh) ^ f) & 7) << 4);
      if (LAY == kLayNT) t.b_rd[q] = w0 + (uint32_t)((((q * 2 + lh) ^ f) & 7) << 4);
      else if (TALL) t.b_rd[q] = tr_off(q * 32, 1);
      else t.b_rd[q] = tr_off((EPI == kEpiSwiglu) ? (q >> 1) * 128 + wn * 64 + (q & 1) * 32 : wn * 128 + q * 32, 2);
    }
  }

  constexpr int kAccMT = kMaxMT + X5;
  f32x16 acc[kMaxMT][4], accx[4];   // accx: the register-fed fifth block (X5 only)
#pragma unroll
  for (int i = 0; i < kMaxMT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  if constexpr (X5) {
    // 256 staged rows: every wave row is full; the fifth block exists for wave row 0, and for wave row 1 above 288 rows
    if (has_x) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) accx[j][r] = 0.f;
      gemm_k_loop<LAY, kMaxMT, false, 1>(acc, accx, t, smem, n_steps);
    } else {
      gemm_k_loop<LAY, kMaxMT, false, 0>(acc, accx, t, smem, n_steps);
    }
  } else {
    switch (n_mt) {
      case 0: gemm_k_loop<LAY, 0, TALL>(acc, accx, t, smem, n_steps); break;
      case 1: gemm_k_loop<LAY, 1, TALL>(acc, accx, t, smem, n_steps); break;
      case 2: gemm_k_loop<LAY, 2, TALL>(acc, accx, t, smem, n_steps); break;
      case 3: gemm_k_loop<LAY, 3, TALL>(acc, accx, t, smem, n_steps); break;
      default:
        if constexpr (!TALL) gemm_k_loop<LAY, 4, TALL>(acc, accx, t, smem, n_steps);   // a tall wave row has at most 96 rows
        break;
    }
  }

  // ---- epilogue: lane holds row l32 of each 32 x 32 block and, per register group q,
  // the 4 consecutive columns q*8 + lh*4 .. +3; blocks leave through the wave's LDS region ----
  char* region = epilogue_region(smem, wave);
  // Scatter epilogue: token, routing weight and single-slot flag of this lane's row in every block, fetched before
  // the first block leaves (a load issued between the blocks would wait for all the adds in front of it: one
  // in-order counter per wave).
  int sc_tok[kAccMT];
  float sc_wt[kAccMT];
  uint32_t sc_one[kAccMT];
  if constexpr (EPI == kEpiScatter) {
#pragma unroll
    for (int mt = 0; mt < kAccMT; ++mt) {
      const int m0 = mt < kMaxMT ? row_base + mt * 32 : x_row0;
      const bool live = !(mt < kMaxMT ? mt >= n_mt : !has_x) && l32 < rows - m0;
      sc_tok[mt] = 0;
      sc_wt[mt] = 0.f;
      int others = 1;
      if (live) {
        const size_t r = (size_t)(row0 + m0 + l32);
        const int tok = p.sc_token[r], slot = p.sc_slot[r];
        sc_tok[mt] = tok;
        sc_wt[mt] = p.sc_w[(size_t)tok * p.sc_k + slot];
        others = 0;
        for (int j = 0; j < p.sc_k; ++j) others += (j != slot && p.sc_row_of[(size_t)tok * p.sc_k + j] >= 0) ? 1 : 0;
      }
      sc_one[mt] = (uint32_t)__builtin_amdgcn_ballot_w64(others == 0);   // lanes r and r + 32 agree: the low half
    }
  }
#pragma unroll
  for (int mt = 0; mt < kAccMT; ++mt) {
    const int m0 = mt < kMaxMT ? row_base + mt * 32 : x_row0;   // first row of the block inside the tile
    const int rows_valid = min(32, rows - m0);
    if ((mt < kMaxMT ? mt >= n_mt : !has_x) || rows_valid <= 0) continue;      // wave-uniform
    const f32x16* am = mt < kMaxMT ? acc[mt < kMaxMT ? mt : 0] : accx;         // resolved at compile time (unrolled)
    const size_t grow0 = (size_t)(row0 + m0);
    const size_t grow = grow0 + l32;                  // this lane's row (may be past the end: never stored)
    if (EPI == kEpiSwiglu) {
      const int c0 = ntile * (S::kCols / 2) + wn * 64;   // this wave's 64 gate columns and the 64 matching up columns
      u32x2 pa[2][4], ph[4][4];                       // ph: the pre-activations, gate columns then up columns
#pragma unroll
      for (int ng = 0; ng < 2; ++ng)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float g[4], u[4], a[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            g[x] = am[ng][q * 4 + x];
            u[x] = am[ng + 2][q * 4 + x];
            a[x] = g[x] * sigmoid_bf16_(g[x]) * u[x];
          }
          pa[ng][q] = u32x2{pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3])};
          ph[ng][q] = u32x2{pack_bf16(g[0], g[1]), pack_bf16(g[2], g[3])};
          ph[ng + 2][q] = u32x2{pack_bf16(u[0], u[1]), pack_bf16(u[2], u[3])};
        }
      store_block_via_lds<2>(region, pa, p.C + grow0 * p.ldc + c0, p.ldc, rows_valid, p.N - c0);
      if (p.C2) {
        __bf16* h = p.C2 + grow0 * (size_t)(2 * p.N) + c0;
        store_block_via_lds<4, false, true>(region, ph, h, 2 * p.N, rows_valid, p.N - c0, h + p.N);
      }
    } else if (EPI == kEpiSwigluGrad) {
      // SwiGLU_grad on the act_grad tile (Section 2.2, Figure 2b): the accumulators hold dA; with the saved
      // pre-activations (g, u): d_gate = dA*u*s*(1 + g*(1 - s)), d_up = dA*g*s, s = sigmoid(g)
      const int c0 = ntile * S::kCols + wn * 128;
      u32x2 pdg[4][4], pdu[4][4];
      const bool row_ok = l32 < rows_valid;
      const __bf16* h = p.G + grow * (size_t)(2 * p.N);
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = c0 + nt * 32 + q * 8 + lh * 4;
          u32x2 gv = {0u, 0u}, uv = {0u, 0u};
          if (row_ok && c < p.N) {
            gv = *reinterpret_cast<const u32x2*>(h + c);
            uv = *reinterpret_cast<const u32x2*>(h + p.N + c);
          }
          const float g[4] = {bf16_lo(gv.x), bf16_hi(gv.x), bf16_lo(gv.y), bf16_hi(gv.y)};
          const float u[4] = {bf16_lo(uv.x), bf16_hi(uv.x), bf16_lo(uv.y), bf16_hi(uv.y)};
          float dg[4], du[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const float da = am[nt][q * 4 + x];
            const float sg = sigmoid_bf16_(g[x]);
            dg[x] = da * u[x] * sg * (1.f + g[x] * (1.f - sg));
            du[x] = da * g[x] * sg;
          }
          pdg[nt][q] = u32x2{pack_bf16(dg[0], dg[1]), pack_bf16(dg[2], dg[3])};
          pdu[nt][q] = u32x2{pack_bf16(du[0], du[1]), pack_bf16(du[2], du[3])};
        }
      __bf16* o = p.C + grow0 * p.ldc + c0;
      store_block_via_lds<4>(region, pdg, o, p.ldc, rows_valid, p.N - c0);
      store_block_via_lds<4>(region, pdu, o + p.N, p.ldc, rows_valid, p.N - c0);
    } else if (EPI == kEpiScatter) {
      const int c0 = ntile * S::kCols + wn * 128;
      const float w = sc_wt[mt];
      u32x2 pk[4][4];
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          pk[nt][q] = u32x2{pack_bf16(w * am[nt][q * 4 + 0], w * am[nt][q * 4 + 1]),
                            pack_bf16(w * am[nt][q * 4 + 2], w * am[nt][q * 4 + 3])};
      scatter_block_via_lds(region, pk, p.C + c0, p.ldc, sc_tok[mt], sc_one[mt], rows_valid, p.N - c0);
    } else {
      const int c0 = ntile * S::kCols + wn * 128;
      u32x2 pk[4][4];
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          pk[nt][q] = u32x2{pack_bf16(am[nt][q * 4 + 0], am[nt][q * 4 + 1]),
                            pack_bf16(am[nt][q * 4 + 2], am[nt][q * 4 + 3])};
      store_block_via_lds<4>(region, pk, p.C + grow0 * p.ldc + c0, p.ldc, rows_valid, p.N - c0);
    }
  }
}

// Shape of a tile of the M-tile map by its rows: wide up to 256, wide with the register-fed block up to 320,
// tall above (the map builder makes such tiles only with <= 384 rows and gives each a pair slot of its own).
__device__ __forceinline__ bool tile_is_tall(int rows) { return rows > kWideRows; }

template <int LAY, int EPI>
__device__ __forceinline__ void gemm_map_tile_bf16(const GemmParams& p, int mtile, int ntile, bool tall, char* smem) {
  if (tall) gemm_tile_bf16<LAY, EPI, true>(p, mtile, ntile, smem);
  else if (__builtin_amdgcn_readfirstlane(p.tiles.rows[mtile]) > kBM) gemm_tile_bf16<LAY, EPI, false, 1>(p, mtile, ntile, smem);
  else gemm_tile_bf16<LAY, EPI, false>(p, mtile, ntile, smem);
}

// Work item `rem` (0 .. 2*n_ntiles-1) of tile pair (m0, m0+1): a tall tile owns the whole slot as
// 2*n_ntiles narrow N tiles; otherwise the items alternate between the two siblings, N-tile-major.
// Returns false for an item that does not exist.
__device__ __forceinline__ bool pair_work_item(const GemmParams& p, int m0, int rem, int n_m, int out_cols_per_ntile,
                                               int& mtile, int& ntile, bool& tall) {
  tall = tile_is_tall(__builtin_amdgcn_readfirstlane(p.tiles.rows[m0]));   // scalar: the branch below contains barriers
  if (tall) {
    mtile = m0;
    ntile = rem;
    return ntile * (out_cols_per_ntile / 2) < p.N;
  }
  mtile = m0 + (rem & 1);
  ntile = rem >> 1;
  return mtile < n_m && __builtin_amdgcn_readfirstlane(p.tiles.rows[mtile]) > 0;
}

// Tile id for workgroup b in sweep `it` of a grid of G workgroups (G % 8 == 0).
// Workgroups are dealt to the 8 XCDs round-robin by id, so giving XCD x the
// contiguous ids [x*G/8, (x+1)*G/8) keeps tiles that share an operand panel
// (same M tile, neighbouring N tiles) behind the same L2.
__device__ __forceinline__ int xcd_tile_id(int it, int b, int G) {
  return it * G + (b & 7) * (G >> 3) + (b >> 3);
}

// Activation x weight GEMMs over the M-tile map.  The map lists M tiles in pairs
// (entries 2j, 2j+1: siblings of one expert where possible).  Pair j belongs to
// XCD j % 8 (workgroups are dealt to the XCDs round-robin by id); inside an XCD
// the work items run N-tile-major with the two siblings adjacent, so the CUs that
// stream the same weight panel do so at the same time behind the same L2.
template <int LAY, int EPI>
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void grouped_gemm_bf16_kernel(GemmParams p) {
  __shared__ __attribute__((aligned(1024))) char smem[kGemmLdsBytes];
  const int n_m = p.tiles.meta[kMetaMTiles];
  const int xcd = blockIdx.x & 7, lw = blockIdx.x >> 3, W = gridDim.x >> 3;
  const int n_pairs = (n_m + 1) >> 1;
  const int pairs_x = n_pairs > xcd ? (n_pairs - xcd + 7) >> 3 : 0;
  const int per_pair = 2 * p.n_ntiles;
  // The XCD's items are dealt to its W workgroups in rounds.  When the last round would leave at least half of
  // them without an item, its items are halved: each runs as two 128-column items in the tall shape (4 x 1 waves
  // over the same rows) on neighbouring workgroups, which takes ~0.6 of a full item instead of a whole round.
  const int n_items = pairs_x * per_pair;
  const int tail = n_items % W;
  const bool split_tail = tail > 0 && 2 * tail <= W;
  const int n_whole = split_tail ? n_items - tail : n_items;
  constexpr int kOutCols = EPI == kEpiSwiglu ? kBN / 2 : kBN;
  for (int i = lw; i < n_whole; i += W) {
    // the division runs on the vector ALU; pin the (uniform) results back into scalar registers
    const int pl = __builtin_amdgcn_readfirstlane(i / per_pair);
    const int rem = i - pl * per_pair;
    int mtile, ntile;
    bool tall;
    if (!pair_work_item(p, 2 * (pl * 8 + xcd), rem, n_m, kOutCols, mtile, ntile, tall)) continue;
    gemm_map_tile_bf16<LAY, EPI>(p, mtile, ntile, tall, smem);
  }
  if (split_tail && lw < 2 * tail) {
    const int i = n_whole + (lw >> 1), half = lw & 1;
    const int pl = __builtin_amdgcn_readfirstlane(i / per_pair);
    const int rem = i - pl * per_pair;
    int mtile, ntile;
    bool tall;
    if (pair_work_item(p, 2 * (pl * 8 + xcd), rem, n_m, kOutCols, mtile, ntile, tall)) {
      if (tall) {                                   // already a 128-column item
        if (half == 0) gemm_tile_bf16<LAY, EPI, true>(p, mtile, ntile, smem);
      } else if ((2 * ntile + half) * (kOutCols / 2) < p.N) {
        gemm_tile_bf16<LAY, EPI, true>(p, mtile, 2 * ntile + half, smem);
      }
    }
  }
}

}  // namespace moe
