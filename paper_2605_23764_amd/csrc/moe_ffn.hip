// Host side of the C ABI declared in include/moe_ffn.h: argument checks,
// workspace layout, and the launch sequences.  Everything is enqueued on the
// caller's stream; nothing here allocates device memory or synchronises.
#include "../../include/moe_ffn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>

#include "backward.h"
#include "common.h"
#include "gemm_bf16.h"
#include "gemm_f32.h"
#include "microbench.h"
#include "permute_combine.h"
#include "persistent.h"
#include "probe.h"
#include "route.h"
#include "wgrad_bf16.h"
#include "wgrad_panel.h"

using namespace moe;

namespace {

constexpr size_t kAlign = 256;
#if defined(MOE_SCHED_TRACE)
constexpr size_t kSchedTraceBytes = 8192 * 48;   // task time stamps behind the task tables
#else
constexpr size_t kSchedTraceBytes = 0;
#endif
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

inline int elem_bytes(const MoeShape& s) { return s.dtype == MOE_BF16 ? 2 : 4; }
inline int tile_bm(const MoeShape& s) { return s.dtype == MOE_BF16 ? kBM : kFBM; }
inline int tile_wide_max(const MoeShape& s) { return s.dtype == MOE_BF16 ? kWideRows : kFBM; }   // rows one wide M tile can take
// rows per PERMUTE task of the single launch: kPermRows, twice that for rows below 8 KB (a task's fixed cost, ticket
// and trigger, is a few us: T = 4096, H = 2048 ran 2 % faster with 32-row tasks, H = 7168 the same with 16 or 32)
inline int perm_task_rows(const MoeShape& s) { return (size_t)s.H * elem_bytes(s) >= 8192 ? kPermRows : 2 * kPermRows; }
inline long r_max(const MoeShape& s) { return (long)s.T * (s.k < s.E_local ? s.k : s.E_local); }
inline int n_sub(const MoeShape& s) { return (s.T + kSub - 1) / kSub; }
inline int n_groups(const MoeShape& s) { return (s.T + kChunk - 1) / kChunk; }
// pair slots of the tile map: a tall tile (> BM rows) takes two entries, a wide tile of a split expert has > BM/2 rows
inline long max_mtiles(const MoeShape& s) { return 2 * (r_max(s) / tile_bm(s)) + 2 * s.E_local + kMapSlack; }
inline int tile_tall(const MoeShape& s) { return s.dtype == MOE_BF16 ? kTallRows : 0; }
inline int gemm1_ntiles(const MoeShape& s) { return s.dtype == MOE_BF16 ? (s.I + kBN / 2 - 1) / (kBN / 2) : s.I / kFBN; }
inline int gemm2_ntiles(const MoeShape& s) { return s.dtype == MOE_BF16 ? (s.H + kBN - 1) / kBN : s.H / kFBN; }
inline long n_events(const MoeShape& s) { return kEvPerTile + 2 * max_mtiles(s); }
inline long max_tasks_per_queue(const MoeShape& s) {
  const long mq = (max_mtiles(s) + kNumXcd - 1) / kNumXcd + 2;   // tiles are dealt in pairs
  return mq * ((tile_wide_max(s) + kPermRows - 1) / kPermRows + gemm1_ntiles(s) + gemm2_ntiles(s) + 2) + kWave / 2;   // + a halved last round
}

int check_shape(const MoeShape* s) {
  if (!s) return MOE_ERR_INVALID_ARG;
  if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
  if (s->T < 0 || s->H <= 0 || s->I <= 0) return MOE_ERR_UNSUPPORTED_SHAPE;
  if (s->k < 1 || s->k > kMaxK || s->E < s->k || s->E > kMaxE) return MOE_ERR_UNSUPPORTED_SHAPE;
  if (s->E_local < 1 || s->E_local > kMaxE || s->expert_base < 0 || s->expert_base + s->E_local > s->E)
    return MOE_ERR_UNSUPPORTED_SHAPE;
  if (s->H % 64 || s->I % 64 || s->H > (1 << 18) || s->I > (1 << 18)) return MOE_ERR_UNSUPPORTED_SHAPE;
  // 32-bit row*stride products inside the row movers
  if ((double)r_max(*s) * (double)(2 * s->I > s->H ? 2 * s->I : s->H) * elem_bytes(*s) > 9.0e18)
    return MOE_ERR_UNSUPPORTED_SHAPE;
  return MOE_OK;
}

// Device workspace carved from one base pointer.
struct Layout {
  size_t meta, chunk_cnt, tile_expert, tile_row0, tile_rows, events, qhead, tasks;
  // fallback storage when the caller passes saved == NULL
  size_t topk_idx, topk_w, counts, offsets, row_of, token_of, slot_of, Xp, A, Yp;
  size_t fwd_total;
};

Layout make_layout(const MoeShape& s) {
  Layout L{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  const size_t Rm = (size_t)r_max(s), eb = (size_t)elem_bytes(s);
  L.meta = take(kMetaWords * 4);
  L.chunk_cnt = take((size_t)n_sub(s) * s.E_local * 4);
  L.tile_expert = take((size_t)max_mtiles(s) * 4);
  L.tile_row0 = take((size_t)max_mtiles(s) * 4);
  L.tile_rows = take((size_t)max_mtiles(s) * 4);
  L.events = take((size_t)n_events(s) * 4);
  L.qhead = take(kNumQueues * 4);
  L.tasks = take((size_t)kNumXcd * max_tasks_per_queue(s) * sizeof(TaskDesc) + kSchedTraceBytes);
  L.topk_idx = take((size_t)s.T * s.k * 4);
  L.topk_w = take((size_t)s.T * s.k * 4);
  L.counts = take((size_t)s.E_local * 4);
  L.offsets = take((size_t)(s.E_local + 1) * 4);
  L.row_of = take((size_t)s.T * s.k * 4);
  L.token_of = take(Rm * 4);
  L.slot_of = take(Rm * 4);
  L.Xp = take(Rm * s.H * eb);
  L.A = take(Rm * s.I * eb);
  L.Yp = take(Rm * s.H * eb);
  L.fwd_total = off;
  return L;
}

struct Ctx {
  MoeShape s;
  Layout L;
  char* ws;
  MoeSaved sv;      // resolved buffers (caller's or workspace fallback)
  hipStream_t stream;
  int n_cu;
  bool keep_xp;     // the caller passed MoeSaved with Xp: the permuted copy of x is an output
};

// No MoeSaved (inference) or MoeSaved without Xp (the backward then reads x through the permutation as
// well): nobody reads a permuted copy of x, so bf16 GEMM-1 applies the permutation while loading (32-bit
// offsets: x must span < 4 GB) and the PERMUTE step is dropped.
bool gathers_x(const Ctx& c) {
  return !c.keep_xp && c.s.dtype == MOE_BF16 && (size_t)c.s.T * c.s.H * 2 < ((size_t)1 << 32);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
// Single-launch modes hand tiles over between CUs behind one L2 without invalidating the CUs' vector L1;
// that is only sound if no 128-byte line is shared by two tasks' rows, i.e. if the buffers that are both
// written and read inside the launch start on a line boundary (rows are multiples of 128 bytes).
bool aligned128(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 127u) == 0; }

int device_cus() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (!cached[dev]) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

int make_ctx(Ctx& c, const MoeShape* shape, const MoeSaved* saved, void* ws, size_t ws_bytes, void* stream) {
  int st = check_shape(shape);
  if (st != MOE_OK) return st;
  c.s = *shape;
  c.L = make_layout(c.s);
  if (c.s.T == 0) return MOE_OK;   // nothing to do: callers return before touching any pointer
  if (!ws || !aligned16(ws)) return MOE_ERR_INVALID_ARG;
  if (ws_bytes < c.L.fwd_total) return MOE_ERR_WORKSPACE_TOO_SMALL;
  c.ws = static_cast<char*>(ws);
  c.stream = static_cast<hipStream_t>(stream);
  c.keep_xp = saved != nullptr && saved->Xp != nullptr;
  if (saved) {
    c.sv = *saved;
    const void* must[] = {saved->topk_idx, saved->topk_w, saved->counts, saved->offsets, saved->row_of,
                          saved->token_of, saved->slot_of, saved->A, saved->Yp};
    for (const void* q : must)
      if (!q || !aligned16(q)) return MOE_ERR_INVALID_ARG;
    if ((saved->H1 && !aligned16(saved->H1)) || (saved->Xp && !aligned16(saved->Xp))) return MOE_ERR_INVALID_ARG;
    if (!saved->Xp) c.sv.Xp = c.ws + c.L.Xp;   // scratch for the paths that cannot gather (fp32, x of 4 GB or more)
  } else {
    const Layout& L = c.L;
    c.sv.topk_idx = reinterpret_cast<int32_t*>(c.ws + L.topk_idx);
    c.sv.topk_w = reinterpret_cast<float*>(c.ws + L.topk_w);
    c.sv.counts = reinterpret_cast<int32_t*>(c.ws + L.counts);
    c.sv.offsets = reinterpret_cast<int32_t*>(c.ws + L.offsets);
    c.sv.row_of = reinterpret_cast<int32_t*>(c.ws + L.row_of);
    c.sv.token_of = reinterpret_cast<int32_t*>(c.ws + L.token_of);
    c.sv.slot_of = reinterpret_cast<int32_t*>(c.ws + L.slot_of);
    c.sv.Xp = c.ws + L.Xp;
    c.sv.H1 = nullptr;
    c.sv.A = c.ws + L.A;
    c.sv.Yp = c.ws + L.Yp;
  }
  c.n_cu = device_cus();
  return MOE_OK;
}

TileMap tile_map(const Ctx& c) {
  TileMap t;
  t.expert = reinterpret_cast<int32_t*>(c.ws + c.L.tile_expert);
  t.row0 = reinterpret_cast<int32_t*>(c.ws + c.L.tile_row0);
  t.rows = reinterpret_cast<int32_t*>(c.ws + c.L.tile_rows);
  t.meta = reinterpret_cast<int32_t*>(c.ws + c.L.meta);
  return t;
}

RouteParams route_params(const Ctx& c, const float* logits) {
  RouteParams p;
  p.logits = logits;
  p.topk_idx = c.sv.topk_idx; p.topk_w = c.sv.topk_w;
  p.counts = c.sv.counts; p.offsets = c.sv.offsets;
  p.row_of = c.sv.row_of; p.token_of = c.sv.token_of; p.slot_of = c.sv.slot_of;
  p.chunk_cnt = reinterpret_cast<int32_t*>(c.ws + c.L.chunk_cnt);
  p.tiles = tile_map(c);
  p.T = c.s.T; p.E = c.s.E; p.E_local = c.s.E_local; p.expert_base = c.s.expert_base; p.k = c.s.k;
  p.n_sub = n_sub(c.s);
  p.n_groups = n_groups(c.s);
  p.BM = tile_bm(c.s);
  p.granule = c.s.dtype == MOE_BF16 ? kRowGranule : kFBM;
  p.tall = tile_tall(c.s);
  p.wide_max = tile_wide_max(c.s);
  return p;
}

int launch_status() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH; }

PermuteParams permute_params(const Ctx& c, const void* x);

int run_permute(const Ctx& c, const void* x) {
  PermuteParams p = permute_params(c, x);
  long want = (r_max(c.s) + 3) / 4;
  int grid = (int)(want < (long)c.n_cu * 8 ? (want > 0 ? want : 1) : (long)c.n_cu * 8);
  hipLaunchKernelGGL(permute_kernel, dim3(grid), dim3(256), 0, c.stream, p);
  return launch_status();
}

int gemm_grid(const Ctx& c) { return (c.n_cu + 7) / 8 * 8; }

template <typename P, typename T>
P gemm1_params(const Ctx& c, const void* w_gate_up) {
  const MoeShape& s = c.s;
  P p{};
  p.A = static_cast<const T*>(c.sv.Xp); p.B = static_cast<const T*>(w_gate_up);
  p.C = static_cast<T*>(c.sv.A); p.C2 = static_cast<T*>(c.sv.H1);
  p.strideB = (long)s.H * 2 * s.I; p.K = s.H; p.N = s.I;
  p.lda = s.H; p.ldb = 2 * s.I; p.ldc = s.I;
  p.n_ntiles = gemm1_ntiles(s);
  p.tiles = tile_map(c);
  return p;
}

template <typename P, typename T>
P gemm2_params(const Ctx& c, const void* w_down) {
  const MoeShape& s = c.s;
  P p{};
  p.A = static_cast<const T*>(c.sv.A); p.B = static_cast<const T*>(w_down);
  p.C = static_cast<T*>(c.sv.Yp); p.C2 = nullptr;
  p.strideB = (long)s.I * s.H; p.K = s.I; p.N = s.H;
  p.lda = s.I; p.ldb = s.H; p.ldc = s.H;
  p.n_ntiles = gemm2_ntiles(s);
  p.tiles = tile_map(c);
  return p;
}

// x_gather: non-null = read the token rows of x through token_of instead of the permuted copy (bf16 only)
int run_gemm1(const Ctx& c, const void* w_gate_up, const void* x_gather = nullptr) {
  if (c.s.dtype == MOE_BF16) {
    GemmParams p = gemm1_params<GemmParams, __bf16>(c, w_gate_up);
    if (x_gather) {
      p.A = static_cast<const __bf16*>(x_gather);
      p.gather = c.sv.token_of;
    }
    hipLaunchKernelGGL((grouped_gemm_bf16_kernel<kLayNN, kEpiSwiglu>), dim3(gemm_grid(c)), dim3(kGemmThreads), 0, c.stream, p);
  } else
    hipLaunchKernelGGL(grouped_gemm_f32_kernel<kEpiSwiglu>, dim3(gemm_grid(c) * 4), dim3(256), 0, c.stream,
                       gemm1_params<GemmParamsF32, float>(c, w_gate_up));
  return launch_status();
}

int run_gemm2(const Ctx& c, const void* w_down) {
  if (c.s.dtype == MOE_BF16)
    hipLaunchKernelGGL((grouped_gemm_bf16_kernel<kLayNN, kEpiStore>), dim3(gemm_grid(c)), dim3(kGemmThreads), 0, c.stream,
                       gemm2_params<GemmParams, __bf16>(c, w_down));
  else
    hipLaunchKernelGGL(grouped_gemm_f32_kernel<kEpiStore>, dim3(gemm_grid(c) * 4), dim3(256), 0, c.stream,
                       gemm2_params<GemmParamsF32, float>(c, w_down));
  return launch_status();
}

// GEMM-2 with Combine in its epilogue: `out` is zeroed, then every result row is added, weighted, to its token's
// row (packed-bf16 atomics).  Yp is not written.  bf16 only.
int run_gemm2_scatter(const Ctx& c, const void* w_down, void* out, bool zeroed = false) {
  if (!zeroed) {
    const size_t n16 = (size_t)c.s.T * c.s.H * 2 / 16;
    const size_t want = (n16 + 255) / 256;
    const int grid = (int)(want < (size_t)c.n_cu * 8 ? (want > 0 ? want : 1) : (size_t)c.n_cu * 8);
    hipLaunchKernelGGL(zero_fill_kernel, dim3(grid), dim3(256), 0, c.stream, static_cast<uint4*>(out), n16);
  }
  GemmParams p = gemm2_params<GemmParams, __bf16>(c, w_down);
  p.C = static_cast<__bf16*>(out);
  p.sc_token = c.sv.token_of; p.sc_slot = c.sv.slot_of; p.sc_row_of = c.sv.row_of; p.sc_w = c.sv.topk_w; p.sc_k = c.s.k;
  hipLaunchKernelGGL((grouped_gemm_bf16_kernel<kLayNN, kEpiScatter>), dim3(gemm_grid(c)), dim3(kGemmThreads), 0, c.stream, p);
  return launch_status();
}

CombineParams combine_params(const Ctx& c, void* out) {
  CombineParams p;
  p.Yp = c.sv.Yp; p.out = out; p.row_of = c.sv.row_of; p.topk_w = c.sv.topk_w;
  p.T = c.s.T; p.H = c.s.H; p.k = c.s.k;
  return p;
}

PermuteParams permute_params(const Ctx& c, const void* x) {
  PermuteParams p;
  p.x = x; p.Xp = c.sv.Xp; p.token_of = c.sv.token_of;
  p.meta = reinterpret_cast<int32_t*>(c.ws + c.L.meta);
  p.H = c.s.H; p.elem_bytes = elem_bytes(c.s);
  return p;
}

// Polls a scheduler wait may spend before it gives up (each poll is an L2 round
// trip plus a short sleep: the default is several seconds).
uint32_t g_spin_limit = 1u << 20;

// Test hook: nonzero makes the single-launch schedulers behave as if every queue's workers had reported
// several XCDs (device-scope fences on every chain event).
int g_force_device_scope = 0;

// Two-stream backward: the events of its fork and join (dYp ready, dH1 ready, weight gradients done), made on a
// device's first such call and kept; calls hold the mutex while they enqueue, so that no other call's record of
// the same event comes between a record and the wait that refers to it.
constexpr int kMaxDevices = 16;
hipEvent_t g_fork_ev[kMaxDevices][3] = {};
std::mutex g_fork_mutex;

// Everything the scheduler's kernels need; pointers the caller does not have yet may be null (the routing
// launches only read the shapes, the tile counts and the table addresses).
template <bool BF16>
SchedParams<BF16> sched_params(const Ctx& c, const void* x, const float* logits, const void* w_gate_up, const void* w_down,
                               void* out) {
  using P = typename std::conditional<BF16, GemmParams, GemmParamsF32>::type;
  using T = typename std::conditional<BF16, __bf16, float>::type;
  SchedParams<BF16> sp;
  sp.route = route_params(c, logits);
  sp.perm = permute_params(c, x);
  sp.g1 = gemm1_params<P, T>(c, w_gate_up);
  sp.g2 = gemm2_params<P, T>(c, w_down);
  sp.comb = combine_params(c, out);
  sp.no_permute = 0;
  sp.skip_tables = 0;
  sp.zero_dst = nullptr;
  sp.zero_n16 = 0;
  if constexpr (BF16) {
    if (gathers_x(c)) {
      sp.g1.A = static_cast<const T*>(x);
      sp.g1.gather = c.sv.token_of;
      sp.no_permute = 1;
    }
  }
  sp.events = reinterpret_cast<uint32_t*>(c.ws + c.L.events);
  sp.qhead = reinterpret_cast<uint32_t*>(c.ws + c.L.qhead);
  sp.tasks = reinterpret_cast<TaskDesc*>(c.ws + c.L.tasks);
  sp.meta = reinterpret_cast<int32_t*>(c.ws + c.L.meta);
  sp.max_mtiles = (int)max_mtiles(c.s);
  sp.max_tasks_per_q = (int)max_tasks_per_queue(c.s);
  sp.n_events = (int)n_events(c.s);
  // COMBINE tasks of 32 tokens, halved (down to 4, one per wave) while there are fewer than four tasks per CU:
  // all of them become ready at the same moment, so small tasks are what balances the workers
  sp.comb_tokens = kCombineTokens;
#ifndef MOE_COMB_TASKS_PER_CU
#define MOE_COMB_TASKS_PER_CU 2
#endif
  while (sp.comb_tokens > 4 && (c.s.T + sp.comb_tokens - 1) / sp.comb_tokens < MOE_COMB_TASKS_PER_CU * c.n_cu) sp.comb_tokens >>= 1;
  sp.perm_rows = perm_task_rows(c.s);
  sp.workers_per_q = gemm_grid(c) / kNumXcd;
  sp.n_comb_tasks = (c.s.T + sp.comb_tokens - 1) / sp.comb_tokens;
  sp.force_device_scope = g_force_device_scope;
  sp.spin_limit = g_spin_limit;
  sp.timeout_status = MOE_ERR_SCHED_TIMEOUT;
  return sp;
}

// Routing, two launches: the router (top-k, softmax, per-chunk histograms), then prefix sums + M-tile map +
// stable ranks.  The second launch also zeroes the tile scheduler's counters and writes its task tables (one
// workgroup, beside the rank groups), so that either launch mode can follow.
template <bool BF16>
int run_route_t(const Ctx& c, const float* logits, bool tables, void* zero_out) {
  SchedParams<BF16> sp = sched_params<BF16>(c, nullptr, logits, nullptr, nullptr, nullptr);
  sp.skip_tables = tables ? 0 : 1;
  const RouteParams& rp = sp.route;
  int fill_wgs = 0;
  if (zero_out) {
    sp.zero_dst = static_cast<uint4*>(zero_out);
    sp.zero_n16 = (size_t)c.s.T * c.s.H * elem_bytes(c.s) / 16;
    const size_t want = (sp.zero_n16 + kScanRankWaves * kWave - 1) / (kScanRankWaves * kWave);
    fill_wgs = (int)(want < (size_t)c.n_cu * 4 ? want : (size_t)c.n_cu * 4);
  }
  hipLaunchKernelGGL(route_kernel, dim3(rp.n_sub), dim3(512), 0, c.stream, rp);
  hipLaunchKernelGGL(sched_prepare_kernel<BF16>, dim3(1 + (rp.n_groups + kScanRankWaves - 1) / kScanRankWaves + fill_wgs),
                     dim3(kScanRankWaves * kWave), 0, c.stream, sp);
  return launch_status();
}
// tables = false: the caller knows that one launch per operator follows (the task tables take workgroup 0 of the
// second launch, which is the launch's critical path, about as long again as the prefix sums and the tile map).
// zero_out: the layer output, zeroed by further workgroups of the second launch (scatter epilogue follows).
int run_route(const Ctx& c, const float* logits, bool tables = true, void* zero_out = nullptr) {
  return c.s.dtype == MOE_BF16 ? run_route_t<true>(c, logits, tables, zero_out)
                               : run_route_t<false>(c, logits, tables, zero_out);
}

// Dispatch to Combine as ONE launch of tile tasks (after run_route on the same MoeSaved).
template <bool BF16>
int run_persistent(const Ctx& c, const void* x, const void* w_gate_up, const void* w_down, void* out) {
  const SchedParams<BF16> sp = sched_params<BF16>(c, x, nullptr, w_gate_up, w_down, out);
  hipLaunchKernelGGL(persistent_forward_kernel<BF16>, dim3(gemm_grid(c)), dim3(kGemmThreads), 0, c.stream, sp);
  return launch_status();
}

// The same launch with Combine in the GEMM-2 tiles' epilogue (bf16; `out` zeroed by the routing launch).
int run_persistent_scatter(const Ctx& c, const void* x, const void* w_gate_up, const void* w_down, void* out) {
  SchedParams<true> sp = sched_params<true>(c, x, nullptr, w_gate_up, w_down, out);
  sp.g2.C = static_cast<__bf16*>(out);
  sp.g2.sc_token = c.sv.token_of; sp.g2.sc_slot = c.sv.slot_of; sp.g2.sc_row_of = c.sv.row_of;
  sp.g2.sc_w = c.sv.topk_w; sp.g2.sc_k = c.s.k;
  hipLaunchKernelGGL((persistent_forward_kernel<true, true>), dim3(gemm_grid(c)), dim3(kGemmThreads), 0, c.stream, sp);
  return launch_status();
}

int run_combine(const Ctx& c, void* out) {
  CombineParams p = combine_params(c, out);
  long want = ((long)c.s.T + 3) / 4;
  int grid = (int)(want < (long)c.n_cu * 8 ? want : (long)c.n_cu * 8);
  if (c.s.dtype == MOE_BF16)
    hipLaunchKernelGGL(combine_kernel<true>, dim3(grid), dim3(256), 0, c.stream, p);
  else
    hipLaunchKernelGGL(combine_kernel<false>, dim3(grid), dim3(256), 0, c.stream, p);
  return launch_status();
}

// ---- backward ----
struct BwdLayout {
  size_t meta, tile_expert, tile_row0, tile_rows, events, qhead, tasks, tickets, dYp, dH1, dXp, Xp, total;
};

BwdLayout make_bwd_layout(const MoeShape& s) {
  BwdLayout L{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  const size_t Rm = (size_t)r_max(s), eb = (size_t)elem_bytes(s);
  L.meta = take(kMetaWords * 4);
  L.tile_expert = take((size_t)max_mtiles(s) * 4);
  L.tile_row0 = take((size_t)max_mtiles(s) * 4);
  L.tile_rows = take((size_t)max_mtiles(s) * 4);
  L.events = take((size_t)n_events(s) * 4);                 // single-launch data-gradient chain
  L.qhead = take(kNumQueues * 4);
  L.tasks = take((size_t)kNumXcd * max_tasks_per_queue(s) * sizeof(TaskDesc));
  L.tickets = take(2 * kNumXcd * 4);                         // item counters of the two weight-gradient launches
  L.dYp = take(Rm * s.H * eb);
  L.dH1 = take(Rm * 2 * s.I * eb);
  L.dXp = take(Rm * s.H * eb);
  L.Xp = take(Rm * s.H * eb);                                // rows of Xp made here when the forward kept none
  L.total = off;
  return L;
}

struct BwdCtx {
  MoeShape s;
  BwdLayout L;
  char* ws;
  MoeSaved sv;
  hipStream_t stream;
  hipStream_t wgrad_stream;   // nullptr or == stream: everything on `stream`
  int n_cu;
  TileMap tiles;
  int mode;          // MOE_MODE_PERSISTENT: act_grad and gate_grad as one launch under the tile scheduler
};

// Weight gradient of one GEMM: experts with up to 384 rows go to the register-stationary kernel when
// the output splits into full 256 x 128 tiles, everything else to the general kernel.
bool wgrad_panel_fits(int M, int N) { return M % kWpM == 0 && N % kWpN == 0; }

// p.gather != nullptr: the register-stationary kernel reads the rows of p.A through it; the general kernel
// reads `a_general`, in which the caller has placed the rows of the experts that kernel takes.
void launch_wgrad_bf16(GemmParams p, int grid, int n_cu, hipStream_t stream, const __bf16* a_general = nullptr) {
  p.k_lo = 0;
  if (wgrad_panel_fits(p.M, p.N)) {
    // the kernel splits every expert's tile row into column ranges so that each CU gets about four items
    hipLaunchKernelGGL(grouped_wgrad_panel_bf16_kernel, dim3(grid), dim3(kWpThreads), 0, stream, p, 4 * n_cu);
    p.k_lo = kWpMaxRows + 1;
  }
  if (p.gather) { p.A = a_general; p.gather = nullptr; }
  hipLaunchKernelGGL(grouped_wgrad2_bf16_kernel, dim3(2 * grid), dim3(kGemmThreads), 0, stream, p);
}

template <typename T>
int run_backward(const BwdCtx& c, const void* dy, const void* x, const void* w_gate_up, const void* w_down, void* dx,
                 void* dw_gate_up, void* dw_down, float* d_topk_w) {
  constexpr bool BF16 = std::is_same<T, __bf16>::value;
  const MoeShape& s = c.s;
  T* dYp = reinterpret_cast<T*>(c.ws + c.L.dYp);
  T* dH1 = reinterpret_cast<T*>(c.ws + c.L.dH1);
  T* dXp = reinterpret_cast<T*>(c.ws + c.L.dXp);
  const int bm = tile_bm(s);
  const int tn = BF16 ? kBN : kFBN;
  auto ceil_div = [](int a, int b) { return (a + b - 1) / b; };
  const int grid = BF16 ? (c.n_cu + 7) / 8 * 8 : c.n_cu * 4;

  uint32_t* tickets = reinterpret_cast<uint32_t*>(c.ws + c.L.tickets);   // [0, 8): w2_grad, [8, 16): w1_grad

  // backward Dispatch; its extra workgroup rebuilds the M-tile map from the saved counts and zeroes the tickets
  BwdDispatchParams bd;
  bd.dY = dy; bd.Yp = c.sv.Yp; bd.dYp = dYp; bd.row_of = c.sv.row_of; bd.topk_w = c.sv.topk_w;
  bd.d_topk_w = d_topk_w; bd.T = s.T; bd.H = s.H; bd.k = s.k;
  bd.counts = c.sv.counts; bd.E_local = s.E_local; bd.wide_max = tile_wide_max(s); bd.granule = BF16 ? kRowGranule : kFBM;
  bd.tall = tile_tall(s); bd.tiles = c.tiles; bd.zero = tickets; bd.n_zero = 2 * kNumXcd;
  {
    long want = ((long)s.T + 3) / 4;
    int g = (int)(want < (long)c.n_cu * 8 ? want : (long)c.n_cu * 8);
    hipLaunchKernelGGL(bwd_dispatch_kernel<BF16>, dim3(g + 1), dim3(256), 0, c.stream, bd);
  }
  // Two streams: the weight-gradient branch of the graph (w2_grad behind the backward Dispatch, w1_grad behind
  // act_grad) is enqueued on its own stream, so that its workgroups take the CUs that the last tiles of the
  // data-gradient kernels leave idle, and the other way round; joined again before this function returns.
  const bool side = c.wgrad_stream != nullptr && c.wgrad_stream != c.stream;
  hipStream_t sw = side ? c.wgrad_stream : c.stream;
  hipEvent_t* ev = nullptr;
  std::unique_lock<std::mutex> fork_lock(g_fork_mutex, std::defer_lock);
  if (side) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_ERR_LAUNCH;
    fork_lock.lock();
    ev = g_fork_ev[dev];
    for (int i = 0; i < 3; ++i)
      if (!ev[i] && hipEventCreateWithFlags(&ev[i], hipEventDisableTiming) != hipSuccess) return MOE_ERR_LAUNCH;
    if (hipEventRecord(ev[0], c.stream) != hipSuccess || hipStreamWaitEvent(sw, ev[0], 0) != hipSuccess) return MOE_ERR_LAUNCH;
  }

  using P = typename std::conditional<BF16, GemmParams, GemmBwdParamsF32>::type;
  T* xp_ws = reinterpret_cast<T*>(c.ws + c.L.Xp);
  // act_grad + SwiGLU_grad: dH1 = swiglu'(dYp W_down^T ; H1)
  P pa{};
  pa.A = dYp; pa.B = static_cast<const T*>(w_down); pa.C = dH1; pa.G = static_cast<const T*>(c.sv.H1);
  pa.strideB = (long)s.I * s.H; pa.K = s.H; pa.N = s.I;
  pa.lda = s.H; pa.ldb = s.H; pa.ldc = 2 * s.I;
  pa.n_ntiles = ceil_div(s.I, tn);
  pa.tiles = c.tiles;
  // gate_grad: dXp = dH1 W_gate_up^T
  P pg{};
  pg.A = dH1; pg.B = static_cast<const T*>(w_gate_up); pg.C = dXp;
  pg.strideB = (long)s.H * 2 * s.I; pg.K = 2 * s.I; pg.N = s.H;
  pg.lda = 2 * s.I; pg.ldb = 2 * s.I; pg.ldc = s.H;
  pg.n_ntiles = ceil_div(s.H, tn);
  pg.tiles = c.tiles;

  // w2_grad: dW_down[e] = A_e^T dYp_e (needs only dYp: runs first, while dYp is fresh in the caches)
  auto launch_w2 = [&](hipStream_t st) {
    P p{};
    p.A = static_cast<const T*>(c.sv.A); p.B = dYp; p.C = static_cast<T*>(dw_down);
    p.strideC = (long)s.I * s.H; p.M = s.I; p.N = s.H;
    p.lda = s.I; p.ldb = s.H; p.ldc = s.H;
    p.n_ntiles = ceil_div(s.H, tn);
    if constexpr (!BF16) p.n_mtiles = ceil_div(s.I, bm);
    p.E_local = s.E_local; p.offsets = c.sv.offsets;
    if constexpr (BF16) { p.tickets = tickets; p.tiles = c.tiles; launch_wgrad_bf16(p, grid, c.n_cu, st); }
    else hipLaunchKernelGGL(grouped_wgrad_f32_kernel, dim3(grid), dim3(256), 0, st, p);
  };
  if (!side) launch_w2(c.stream);
  // called right behind the launch that completes dH1: w2_grad goes to the other stream, w1_grad may follow there
  auto fork_behind_dh1 = [&]() {
    if (!side) return true;
    launch_w2(sw);
    return hipEventRecord(ev[1], c.stream) == hipSuccess && hipStreamWaitEvent(sw, ev[1], 0) == hipSuccess;
  };
  if constexpr (BF16) {
    if (c.mode == MOE_MODE_PERSISTENT) {
      SchedParams<true> sp{};
      sp.route.tiles = c.tiles;
      sp.g1 = pa; sp.g2 = pg;
      sp.events = reinterpret_cast<uint32_t*>(c.ws + c.L.events);
      sp.qhead = reinterpret_cast<uint32_t*>(c.ws + c.L.qhead);
      sp.tasks = reinterpret_cast<TaskDesc*>(c.ws + c.L.tasks);
      sp.meta = c.tiles.meta;
      sp.max_mtiles = (int)max_mtiles(s);
      sp.max_tasks_per_q = (int)max_tasks_per_queue(s);
      sp.n_events = (int)n_events(s);
      sp.force_device_scope = g_force_device_scope;
      sp.perm_rows = perm_task_rows(s);
      sp.workers_per_q = grid / kNumXcd;
      sp.spin_limit = g_spin_limit;
      sp.timeout_status = MOE_ERR_SCHED_TIMEOUT;
      hipLaunchKernelGGL(dgrad_prepare_kernel, dim3(1), dim3(kGemmThreads), 0, c.stream, sp);
      hipLaunchKernelGGL(persistent_dgrad_kernel, dim3(grid), dim3(kGemmThreads), 0, c.stream, sp);
      if (!fork_behind_dh1()) return MOE_ERR_LAUNCH;
    } else {
      hipLaunchKernelGGL((grouped_gemm_bf16_kernel<kLayNT, kEpiSwigluGrad>), dim3(grid), dim3(kGemmThreads), 0, c.stream, pa);
      if (!fork_behind_dh1()) return MOE_ERR_LAUNCH;
      hipLaunchKernelGGL((grouped_gemm_bf16_kernel<kLayNT, kEpiStore>), dim3(grid), dim3(kGemmThreads), 0, c.stream, pg);
    }
  } else {
    hipLaunchKernelGGL(grouped_dgrad_f32_kernel<kEpiSwigluGrad>, dim3(grid), dim3(256), 0, c.stream, pa);
    if (!fork_behind_dh1()) return MOE_ERR_LAUNCH;
    hipLaunchKernelGGL(grouped_dgrad_f32_kernel<kEpiStore>, dim3(grid), dim3(256), 0, c.stream, pg);
  }
  // w1_grad: dW_gate_up[e] = Xp_e^T dH1_e.  When the forward kept no permuted copy (saved->Xp == NULL) the
  // register-stationary kernel reads x through the permutation and only the rows the general kernel needs are
  // copied first (all rows where nothing can gather).
  {
    P p{};
    p.A = static_cast<const T*>(c.sv.Xp); p.B = dH1; p.C = static_cast<T*>(dw_gate_up);
    p.strideC = (long)s.H * 2 * s.I; p.M = s.H; p.N = 2 * s.I;
    p.lda = s.H; p.ldb = 2 * s.I; p.ldc = 2 * s.I;
    p.n_ntiles = ceil_div(2 * s.I, tn);
    if constexpr (!BF16) p.n_mtiles = ceil_div(s.H, bm);
    p.E_local = s.E_local; p.offsets = c.sv.offsets;
    if (!c.sv.Xp) {
      PermuteParams pp;
      pp.x = x; pp.Xp = xp_ws; pp.token_of = c.sv.token_of; pp.meta = c.tiles.meta;
      pp.H = s.H; pp.elem_bytes = elem_bytes(s);
      const long want = ((long)r_max(s) + 3) / 4;
      const int g = (int)(want < (long)c.n_cu * 8 ? (want > 0 ? want : 1) : (long)c.n_cu * 8);
      bool gather = false;
      if constexpr (BF16) gather = (size_t)s.T * s.H * 2 < ((size_t)1 << 32);   // 32-bit row offsets
      if (gather) {
        // only the rows the general kernel will read: experts above the other kernel's limit, or all of them
        const int k_lo = wgrad_panel_fits(p.M, p.N) ? kWpMaxRows + 1 : 0;
        hipLaunchKernelGGL(permute_large_experts_kernel, dim3(g), dim3(256), 0, sw, pp, c.sv.offsets, s.E_local, k_lo);
        if constexpr (BF16) { p.A = static_cast<const T*>(x); p.gather = c.sv.token_of; }
      } else {
        hipLaunchKernelGGL(permute_kernel, dim3(g), dim3(256), 0, sw, pp);
        p.A = xp_ws;
      }
    }
    if constexpr (BF16) { p.tickets = tickets + kNumXcd; p.tiles = c.tiles; launch_wgrad_bf16(p, grid, c.n_cu, sw, xp_ws); }
    else hipLaunchKernelGGL(grouped_wgrad_f32_kernel, dim3(grid), dim3(256), 0, sw, p);
  }
  // backward Combine: dX[t] = sum over local slots of dXp[row_of[t,j]]
  {
    CombineParams p;
    p.Yp = dXp; p.out = dx; p.row_of = c.sv.row_of; p.topk_w = nullptr;
    p.T = s.T; p.H = s.H; p.k = s.k;
    long want = ((long)s.T + 3) / 4;
    int g = (int)(want < (long)c.n_cu * 8 ? want : (long)c.n_cu * 8);
    hipLaunchKernelGGL(combine_kernel<BF16>, dim3(g), dim3(256), 0, c.stream, p);
  }
  if (side && (hipEventRecord(ev[2], sw) != hipSuccess || hipStreamWaitEvent(c.stream, ev[2], 0) != hipSuccess))
    return MOE_ERR_LAUNCH;
  return launch_status();
}


// ---- SwiGLU + Add microbenchmark: host side shared by the two entry points ----
size_t mb_workspace_bytes(int M) {
  const size_t n = M > 0 ? (size_t)M : 0;
  return align_up(kMbRingBase * 4) + align_up(n * 4) + align_up((2 * n + 2 * kNumXcd) * 4);
}

int mb_check_args(int M, int N, const void* x, const void* y, const void* s, const void* out, int mode, int tile_rows,
                  const void* ws) {
  if (M < 0 || N <= 0 || N % 8 || mode < 0 || mode > 3 || tile_rows < 1 || tile_rows > kMbMaxTileRows)
    return MOE_ERR_INVALID_ARG;
  if (M == 0) return MOE_OK;
  const void* ptrs[] = {x, y, s, out, ws};
  for (const void* q : ptrs)
    if (!q || !aligned16(q)) return MOE_ERR_INVALID_ARG;
  // modes 1 and 3 hand S tiles over between CUs behind one L2 without touching the CUs' vector L1: a tile must
  // consist of whole 128-byte lines, or a CU could keep a line it read for one tile while its neighbour is written
  if ((mode == 1 || mode == 3) && (!aligned128(s) || ((size_t)tile_rows * N * 2) % 128 != 0)) return MOE_ERR_INVALID_ARG;
  return MOE_OK;
}

// `ws` holds mb_workspace_bytes(M) bytes; `status` = where the status word goes (nullptr: word 2 of ws).
int mb_launch(int M, int N, const void* d_x, const void* d_y, void* d_s, void* d_out, int mode, int tile_rows, void* ws,
              uint32_t* status, void* stream) {
  const int chk = mb_check_args(M, N, d_x, d_y, d_s, d_out, mode, tile_rows, ws);
  if (chk != MOE_OK || M == 0) return chk;
  MicrobenchParams p;
  p.X = static_cast<const __bf16*>(d_x); p.Y = static_cast<const __bf16*>(d_y);
  p.S = static_cast<__bf16*>(d_s); p.Out = static_cast<__bf16*>(d_out);
  p.M = M; p.N = N;
  p.tile_rows = tile_rows;
  p.n_tiles = (M + tile_rows - 1) / tile_rows;
  // rings are addressed relative to the header block, so they start behind the event counters
  p.queue = static_cast<uint32_t*>(ws);
  p.status = status ? status : p.queue + 2;
  p.events = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + align_up(kMbRingBase * 4));
  p.ring_base = (int)((align_up(kMbRingBase * 4) + align_up((size_t)M * 4)) / 4);
  p.spin_limit = g_spin_limit;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int workers = device_cus() * 4;   // four 256-thread workgroups per CU; a multiple of 8
  const int grid = p.n_tiles < workers ? (p.n_tiles + 7) / 8 * 8 : workers;
  if (mode == 0) {
    hipLaunchKernelGGL(mb_swiglu_kernel, dim3(grid), dim3(256), 0, st, p);
    hipLaunchKernelGGL(mb_add_kernel, dim3(grid), dim3(256), 0, st, p);
  } else {
    hipLaunchKernelGGL(mb_clear_kernel, dim3(std::min((p.n_tiles + 255) / 256, 1024)), dim3(256), 0, st, p,
                       mode == 3 ? kNumXcd : 1);
    if (mode == 1) hipLaunchKernelGGL(mb_static_kernel, dim3(grid), dim3(256), 0, st, p);
    else if (mode == 2) hipLaunchKernelGGL(mb_dynamic_kernel<false>, dim3(grid), dim3(256), 0, st, p);
    else hipLaunchKernelGGL(mb_dynamic_kernel<true>, dim3(grid), dim3(256), 0, st, p);
  }
  return launch_status();
}

// Scratch of the entry point that allocates nothing: the microbenchmark's workspace for up to kMbScratchMaxM
// rows as a file-scope device array (each GPU the library runs on holds its own copy until the process ends).
// In host code the array's name is only a handle for hipGetSymbolAddress; the device address is looked up once
// per device, with that device current, and kept.
constexpr int kMbScratchMaxM = 32768;
constexpr size_t kMbScratchBytes = 512 + (size_t)kMbScratchMaxM * 4 + ((2 * (size_t)kMbScratchMaxM + 2 * kNumXcd) * 4 + 255) / 256 * 256;
static __device__ __align__(256) __attribute__((used)) unsigned char g_mb_scratch[kMbScratchBytes];

int mb_scratch_ptr(void** out) {
  static std::mutex mu;
  static void* ptr[64] = {nullptr};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MOE_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(g_mb_scratch)) != hipSuccess || !q) return MOE_ERR_LAUNCH;
    ptr[dev] = q;
  }
  *out = ptr[dev];
  return MOE_OK;
}

}  // namespace

extern "C" {

const char* moe_status_string(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument";
    case MOE_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
    case MOE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MOE_ERR_LAUNCH: return "HIP launch failed";
    case MOE_ERR_SCHED_TIMEOUT: return "persistent scheduler wait timed out";
    case MOE_ERR_XCD_PLACEMENT: return "workgroups of one class (id % 8) span several XCDs";
    default: return "unknown status";
  }
}

int moe_ffn_workspace_bytes(const MoeShape* shape, size_t* fwd_bytes, size_t* bwd_bytes) {
  int st = check_shape(shape);
  if (st != MOE_OK) return st;
  Layout L = make_layout(*shape);
  if (fwd_bytes) *fwd_bytes = L.fwd_total;
  if (bwd_bytes) *bwd_bytes = make_bwd_layout(*shape).total;
  return MOE_OK;
}

int moe_route(const MoeShape* shape, const float* d_logits, const MoeSaved* saved, void* d_workspace,
              size_t workspace_bytes, void* stream) {
  Ctx c;
  int st = make_ctx(c, shape, saved, d_workspace, workspace_bytes, stream);
  if (st != MOE_OK || c.s.T == 0) return st;
  if (!d_logits || !saved) return MOE_ERR_INVALID_ARG;
  return run_route(c, d_logits);
}

int moe_permute(const MoeShape* shape, const void* d_x, const MoeSaved* saved, void* d_workspace,
                size_t workspace_bytes, void* stream) {
  Ctx c;
  int st = make_ctx(c, shape, saved, d_workspace, workspace_bytes, stream);
  if (st != MOE_OK || c.s.T == 0) return st;
  if (!d_x || !aligned16(d_x) || !saved) return MOE_ERR_INVALID_ARG;
  return run_permute(c, d_x);
}

int moe_grouped_gemm_swiglu(const MoeShape* shape, const void* d_w_gate_up, const MoeSaved* saved,
                            void* d_workspace, size_t workspace_bytes, void* stream) {
  Ctx c;
  int st = make_ctx(c, shape, saved, d_workspace, workspace_bytes, stream);
  if (st != MOE_OK || c.s.T == 0) return st;
  if (!d_w_gate_up || !aligned16(d_w_gate_up) || !saved) return MOE_ERR_INVALID_ARG;
  return run_gemm1(c, d_w_gate_up);
}

int moe_grouped_gemm(const MoeShape* shape, const void* d_w_down, const MoeSaved* saved, void* d_workspace,
                     size_t workspace_bytes, void* stream) {
  Ctx c;
  int st = make_ctx(c, shape, saved, d_workspace, workspace_bytes, stream);
  if (st != MOE_OK || c.s.T == 0) return st;
  if (!d_w_down || !aligned16(d_w_down) || !saved) return MOE_ERR_INVALID_ARG;
  return run_gemm2(c, d_w_down);
}

int moe_combine(const MoeShape* shape, const MoeSaved* saved, void* d_out, void* d_workspace,
                size_t workspace_bytes, void* stream) {
  Ctx c;
  int st = make_ctx(c, shape, saved, d_workspace, workspace_bytes, stream);
  if (st != MOE_OK || c.s.T == 0) return st;
  if (!d_out || !aligned16(d_out) || !saved) return MOE_ERR_INVALID_ARG;
  return run_combine(c, d_out);
}

int moe_grouped_gemm_scatter(const MoeShape* shape, const void* d_w_down, const MoeSaved* saved, void* d_out,
                             void* d_workspace, size_t workspace_bytes, void* stream) {
  Ctx c;
  int st = make_ctx(c, shape, saved, d_workspace, workspace_bytes, stream);
  if (st != MOE_OK) return st;
  if (c.s.dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
  if (c.s.T == 0) return MOE_OK;
  if (!d_w_down || !aligned16(d_w_down) || !d_out || !aligned16(d_out) || !saved) return MOE_ERR_INVALID_ARG;
  return run_gemm2_scatter(c, d_w_down, d_out);
}

int moe_ffn_forward_scatter(const MoeShape* shape, const void* d_x, const float* d_logits, const void* d_w_gate_up,
                            const void* d_w_down, void* d_out, const MoeSaved* saved, void* d_workspace,
                            size_t workspace_bytes, int mode, void* stream) {
  Ctx c;
  int st = make_ctx(c, shape, saved, d_workspace, workspace_bytes, stream);
  if (st != MOE_OK) return st;
  if (c.s.dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
  if (mode != MOE_MODE_SERIALIZED && mode != MOE_MODE_PERSISTENT) return MOE_ERR_INVALID_ARG;
  if (c.s.T == 0) return MOE_OK;
  const void* ptrs[] = {d_x, d_logits, d_w_gate_up, d_w_down, d_out};
  for (const void* q : ptrs)
    if (!q || !aligned16(q)) return MOE_ERR_INVALID_ARG;
  if (mode == MOE_MODE_PERSISTENT) {
    if (!aligned128(c.ws) || !aligned128(c.sv.Xp) || !aligned128(c.sv.A)) return MOE_ERR_INVALID_ARG;
    if ((st = run_route(c, d_logits, true, d_out)) != MOE_OK) return st;
    return run_persistent_scatter(c, d_x, d_w_gate_up, d_w_down, d_out);
  }
  if ((st = run_route(c, d_logits, false, d_out)) != MOE_OK) return st;   // the output is zeroed beside the rank step
  if (!gathers_x(c) && (st = run_permute(c, d_x)) != MOE_OK) return st;
  if ((st = run_gemm1(c, d_w_gate_up, gathers_x(c) ? d_x : nullptr)) != MOE_OK) return st;
  return run_gemm2_scatter(c, d_w_down, d_out, true);
}

// Dispatch -> GEMM-1 + SwiGLU -> GEMM-2 -> Combine on routing results that are already in `saved` / the workspace.
static int run_dispatch_to_combine(const Ctx& c, const void* d_x, const void* d_w_gate_up, const void* d_w_down,
                                   void* d_out, int mode) {
  if (mode != MOE_MODE_SERIALIZED && mode != MOE_MODE_PERSISTENT) return MOE_ERR_INVALID_ARG;
  const void* ptrs[] = {d_x, d_w_gate_up, d_w_down, d_out};
  for (const void* q : ptrs)
    if (!q || !aligned16(q)) return MOE_ERR_INVALID_ARG;
  if (mode == MOE_MODE_PERSISTENT) {
    // Xp (PERMUTE -> GEMM-1) and A (GEMM-1 -> GEMM-2) change hands inside the launch; the workspace holds
    // their fallback storage at 256-byte offsets
    if (!aligned128(c.ws) || !aligned128(c.sv.Xp) || !aligned128(c.sv.A)) return MOE_ERR_INVALID_ARG;
    return c.s.dtype == MOE_BF16 ? run_persistent<true>(c, d_x, d_w_gate_up, d_w_down, d_out)
                                 : run_persistent<false>(c, d_x, d_w_gate_up, d_w_down, d_out);
  }
  int st;
  if (!gathers_x(c) && (st = run_permute(c, d_x)) != MOE_OK) return st;
  if ((st = run_gemm1(c, d_w_gate_up, gathers_x(c) ? d_x : nullptr)) != MOE_OK) return st;
  if ((st = run_gemm2(c, d_w_down)) != MOE_OK) return st;
  return run_combine(c, d_out);
}

int moe_dispatch_to_combine(const MoeShape* shape, const void* d_x, const void* d_w_gate_up, const void* d_w_down,
                            void* d_out, const MoeSaved* saved, void* d_workspace, size_t workspace_bytes, int mode,
                            void* stream) {
  Ctx c;
  int st = make_ctx(c, shape, saved, d_workspace, workspace_bytes, stream);
  if (st != MOE_OK || c.s.T == 0) return st;
  if (!saved) return MOE_ERR_INVALID_ARG;
  return run_dispatch_to_combine(c, d_x, d_w_gate_up, d_w_down, d_out, mode);
}

int moe_ffn_forward(const MoeShape* shape, const void* d_x, const float* d_logits, const void* d_w_gate_up,
                    const void* d_w_down, void* d_out, const MoeSaved* saved, void* d_workspace,
                    size_t workspace_bytes, int mode, void* stream) {
  Ctx c;
  int st = make_ctx(c, shape, saved, d_workspace, workspace_bytes, stream);
  if (st != MOE_OK) return st;
  if (mode != MOE_MODE_SERIALIZED && mode != MOE_MODE_PERSISTENT) return MOE_ERR_INVALID_ARG;
  if (c.s.T == 0) return MOE_OK;
  const void* ptrs[] = {d_x, d_logits, d_w_gate_up, d_w_down, d_out};
  for (const void* q : ptrs)
    if (!q || !aligned16(q)) return MOE_ERR_INVALID_ARG;
  if (mode == MOE_MODE_PERSISTENT && (!aligned128(c.ws) || !aligned128(c.sv.Xp) || !aligned128(c.sv.A)))
    return MOE_ERR_INVALID_ARG;   // before anything is enqueued
  if ((st = run_route(c, d_logits, mode == MOE_MODE_PERSISTENT)) != MOE_OK) return st;
  return run_dispatch_to_combine(c, d_x, d_w_gate_up, d_w_down, d_out, mode);
}

int moe_ffn_backward(const MoeShape* shape, const void* d_dy, const void* d_x, const void* d_w_gate_up,
                     const void* d_w_down, const MoeSaved* saved, void* d_dx, void* d_dw_gate_up,
                     void* d_dw_down, float* d_dtopk_w, void* d_workspace, size_t workspace_bytes, int mode,
                     void* stream) {
  return moe_ffn_backward_two_streams(shape, d_dy, d_x, d_w_gate_up, d_w_down, saved, d_dx, d_dw_gate_up, d_dw_down,
                                      d_dtopk_w, d_workspace, workspace_bytes, mode, stream, nullptr);
}

int moe_ffn_backward_two_streams(const MoeShape* shape, const void* d_dy, const void* d_x, const void* d_w_gate_up,
                                 const void* d_w_down, const MoeSaved* saved, void* d_dx, void* d_dw_gate_up,
                                 void* d_dw_down, float* d_dtopk_w, void* d_workspace, size_t workspace_bytes,
                                 int mode, void* stream, void* wgrad_stream) {
  int st = check_shape(shape);
  if (st != MOE_OK) return st;
  // MOE_MODE_PERSISTENT (bf16 only): the two data-gradient GEMMs run as one launch under the tile scheduler
  if (mode != MOE_MODE_SERIALIZED && !(mode == MOE_MODE_PERSISTENT && shape->dtype == MOE_BF16)) return MOE_ERR_INVALID_ARG;
  if (shape->T == 0) return MOE_OK;
  // 32-bit byte offsets of segment rows inside the weight-gradient loads
  if ((double)shape->T * (2 * shape->I > shape->H ? 2 * shape->I : shape->H) * elem_bytes(*shape) >= 4.0e9)
    return MOE_ERR_UNSUPPORTED_SHAPE;
  BwdCtx c;
  c.s = *shape;
  c.L = make_bwd_layout(c.s);
  if (!d_workspace || !aligned16(d_workspace) || !saved) return MOE_ERR_INVALID_ARG;
  // dH1 (act_grad -> gate_grad inside the single launch) lives in the workspace at a 256-byte offset
  if (mode == MOE_MODE_PERSISTENT && !aligned128(d_workspace)) return MOE_ERR_INVALID_ARG;
  if (workspace_bytes < c.L.total) return MOE_ERR_WORKSPACE_TOO_SMALL;
  const void* must[] = {d_dy, d_w_gate_up, d_w_down, d_dx, d_dw_gate_up, d_dw_down, d_dtopk_w,
                        saved->topk_w, saved->counts, saved->offsets, saved->row_of,
                        saved->H1, saved->A, saved->Yp};
  for (const void* q : must)
    if (!q || !aligned16(q)) return MOE_ERR_INVALID_ARG;
  // the dispatched copy saved->Xp is used if the forward kept one; otherwise x is read through the permutation
  if (saved->Xp ? !aligned16(saved->Xp) : (!d_x || !aligned16(d_x) || !saved->token_of || !aligned16(saved->token_of)))
    return MOE_ERR_INVALID_ARG;
  c.ws = static_cast<char*>(d_workspace);
  c.sv = *saved;
  c.stream = static_cast<hipStream_t>(stream);
  c.wgrad_stream = static_cast<hipStream_t>(wgrad_stream);
  c.n_cu = device_cus();
  c.mode = mode;
  c.tiles.expert = reinterpret_cast<int32_t*>(c.ws + c.L.tile_expert);
  c.tiles.row0 = reinterpret_cast<int32_t*>(c.ws + c.L.tile_row0);
  c.tiles.rows = reinterpret_cast<int32_t*>(c.ws + c.L.tile_rows);
  c.tiles.meta = reinterpret_cast<int32_t*>(c.ws + c.L.meta);
  return c.s.dtype == MOE_BF16
             ? run_backward<__bf16>(c, d_dy, d_x, d_w_gate_up, d_w_down, d_dx, d_dw_gate_up, d_dw_down, d_dtopk_w)
             : run_backward<float>(c, d_dy, d_x, d_w_gate_up, d_w_down, d_dx, d_dw_gate_up, d_dw_down, d_dtopk_w);
}

// workspace: queue headers and status word | event counters [n_tiles] | rings; sized for one-row tiles
size_t moe_microbench_workspace_bytes(int M) { return mb_workspace_bytes(M); }

int moe_microbench_swiglu_add(int M, int N, const void* d_x, const void* d_y, void* d_s, void* d_out, int mode,
                              int tile_rows, void* d_workspace, size_t workspace_bytes, void* stream) {
  if (M > 0 && d_workspace && workspace_bytes < mb_workspace_bytes(M)) {
    // argument errors take precedence over the size of the workspace
    const int st = mb_check_args(M, N, d_x, d_y, d_s, d_out, mode, tile_rows, d_workspace);
    return st != MOE_OK ? st : MOE_ERR_WORKSPACE_TOO_SMALL;
  }
  return mb_launch(M, N, d_x, d_y, d_s, d_out, mode, tile_rows, d_workspace, nullptr, stream);
}

int moe_microbench_swiglu_add_static_scratch(int M, int N, const void* d_x, const void* d_y, void* d_s, void* d_out,
                                             int mode, int tile_rows, uint32_t* d_status, void* stream) {
  if (M > kMbScratchMaxM) return MOE_ERR_UNSUPPORTED_SHAPE;
  if (d_status && (reinterpret_cast<uintptr_t>(d_status) & 3)) return MOE_ERR_INVALID_ARG;
  void* scratch = nullptr;
  const int st = mb_scratch_ptr(&scratch);
  if (st != MOE_OK) return st;
  return mb_launch(M, N, d_x, d_y, d_s, d_out, mode, tile_rows, scratch, d_status, stream);
}

int moe_probe_mfma_bf16(int n_workgroups, int mfma_per_wave, int random_operands, void* d_sink, void* stream) {
  if (n_workgroups < 1 || n_workgroups > (1 << 20) || mfma_per_wave < 8 || mfma_per_wave % 8 || mfma_per_wave > (1 << 24) ||
      !d_sink || (reinterpret_cast<uintptr_t>(d_sink) & 3))
    return MOE_ERR_INVALID_ARG;
  hipLaunchKernelGGL(probe_mfma_bf16_kernel, dim3(n_workgroups), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                     mfma_per_wave, random_operands ? 1 : 0, static_cast<float*>(d_sink));
  return launch_status();
}

int moe_probe_copy(const void* d_src, void* d_dst, size_t bytes, void* stream) {
  if (!d_src || !d_dst || bytes % 16 || ((reinterpret_cast<uintptr_t>(d_src) | reinterpret_cast<uintptr_t>(d_dst)) & 15))
    return MOE_ERR_INVALID_ARG;
  if (bytes == 0) return MOE_OK;
  const size_t n16 = bytes / 16;
  const size_t want = (n16 + (size_t)kProbeThreads * kProbeCopyUnroll - 1) / ((size_t)kProbeThreads * kProbeCopyUnroll);
  const int grid = (int)(want < (size_t)(device_cus() * 8) ? want : (size_t)(device_cus() * 8));
  hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(d_src), static_cast<u32x4*>(d_dst), n16);
  return launch_status();
}

int moe_probe_read(const void* d_src, size_t bytes, void* d_sink, void* stream) {
  if (!d_src || !d_sink || bytes % 16 || (reinterpret_cast<uintptr_t>(d_src) & 15) || (reinterpret_cast<uintptr_t>(d_sink) & 3))
    return MOE_ERR_INVALID_ARG;
  if (bytes == 0) return MOE_OK;
  const size_t n16 = bytes / 16;
  const size_t want = (n16 + (size_t)kProbeThreads * kProbeCopyUnroll - 1) / ((size_t)kProbeThreads * kProbeCopyUnroll);
  const int grid = (int)(want < (size_t)(device_cus() * 8) ? want : (size_t)(device_cus() * 8));
  hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(d_src), n16, static_cast<uint32_t*>(d_sink));
  return launch_status();
}

int moe_probe_write(void* d_dst, size_t bytes, uint32_t word, void* stream) {
  if (!d_dst || bytes % 16 || (reinterpret_cast<uintptr_t>(d_dst) & 15)) return MOE_ERR_INVALID_ARG;
  if (bytes == 0) return MOE_OK;
  const size_t n16 = bytes / 16;
  const size_t grid = (n16 + kProbeThreads - 1) / kProbeThreads;
  if (grid > 0x7fffffffu) return MOE_ERR_INVALID_ARG;   // 8 TB
  hipLaunchKernelGGL(probe_write_kernel, dim3((unsigned)grid), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<u32x4*>(d_dst), n16, word);
  return launch_status();
}

#if defined(MOE_SCHED_TRACE)
// Tracing variant only: reads (reset == 0, out: 16 words on the host) or clears the cycle counters of the
// register-stationary weight-gradient kernel.
int moe_trace_wgrad_cycles(unsigned long long* out, int reset) {
  if (reset) {
    const unsigned long long z[16] = {0};
    return hipMemcpyToSymbol(HIP_SYMBOL(g_wgrad_cycles), z, sizeof(z)) == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH;
  }
  if (!out) return MOE_ERR_INVALID_ARG;
  return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_wgrad_cycles), 16 * sizeof(unsigned long long)) == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH;
}
#endif

int moe_microbench_last_status(const void* d_workspace) {
  if (!d_workspace) return MOE_ERR_INVALID_ARG;
  uint32_t word = 0;
  if (hipMemcpy(&word, static_cast<const char*>(d_workspace) + 8, 4, hipMemcpyDeviceToHost) != hipSuccess)
    return MOE_ERR_LAUNCH;
  return (word & 2u) ? MOE_ERR_XCD_PLACEMENT : (word ? MOE_ERR_SCHED_TIMEOUT : MOE_OK);
}

int moe_ffn_debug_set_spin_limit(uint32_t polls) {
  g_spin_limit = polls;
  return MOE_OK;
}

int moe_ffn_debug_force_device_scope(int on) {
  g_force_device_scope = on ? 1 : 0;
  return MOE_OK;
}

int moe_ffn_debug_layout(const MoeShape* shape, int backward, int64_t* out, int n_out) {
  int st = check_shape(shape);
  if (st != MOE_OK) return st;
  if (!out || n_out < MOE_LAYOUT_WORDS) return MOE_ERR_INVALID_ARG;
  int64_t v[MOE_LAYOUT_WORDS] = {0};
  if (backward) {
    const BwdLayout L = make_bwd_layout(*shape);
    v[0] = (int64_t)L.meta; v[1] = (int64_t)L.tile_expert; v[2] = (int64_t)L.tile_row0; v[3] = (int64_t)L.tile_rows;
    v[4] = (int64_t)L.events; v[5] = (int64_t)L.qhead; v[6] = (int64_t)L.tasks;
  } else {
    const Layout L = make_layout(*shape);
    v[0] = (int64_t)L.meta; v[1] = (int64_t)L.tile_expert; v[2] = (int64_t)L.tile_row0; v[3] = (int64_t)L.tile_rows;
    v[4] = (int64_t)L.events; v[5] = (int64_t)L.qhead; v[6] = (int64_t)L.tasks;
  }
  v[7] = max_mtiles(*shape); v[8] = max_tasks_per_queue(*shape); v[9] = n_events(*shape);
  v[10] = kEvPerTile; v[11] = kEvGemm2; v[12] = kMetaMTiles; v[13] = kMetaQueueCount0; v[14] = kMetaGemm2Total;
  v[15] = kNumXcd; v[16] = perm_task_rows(*shape); v[17] = gemm1_ntiles(*shape); v[18] = gemm2_ntiles(*shape);
  v[19] = tile_wide_max(*shape); v[20] = tile_tall(*shape); v[21] = kGemm2Lag; v[22] = (int64_t)sizeof(TaskDesc);
  v[23] = backward ? (shape->dtype == MOE_BF16 ? (shape->I + kBN - 1) / kBN : shape->I / kFBN) : 0;   // act_grad N tiles
  v[24] = kMetaFallbackWorkers;
  for (int i = 0; i < MOE_LAYOUT_WORDS; ++i) out[i] = v[i];
  return MOE_OK;
}

int moe_ffn_last_status(const MoeShape* shape, const void* d_workspace) {
  int st = check_shape(shape);
  if (st != MOE_OK) return st;
  if (!d_workspace) return MOE_ERR_INVALID_ARG;
  Layout L = make_layout(*shape);
  int32_t word = 0;
  if (hipMemcpy(&word, static_cast<const char*>(d_workspace) + L.meta + kMetaStatus * 4, 4,
                hipMemcpyDeviceToHost) != hipSuccess)
    return MOE_ERR_LAUNCH;
  return word;
}

}  // extern "C"
