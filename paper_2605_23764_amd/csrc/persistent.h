// Single-launch persistent tile scheduler (paper Sections 4.3-4.4, the unified
// runtime; this is its one-GPU analogue on homogeneous CUs).
//
// Every workgroup is a worker: it takes the next task index of a queue with one
// atomic ticket, loads the task descriptor (TD, the paper's Table 1 in spirit:
// task type, tile coordinates, dependent event + threshold; the trigger event
// follows from type and tile), spins until the dependent event counter has reached
// its threshold, runs the handler, makes its outputs visible device-wide and bumps
// the trigger counter.  Queue order is a topological order of the layer's DAG and
// tickets are consumed in order, so every wait is on work that an earlier ticket
// holder is already running: no cycles, no scheduler state besides the counters
// (Section 4.3's progress argument).  Handlers are the same device functions the
// serialized launches run, so results are bit-identical for any legal order.
//
// The single launch covers the paper's own interval, Dispatch to Combine (Section 5.2 starts the
// clock at Dispatch).  Routing runs ahead of it as two small launches at full occupancy (the
// router, then prefix sums + stable ranks): a worker here is a 4-wave workgroup that owns a whole
// CU for the sake of the GEMM tiles, the wrong shape for the latency-bound routing steps.  The
// second routing launch also zeroes the event counters and queue heads and materialises the task
// descriptors, so nothing but the persistent kernel itself stands between Dispatch and Combine.
//
// Queues
//   X0..X7        one per XCD: PERMUTE parts, GEMM-1 tiles, GEMM-2 tiles of the M-tile
//                 pairs dealt to that XCD (pair % 8), so tiles sharing an activation
//                 or weight panel sit behind one L2.  These TDs depend on the routing result
//                 (Section 5.1: tile offsets are only known once routing is) and are materialised on
//                 the device by the workgroup that finishes the prefix sums.  GEMM-2 tiles of pair j are queued
//                 behind the GEMM-1 tiles of pair j+1: a consumer is issued about
//                 one sweep after its producers, close enough for L2 reuse, far
//                 enough not to stall the queue.
//   C  (global)   COMBINE x token groups, after every GEMM-2 tile
// XCD queues are private to the workers of that XCD (no stealing), so the PERMUTE ->
// GEMM-1 -> GEMM-2 chain of an M tile is produced and consumed behind one L2.  That
// lets those events skip the device-scope cache maintenance: a device-scope release
// (buffer_wbl2) stalls for a write-back of everything dirty in the XCD's L2 (about
// 30 us per task when all CUs do it) and a device-scope acquire (buffer_inv) drops
// the L2 contents the sibling tiles are sharing.  Inside an XCD it is enough that the
// producer's stores have been acknowledged by the L2 before the counter moves; every
// 128-byte line of Xp and A is written by one task, completely, before any task reads it
// within a launch (rows are multiples of 128 bytes and the host requires 128-byte aligned
// buffers in this mode), so no CU can hold a stale copy of a line in its vector L1 and
// there is nothing to invalidate on the consumer side.  The event that crosses XCDs
// (GEMM-2 -> COMBINE) keeps the full device-scope fences; since COMBINE needs every
// GEMM-2 tile, a worker publishes its GEMM-2 completions once, after its queue has drained.
//
// Placement is checked, not assumed: every worker reads the id of the XCD it really runs on
// (hardware register XCC_ID) and reports it when it starts; a queue whose workers do not all
// sit on one XCD (another partition mode, a CU mask) uses device-scope fences for its chain
// events instead.
#pragma once
#include <type_traits>

#include "common.h"
#include "gemm_bf16.h"
#include "gemm_f32.h"
#include "permute_combine.h"
#include "route.h"
#include "wave_sync.h"

namespace moe {

constexpr int kPermRows = 16;            // least rows per PERMUTE task (four per wave): small, so that a queue's PERMUTE tasks
                                         // spread evenly over its workers whatever their number
constexpr int kCombineTokens = 32;       // tokens per COMBINE task (fewer when that would leave CUs without one)
constexpr int kGemm2Lag = 1 << 20;       // GEMM-2 of tile pair j is queued behind GEMM-1 of pair j + lag, clamped to the queue's pairs:
                                         // as it stands, all GEMM-1 tiles of an XCD first (its GEMM-2 tiles fill their last round and
                                         // find their producers long done; a lag of 1..3 pairs measured equal at T = 8192, 2 % slower at T = 4096)

enum TaskType { kTaskPermute = 0, kTaskGemm1 = 1, kTaskGemm2 = 2 };
constexpr int kTaskTypeMask = 0x7F;
constexpr int kTaskNarrow = 0x80;        // flag in the type byte: the index counts 128-column tiles and the tile runs in the tall shape

// Event counters (uint32, zero at kernel start).
enum EventId { kEvArrive = 0, kEvGemm2 = 3, kEvPerTile = 4 };
//   kEvArrive .. +2              placement check: workers that have started, and per queue the XCDs its workers run on
//   kEvGemm2                     finished GEMM-2 tiles, published device-wide
//   kEvPerTile + m               rows of M tile m are in Xp      (PERMUTE parts of m)
//   kEvPerTile + max_mtiles + m  A rows of M tile m are complete (GEMM-1 tiles of m)
constexpr int kNoEvent = -1;             // dep_event of a task that waits for nothing

enum QueueId { kQXcd0 = 0, kQCombine = kNumXcd, kNumQueues = 16 };

enum SchedMetaWord { kMetaQueueCount0 = 4, kMetaGemm2Total = 12, kMetaFallbackWorkers = 13 };   // after MetaWord
//   kMetaFallbackWorkers         workers of the last single launch that used device-wide fences for their chain events

struct TaskDesc {
  int32_t type_n;      // TaskType | (N tile or part index << 8)
  int32_t m;           // M tile
  int32_t dep_event;   // counter that must reach `threshold` before the task may start (kNoEvent: none)
  int32_t threshold;
};

template <bool BF16>
struct SchedParams {
  RouteParams route;
  PermuteParams perm;
  typename std::conditional<BF16, GemmParams, GemmParamsF32>::type g1, g2;
  CombineParams comb;
  uint32_t* events;
  uint32_t* qhead;         // [kNumQueues]
  TaskDesc* tasks;         // [kNumXcd][max_tasks_per_q]
  int32_t* meta;
  int max_mtiles, max_tasks_per_q;
  int n_events;
  int n_comb_tasks;
  int workers_per_q;       // workers per XCD queue (grid of the single launch / 8): decides whether a queue's last round of GEMM-2 tasks is halved
  int comb_tokens;         // tokens per COMBINE task
  int perm_rows;           // rows per PERMUTE task
  int no_permute;          // nobody needs Xp: GEMM-1 gathers its rows from x through token_of
  int force_device_scope;  // test hook: behave as if a worker had reported a foreign XCD
  int skip_tables;         // routing launch: the serialized operators follow, nobody reads counters or task tables
  uint4* zero_dst;         // routing launch, optional: zero_n16 16-byte vectors that further workgroups of the launch
  size_t zero_n16;         // set to zero (the layer output ahead of a GEMM-2 that adds its rows into it)
  uint32_t spin_limit;     // polls before a wait gives up (MOE_ERR_SCHED_TIMEOUT)
  int32_t timeout_status;
};

// Optional per-task time stamps (100 MHz wall clock) for a tile-level timeline;
// compiled in only with -DMOE_SCHED_TRACE, the buffer then sits behind the task tables.
#if defined(MOE_SCHED_TRACE)
struct TraceRec { int32_t wg, kind, a, b; long long t_fetch, t_start, t_end; };
#define MOE_TRACE_DECL TraceRec tr_; tr_.wg = blockIdx.x;
#define MOE_TRACE_FETCH(kind_, a_, b_) { tr_.kind = (kind_); tr_.a = (a_); tr_.b = (b_); tr_.t_fetch = wall_clock64(); }
#define MOE_TRACE_START tr_.t_start = wall_clock64();
#define MOE_TRACE_END(sp_)                                                                                   \
  {                                                                                                          \
    tr_.t_end = wall_clock64();                                                                              \
    if (threadIdx.x == 0) {                                                                                  \
      TraceRec* base_ = reinterpret_cast<TraceRec*>((sp_).tasks + (size_t)kNumXcd * (sp_).max_tasks_per_q);  \
      int slot_ = atomicAdd(reinterpret_cast<int*>(&(sp_).qhead[kNumQueues - 1]), 1);                        \
      if (slot_ < 8192) base_[slot_] = tr_;                                                                  \
    }                                                                                                        \
  }
#else
#define MOE_TRACE_DECL
#define MOE_TRACE_FETCH(kind_, a_, b_)
#define MOE_TRACE_START
#define MOE_TRACE_END(sp_)
#endif

// One ticket of queue `q` for the whole workgroup (wave 0 draws, LDS broadcasts).
__device__ __forceinline__ int sched_fetch(uint32_t* qhead, int q, volatile int* s_box, int wave) {
  if (wave == 0) s_box[0] = (int)wave_atomic_add(&qhead[q], 1u);   // every lane stores the same value
  __syncthreads();
  const int t = __builtin_amdgcn_readfirstlane(s_box[0]);
  __syncthreads();
  return t;
}

enum EventScope { kScopeDevice = 0, kScopeXcd = 1 };

// Start-up report of a worker that serves queue `q`: the XCD it really runs on (wave_sync.h, placement check).
template <bool BF16>
__device__ __forceinline__ void sched_arrive(const SchedParams<BF16>& sp, int q, int wave) {
  if (wave == 0) placement_report(&sp.events[kEvArrive], q, sp.force_device_scope != 0);
}

// Scope of the chain events of this worker's queue: XCD-local if all workers of the queue have reported the same
// XCD, device-wide otherwise (also when the bounded wait for the reports expires, which is recorded in the
// status word).  Every worker of a queue reaches the same verdict, since it is taken after all have reported.
// Called once per worker, ahead of its first wait or trigger.
template <bool BF16>
__device__ __forceinline__ int sched_chain_scope(const SchedParams<BF16>& sp, int q, volatile int* s_box, int wave) {
  if (wave == 0) {
    uint32_t polls = 0;
    int scope = kScopeXcd;
    for (;;) {
      if (ev_load(&sp.events[kEvArrive]) >= gridDim.x) break;
      if (++polls > sp.spin_limit) { scope = kScopeDevice; break; }
      __builtin_amdgcn_s_sleep(1);
    }
    if (scope == kScopeDevice) __hip_atomic_store(&sp.meta[kMetaStatus], sp.timeout_status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else if (!placement_class_ok(&sp.events[kEvArrive], q)) scope = kScopeDevice;
    if (scope == kScopeDevice) wave_atomic_add(reinterpret_cast<uint32_t*>(&sp.meta[kMetaFallbackWorkers]), 1u);
    s_box[1] = scope;
  }
  __syncthreads();
  const int scope = __builtin_amdgcn_readfirstlane(s_box[1]);
  __syncthreads();
  return scope;
}

// Wait until events[ev] >= threshold (bounded).  Returns false on timeout after
// recording the status word; the caller then skips the task without triggering.
template <bool BF16>
__device__ __forceinline__ bool sched_wait(const SchedParams<BF16>& sp, int ev, uint32_t threshold, volatile int* s_box,
                                           int wave, int scope = kScopeDevice) {
  if (wave == 0) {
    uint32_t polls = 0;
    int ok = 1;
    for (;;) {
      if (ev_load(&sp.events[ev]) >= threshold) break;
      if (++polls > sp.spin_limit) { ok = 0; break; }
      __builtin_amdgcn_s_sleep(1);
    }
    if (!ok) __hip_atomic_store(&sp.meta[kMetaStatus], sp.timeout_status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_box[1] = ok;
  }
  __syncthreads();
  const int ok = __builtin_amdgcn_readfirstlane(s_box[1]);
  if (scope == kScopeDevice) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // producers' data, not only the counter
  else __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  __syncthreads();
  return ok != 0;
}

// Outputs of this workgroup become visible (device-wide, or to the workgroups behind the same L2), then
// the counter moves.
template <bool BF16>
__device__ __forceinline__ void sched_trigger(const SchedParams<BF16>& sp, int ev, int wave, int scope = kScopeDevice,
                                              uint32_t inc = 1u) {
  if (scope == kScopeDevice) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  } else {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    wait_own_stores();                                          // ... acknowledged by the XCD's L2
  }
  __syncthreads();
  if (wave == 0) wave_atomic_add(&sp.events[ev], inc);
}

// Zero the counters and queue heads, then materialise the per-XCD task tables from the fresh tile map.
// Whole workgroup, after the tile map is complete: a wave per queue, the lanes of the wave fill a block
// of descriptors in parallel (block offsets are wave-uniform running sums).
// BWD: the chain is act_grad (as "GEMM-1": no PERMUTE ahead of it, nothing to wait for; its narrow tall
// tiles are 128 columns wide) followed by gate_grad (as "GEMM-2").
template <bool BF16, bool BWD = false>
__device__ __forceinline__ void build_task_tables(const SchedParams<BF16>& sp) {
  __shared__ int s_extra[kNumXcd];   // per queue: GEMM-2 tasks added by halving its last round
  for (int i = threadIdx.x; i < sp.n_events; i += blockDim.x) sp.events[i] = 0;
  if (threadIdx.x < kNumQueues) sp.qhead[threadIdx.x] = 0;
  if (threadIdx.x == 0) sp.meta[kMetaFallbackWorkers] = 0;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), n_waves = blockDim.x / kWave;
  const int n_mtiles = sp.meta[kMetaMTiles];
  const int nN1 = sp.g1.n_ntiles, nN2 = sp.g2.n_ntiles;
  // the tile map lists M tiles in pairs (siblings of one expert where possible); queue q owns pairs q, q+8, ...
  const int n_pairs = (n_mtiles + 1) >> 1;
  auto parts_of = [&](int m) { return (sp.route.tiles.rows[m] + sp.perm_rows - 1) / sp.perm_rows; };
  constexpr int kTallAbove = BF16 ? kWideRows : (1 << 30);   // a bf16 tile with more rows runs in the tall shape
  const bool permute = !(sp.no_permute || BWD);
  for (int q = wave; q < kNumXcd; q += n_waves) {
    const int Pq = n_pairs > q ? (n_pairs - q + kNumXcd - 1) / kNumXcd : 0;
    TaskDesc* tq = sp.tasks + (size_t)q * sp.max_tasks_per_q;
    int n = 0, n_g2 = 0;
    constexpr int kTallCols1 = BWD ? 128 : 64;   // output columns of a narrow GEMM-1 tile of a tall M tile
    for (int j = 0; j < (permute ? Pq : 0); ++j)
      for (int s = 0; s < 2; ++s) {
        const int m = 2 * (q + kNumXcd * j) + s;
        if (m >= n_mtiles) continue;
        const int parts = parts_of(m);   // 0 for the unused half of a tall tile's slot
        for (int part = lane; part < parts; part += kWave)
          tq[n + part] = TaskDesc{kTaskPermute | (part << 8), m, kNoEvent, 0};
        n += parts;
      }
    // GEMM tiles of a slot N-tile-major with the two siblings adjacent (they stream the same weight panel
    // at the same time); a tall tile fills its slot with twice as many half-width N tiles
    const int lag = min(kGemm2Lag, max(Pq, 1));
    for (int j = 0; j < Pq + lag; ++j) {
      if (j < Pq) {
        const int m0 = 2 * (q + kNumXcd * j);
        const int rows0 = sp.route.tiles.rows[m0];
        const bool tall = rows0 > kTallAbove;
        const int n_sib = rows0 <= 0 ? 0 : tall ? 1 : ((m0 + 1 < n_mtiles && sp.route.tiles.rows[m0 + 1] > 0) ? 2 : 1);   // 0: empty slot
        const int n_nt = tall ? (sp.g1.N + kTallCols1 - 1) / kTallCols1 : nN1;
        const int parts0 = parts_of(m0), parts1 = n_sib > 1 ? parts_of(m0 + 1) : 0;
        for (int i = lane; i < n_nt * n_sib; i += kWave) {
          const int nt = i / n_sib, sib = i - nt * n_sib;
          tq[n + i] = permute ? TaskDesc{kTaskGemm1 | (nt << 8), m0 + sib, kEvPerTile + m0 + sib, sib ? parts1 : parts0}
                              : TaskDesc{kTaskGemm1 | (nt << 8), m0 + sib, kNoEvent, 0};
        }
        n += n_nt * n_sib;
      }
      if (j >= lag) {
        const int m0 = 2 * (q + kNumXcd * (j - lag));
        const bool tall = sp.route.tiles.rows[m0] > kTallAbove;
        const int n_sib = sp.route.tiles.rows[m0] <= 0 ? 0 : tall ? 1 : ((m0 + 1 < n_mtiles && sp.route.tiles.rows[m0 + 1] > 0) ? 2 : 1);
        const int n_nt = tall ? (sp.g2.N + 127) / 128 : nN2;
        const int g1_tiles = tall ? (sp.g1.N + kTallCols1 - 1) / kTallCols1 : nN1;   // GEMM-1 tiles that complete a row block of A
        for (int i = lane; i < n_nt * n_sib; i += kWave) {
          const int nt = i / n_sib, sib = i - nt * n_sib;
          tq[n + i] = TaskDesc{kTaskGemm2 | (nt << 8), m0 + sib, kEvPerTile + sp.max_mtiles + m0 + sib, g1_tiles};
        }
        n += n_nt * n_sib;
        n_g2 += n_nt * n_sib;
      }
    }
    // The queue's GEMM-2 tasks are its last n_g2 entries (they follow all of its GEMM-1 tasks) and are drawn by
    // workers_per_q workers in what amounts to rounds.  A last round that would leave at least half of them without
    // a task is halved, as in the serialized kernels: each of its wide tasks becomes two 128-column tasks in the
    // tall shape (one, if the second half lies past the last column).
    int extra = 0;
    if (BF16 && lag >= Pq && sp.workers_per_q > 0) {
      const int tail = n_g2 % sp.workers_per_q;
      if (tail > 0 && 2 * tail <= sp.workers_per_q && tail <= kWave / 2) {
        const int n_half = (sp.g2.N + 127) / 128;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // this wave's own descriptors, written by other lanes
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        TaskDesc td = TaskDesc{0, 0, kNoEvent, 0};
        int cnt = 0;
        if (lane < tail) {
          td = tq[n - tail + lane];
          const bool wide = sp.route.tiles.rows[td.m] <= kTallAbove;
          cnt = wide && 2 * (td.type_n >> 8) + 1 < n_half ? 2 : 1;
          if (wide) td.type_n = kTaskGemm2 | kTaskNarrow | ((2 * (td.type_n >> 8)) << 8);
        }
        const int incl = wave_incl_scan(cnt, lane);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // all reads of the old entries ahead of the writes below
        __builtin_amdgcn_wave_barrier();
        if (lane < tail) {
          const int at = n - tail + incl - cnt;
          tq[at] = td;
          if (cnt == 2) tq[at + 1] = TaskDesc{td.type_n + (1 << 8), td.m, td.dep_event, td.threshold};
        }
        extra = __shfl(incl, kWave - 1, kWave) - tail;
        n += extra;
      }
    }
    if (lane == 0) {
      sp.meta[kMetaQueueCount0 + q] = n;
      s_extra[q] = extra;
    }
  }
  __syncthreads();
  // COMBINE waits for every GEMM-2 tile: count them
  if (wave == 0) {
    int total = 0;
    for (int m = lane; m < n_mtiles; m += kWave) {
      const int rows = sp.route.tiles.rows[m];
      total += rows > kTallAbove ? (sp.g2.N + 127) / 128 : (rows > 0 ? nN2 : 0);
    }
    if (lane < kNumXcd) total += s_extra[lane];
    total = wave_incl_scan(total, lane);
    if (lane == kWave - 1) sp.meta[kMetaGemm2Total] = total;
  }
}

// Second routing launch (both launch modes): prefix sums and M-tile map by workgroup 0, stable ranks by the
// others, plus, in workgroup 0, the tile scheduler's counters and task tables.
template <bool BF16>
__global__ __launch_bounds__(kScanRankWaves * kWave) void sched_prepare_kernel(SchedParams<BF16> sp) {
  __shared__ int32_t s_lds[kScanRankWaves * kRankLdsWords];   // rank: 4 * kMaxE words per wave; scan: (5 * kMaxE + 66) words
  if (blockIdx.x == 0) {
    scan_all(sp.route, s_lds, s_lds + kMaxE + 64);
    __threadfence_block();
    __syncthreads();   // tile map (written by wave 0) complete before every wave reads it
    if (!sp.skip_tables) build_task_tables<BF16>(sp);
    return;
  }
  const int rank_wgs = (sp.route.n_groups + kScanRankWaves - 1) / kScanRankWaves;
  if ((int)blockIdx.x > rank_wgs) {       // fill workgroups: the launch lasts as long as workgroup 0's chain anyway
    const size_t stride = (size_t)(gridDim.x - 1 - rank_wgs) * blockDim.x;
    for (size_t i = (size_t)(blockIdx.x - 1 - rank_wgs) * blockDim.x + threadIdx.x; i < sp.zero_n16; i += stride)
      sp.zero_dst[i] = make_uint4(0, 0, 0, 0);
    return;
  }
  const int wave = threadIdx.x / kWave;
  const int group = (blockIdx.x - 1) * kScanRankWaves + wave;
  if (group < sp.route.n_groups) rank_chunk(sp.route, group, s_lds + wave * kRankLdsWords);
}

// Vector tasks of a 4-wave worker: 16-byte vectors per lane and pass matched to the row length (a row of H = 7168
// bf16 is 14 per lane, of H = 2048 four): a pass wider than the row spends its instructions on vectors that do not
// exist (COMBINE) or falls through to a one-vector-at-a-time tail (PERMUTE).
template <typename F>
__device__ __forceinline__ void with_row_vectors(int vec_per_row, F&& f) {
  if (vec_per_row >= 14 * kWave) f(std::integral_constant<int, 14>{});
  else if (vec_per_row >= 7 * kWave) f(std::integral_constant<int, 7>{});
  else f(std::integral_constant<int, 4>{});
}

// SCATTER (bf16): GEMM-2 tiles add their weighted rows into the zeroed layer output from their epilogue
// (kEpiScatter), and the launch has no COMBINE tasks: nothing waits for the whole chip's GEMM-2 tiles.
template <bool BF16, bool SCATTER = false>
__device__ __forceinline__ void run_tile_task(const SchedParams<BF16>& sp, const TaskDesc& td, char* smem, volatile int* s_box,
                                              int wave, int q, long long& t_start, uint32_t& gemm2_done, int& scope) {
  const int type_n = __builtin_amdgcn_readfirstlane(td.type_n);
  const int type = type_n & kTaskTypeMask, idx = type_n >> 8, m = __builtin_amdgcn_readfirstlane(td.m);
  const bool narrow = (type_n & kTaskNarrow) != 0;
  const int dep = __builtin_amdgcn_readfirstlane(td.dep_event);
  if (scope < 0) scope = sched_chain_scope(sp, q, s_box, wave);
  // the chain waits on tasks of its own XCD queue
  if (dep != kNoEvent && !sched_wait(sp, dep, (uint32_t)__builtin_amdgcn_readfirstlane(td.threshold), s_box, wave, scope)) return;
#if defined(MOE_SCHED_TRACE)
  t_start = wall_clock64();
#else
  (void)t_start;
#endif
  if (type == kTaskPermute) {
    const int row0 = sp.route.tiles.row0[m], rows = sp.route.tiles.rows[m];
    const int r0 = row0 + idx * sp.perm_rows;
    with_row_vectors(sp.perm.H * sp.perm.elem_bytes / 16, [&](auto uv) {
      permute_rows<decltype(uv)::value>(sp.perm, r0, min(r0 + sp.perm_rows, row0 + rows), wave, blockDim.x / kWave);
    });
    sched_trigger(sp, kEvPerTile + m, wave, scope);
  } else if (type == kTaskGemm1) {
    if constexpr (BF16) gemm_map_tile_bf16<kLayNN, kEpiSwiglu>(sp.g1, m, idx, tile_is_tall(__builtin_amdgcn_readfirstlane(sp.route.tiles.rows[m])), smem);
    else gemm_tile_f32<kEpiSwiglu>(sp.g1, m, idx, reinterpret_cast<float*>(smem));
    sched_trigger(sp, kEvPerTile + sp.max_mtiles + m, wave, scope);
  } else {
    if constexpr (BF16) gemm_map_tile_bf16<kLayNN, SCATTER ? kEpiScatter : kEpiStore>(sp.g2, m, idx, narrow || tile_is_tall(__builtin_amdgcn_readfirstlane(sp.route.tiles.rows[m])), smem);
    else gemm_tile_f32<kEpiStore>(sp.g2, m, idx, reinterpret_cast<float*>(smem));
    // COMBINE waits for every GEMM-2 tile, so completions are counted here and published once per
    // worker after its queue has drained: a device-scope release per tile would write back the
    // XCD's whole L2 each time (about 30 us per tile in a trace)
    ++gemm2_done;
  }
}

template <bool BF16, bool SCATTER = false>
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void persistent_forward_kernel(SchedParams<BF16> sp) {
  static_assert(BF16 || !SCATTER, "the scatter epilogue exists for bf16 only");
  __shared__ __attribute__((aligned(1024))) char smem[kGemmLdsBytes];
  // between tasks the staging area is idle: its first words carry the ticket and the wait result
  volatile int* s_box = reinterpret_cast<volatile int*>(smem);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  MOE_TRACE_DECL

  // ---- queue X of this workgroup's XCD: dispatch + grouped GEMMs ----
  const int q = blockIdx.x % kNumXcd;   // workgroups are dealt to XCDs round-robin: one XCD per class (checked: sched_arrive)
  sched_arrive(sp, q, wave);
  {
    const int count = __builtin_amdgcn_readfirstlane(sp.meta[kMetaQueueCount0 + q]);
    uint32_t gemm2_done = 0;
    int scope = -1;
    for (;;) {
      const int t = sched_fetch(sp.qhead, kQXcd0 + q, s_box, wave);
      if (t >= count) break;
      const TaskDesc td = sp.tasks[(size_t)q * sp.max_tasks_per_q + t];
      MOE_TRACE_FETCH(td.type_n & kTaskTypeMask, td.m, td.type_n >> 8)
      long long t_start = 0;
      run_tile_task<BF16, SCATTER>(sp, td, smem, s_box, wave, q, t_start, gemm2_done, scope);
#if defined(MOE_SCHED_TRACE)
      tr_.t_start = t_start;
#endif
      MOE_TRACE_END(sp)
    }
    if (SCATTER) return;   // no COMBINE tasks; the adds are complete when the launch is
    if (gemm2_done) sched_trigger(sp, kEvGemm2, wave, kScopeDevice, gemm2_done);
  }

  // ---- queue C: combine ----
  const uint32_t g2_total = (uint32_t)__builtin_amdgcn_readfirstlane(sp.meta[kMetaGemm2Total]);
  bool yp_ready = false;   // every GEMM-2 tile seen and acquired: once per worker (Yp never changes afterwards)
  for (;;) {
    const int t = sched_fetch(sp.qhead, kQCombine, s_box, wave);
    if (t >= sp.n_comb_tasks) break;
    MOE_TRACE_FETCH(3, t, 0)
    if (!yp_ready && !sched_wait(sp, kEvGemm2, g2_total, s_box, wave)) continue;
    yp_ready = true;
    MOE_TRACE_START
    // Four waves per CU have to hide the latency the combine kernel hides with thirty-two: a token's slots are
    // fetched while the token before it is reduced, and up to four of its rows are in flight at once.
    const int t0 = t * sp.comb_tokens, t1 = min(t0 + sp.comb_tokens, sp.comb.T), nw = blockDim.x / kWave;
    with_row_vectors(sp.comb.H / (BF16 ? 8 : 4), [&](auto uv) {
      int rowv, rowv_n = -1;
      float wv, wv_n = 0.f;
      if (t0 + wave < t1) combine_load_slots(sp.comb, t0 + wave, rowv, wv);
      for (int tok = t0 + wave; tok < t1; tok += nw) {
        if (tok + nw < t1) combine_load_slots(sp.comb, tok + nw, rowv_n, wv_n);
        combine_token_rows<BF16, decltype(uv)::value, 4>(sp.comb, tok, rowv, wv);
        rowv = rowv_n;
        wv = wv_n;
      }
    });
    MOE_TRACE_END(sp)
  }
}

// ---- backward: the two data-gradient GEMMs as one launch --------------------------------------
// act_grad (+ SwiGLU_grad) and gate_grad form the same kind of chain as GEMM-1 -> GEMM-2: a gate_grad
// tile of M tile m needs every act_grad tile of m (all columns of dH1 for those rows), and both run in
// the same workgroup shape.  One launch, per-XCD ticket queues, XCD-local events: gate_grad tiles fill
// the CUs that act_grad's last, partly empty round leaves idle (its N extent is small: 368 tiles on
// 256 CUs at H = 7168, I = 2048, 32 experts of ~254 rows).  sp.g1 = act_grad, sp.g2 = gate_grad,
// sp.route.tiles = the backward's M-tile map; the other members of sp are unused.

// One workgroup: zero the counters, then build the per-XCD task tables from the finished tile map.
__global__ __launch_bounds__(kGemmThreads) void dgrad_prepare_kernel(SchedParams<true> sp) {
  build_task_tables<true, true>(sp);
}

__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void persistent_dgrad_kernel(SchedParams<true> sp) {
  __shared__ __attribute__((aligned(1024))) char smem[kGemmLdsBytes];
  volatile int* s_box = reinterpret_cast<volatile int*>(smem);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int q = blockIdx.x % kNumXcd;   // workgroups are dealt to XCDs round-robin by id (checked: sched_arrive)
  sched_arrive(sp, q, wave);
  const int count = __builtin_amdgcn_readfirstlane(sp.meta[kMetaQueueCount0 + q]);
  int scope = -1;
  for (;;) {
    const int t = sched_fetch(sp.qhead, kQXcd0 + q, s_box, wave);
    if (t >= count) break;
    const TaskDesc td = sp.tasks[(size_t)q * sp.max_tasks_per_q + t];
    const int type_n = __builtin_amdgcn_readfirstlane(td.type_n);
    const int type = type_n & kTaskTypeMask, idx = type_n >> 8, m = __builtin_amdgcn_readfirstlane(td.m);
    const bool tall = (type_n & kTaskNarrow) != 0 || tile_is_tall(__builtin_amdgcn_readfirstlane(sp.route.tiles.rows[m]));
    if (type == kTaskGemm1) {
      gemm_map_tile_bf16<kLayNT, kEpiSwigluGrad>(sp.g1, m, idx, tall, smem);
      if (scope < 0) scope = sched_chain_scope(sp, q, s_box, wave);
      sched_trigger(sp, kEvPerTile + sp.max_mtiles + m, wave, scope);
    } else {
      if (scope < 0) scope = sched_chain_scope(sp, q, s_box, wave);
      if (!sched_wait(sp, __builtin_amdgcn_readfirstlane(td.dep_event), (uint32_t)__builtin_amdgcn_readfirstlane(td.threshold),
                      s_box, wave, scope))
        continue;   // bounded wait expired: status word set, the task is skipped, the queue still drains
      gemm_map_tile_bf16<kLayNT, kEpiStore>(sp.g2, m, idx, tall, smem);
    }
  }
}

}  // namespace moe
