// SwiGLU + Add microbenchmark (paper Section 6): a producer-consumer pair of
// elementwise operators, S = silu(X[:, :N]) * X[:, N:] followed by Out = S + Y, run
//   serial        two launches, each operator sweeps all rows before the next starts;
//   interleaved   one launch, row tiles, a STATIC order in which the Add tile of a row
//                 block follows its SwiGLU tile closely (Section 6.1), dependencies
//                 through per-tile event counters, every worker walks its own
//                 precomputed share of the order (no scheduling decision at run time);
//   dynamic       one launch, the same tiles and dependencies, but workers pop tasks
//                 from a shared ready queue and a finished SwiGLU tile pushes its Add
//                 tile (Section 6.2: dispatch decided on the device path).  With one queue for
//                 the device the consumer of a tile may sit on any XCD, so every hand-off
//                 pays a device-wide release; with one queue per XCD (mode 3) placement is
//                 still decided at run time but stays inside the producer's XCD, which
//                 isolates the cost of the queue itself.
// The modes run the same per-tile device functions, so their results are
// bit-identical.
#pragma once
#include "common.h"
#include "wave_sync.h"

namespace moe {

constexpr int kMbMaxTileRows = 64;  // rows per tile task: 1 .. 64, chosen per call
constexpr int kMbRingBase = 16 * kNumXcd;

// Queue x of n_q (1: one device queue; 8: one per XCD, tile t belongs to queue t % 8).
struct MbQueue { int n_local, ring; };   // tiles owned, first ring word
__device__ __forceinline__ MbQueue mb_queue(int ring_base, int n_tiles, int n_q, int x) {
  MbQueue q;
  q.n_local = n_tiles > x ? (n_tiles - x + n_q - 1) / n_q : 0;
  q.ring = ring_base + x * 2 * ((n_tiles + n_q - 1) / n_q);
  return q;
}

struct MicrobenchParams {
  const __bf16* X;     // [M, 2N]
  const __bf16* Y;     // [M, N]
  __bf16* S;           // [M, N] intermediate
  __bf16* Out;         // [M, N]
  int M, N;            // N multiple of 8
  uint32_t* events;    // [n_tiles] static mode: SwiGLU tile done
  uint32_t* queue;     // [16x] head and [16x + 1] tail of queue x (8 headers); [4..6] placement check (wave_sync.h);
                       // rings from word ring_base: entries are local task id + 1, 0 = not yet published
  uint32_t* status;    // one word, zeroed per call: bit 0 = a bounded wait expired, bit 1 = in a mode that relies on
                       // XCD-local hand-offs the workgroups of one class (id % 8) do not all run on one XCD
  int n_tiles, tile_rows;
  int ring_base;       // first ring word, relative to queue
  uint32_t spin_limit;
};

// rows [r0, r1): S = silu(gate) * up, by the whole workgroup
__device__ __forceinline__ void mb_swiglu_rows(const MicrobenchParams& p, int r0, int r1) {
  const int vec = p.N / 8;
  for (int i = threadIdx.x; i < (r1 - r0) * vec; i += blockDim.x) {
    const int r = r0 + i / vec, v = i % vec;
    const uint4 g = reinterpret_cast<const uint4*>(p.X + (size_t)r * 2 * p.N)[v];
    const uint4 u = reinterpret_cast<const uint4*>(p.X + (size_t)r * 2 * p.N + p.N)[v];
    const uint32_t gw[4] = {g.x, g.y, g.z, g.w}, uw[4] = {u.x, u.y, u.z, u.w};
    uint32_t o[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const float g0 = bf16_lo(gw[x]), g1 = bf16_hi(gw[x]);
      o[x] = pack_bf16(g0 * sigmoidf_(g0) * bf16_lo(uw[x]), g1 * sigmoidf_(g1) * bf16_hi(uw[x]));
    }
    reinterpret_cast<uint4*>(p.S + (size_t)r * p.N)[v] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// rows [r0, r1): Out = S + Y
__device__ __forceinline__ void mb_add_rows(const MicrobenchParams& p, int r0, int r1) {
  const int vec = p.N / 8;
  for (int i = threadIdx.x; i < (r1 - r0) * vec; i += blockDim.x) {
    const int r = r0 + i / vec, v = i % vec;
    const uint4 a = reinterpret_cast<const uint4*>(p.S + (size_t)r * p.N)[v];
    const uint4 b = reinterpret_cast<const uint4*>(p.Y + (size_t)r * p.N)[v];
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
    uint32_t o[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) o[x] = pack_bf16(bf16_lo(aw[x]) + bf16_lo(bw[x]), bf16_hi(aw[x]) + bf16_hi(bw[x]));
    reinterpret_cast<uint4*>(p.Out + (size_t)r * p.N)[v] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

__global__ __launch_bounds__(256) void mb_swiglu_kernel(MicrobenchParams p) {
  for (int t = blockIdx.x; t < p.n_tiles; t += gridDim.x)
    mb_swiglu_rows(p, t * p.tile_rows, min(p.M, (t + 1) * p.tile_rows));
}
__global__ __launch_bounds__(256) void mb_add_kernel(MicrobenchParams p) {
  for (int t = blockIdx.x; t < p.n_tiles; t += gridDim.x)
    mb_add_rows(p, t * p.tile_rows, min(p.M, (t + 1) * p.tile_rows));
}

__global__ void mb_clear_kernel(MicrobenchParams p, int n_q) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < p.n_tiles; i += gridDim.x * blockDim.x) {
    p.events[i] = 0;
    const int x = i % n_q, j = i / n_q;
    const MbQueue q = mb_queue(p.ring_base, p.n_tiles, n_q, x);
    p.queue[q.ring + j] = (uint32_t)j + 1;          // every SwiGLU task is ready from the start
    p.queue[q.ring + q.n_local + j] = 0;            // Add tasks arrive later
  }
  if (blockIdx.x == 0 && threadIdx.x < kNumXcd) {
    const int x = threadIdx.x;
    p.queue[16 * x] = 0;
    p.queue[16 * x + 1] = x < n_q ? (uint32_t)mb_queue(p.ring_base, p.n_tiles, n_q, x).n_local : 0u;
    if (x == 0) *p.status = 0;
    if (x < 3) p.queue[4 + x] = 0;
  }
}

// Status bits (wave-uniform: called by the whole of wave 0).
__device__ __forceinline__ void mb_flag(const MicrobenchParams& p, uint32_t bit) {
  wave_atomic_or(p.status, bit);
}
// Modes 1 and 3 hand tiles over between the workgroups of one class (id % 8) through the L2 they are taken to
// share.  Every worker reports the XCD it runs on; the one that reports last sees all reports and flags the launch
// if some class is spread over several XCDs.  No worker waits for this.
__device__ __forceinline__ void mb_check_placement(const MicrobenchParams& p, int wave) {
  if (wave == 0 && placement_report(&p.queue[4], (int)(blockIdx.x % kNumXcd)) == gridDim.x - 1 && !placement_all_ok(&p.queue[4]))
    mb_flag(p, 2u);
}

// Both single-launch kernels keep their control flow wave-uniform: wave 0 draws tickets, polls
// and publishes as a whole (scalar branches, single-lane atomics from wave_sync.h), LDS carries
// the result to the other waves between two barriers.

// Static schedule: worker w (of W, a multiple of 8 so that w % 8 is its XCD) runs round r = 0, 1, ...:
// SwiGLU tile r*W + w, then the Add tile of its XCD neighbour (worker (w + 8) % W of the same
// round), which it waits for through that tile's event counter.  The order is a pure function of
// (w, r): nothing is decided, fetched or updated at run time except the counters.
// Because producer and consumer are known to share an XCD, the hand-off needs no device-wide
// release (which writes back that XCD's whole L2): every producing wave waits until its stores have
// reached the L2 (wait_own_stores), the consumer reads lines its CU has never touched in this launch
// through that same L2 (the host requires tiles of whole 128-byte lines in this mode, so no line of S is
// shared by two tiles and no CU's vector L1 can hold a stale one).  Workers w and w + 8 share an XCD when
// workgroups are dealt round-robin; every worker reports the XCD it really runs on and the status word
// tells if a class (w % 8) was spread over several.
__global__ __launch_bounds__(256) void mb_static_kernel(MicrobenchParams p) {
  __shared__ int s_box[2];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int W = gridDim.x, w = blockIdx.x;
  mb_check_placement(p, wave);
  for (int base = 0; base < p.n_tiles; base += W) {
    const int ts = base + w;
    if (ts < p.n_tiles) {
      mb_swiglu_rows(p, ts * p.tile_rows, min(p.M, (ts + 1) * p.tile_rows));
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      wait_own_stores();
      __syncthreads();
      if (wave == 0) wave_atomic_add(&p.events[ts], 1u);
    }
    const int ta = base + (w + 8) % W;
    if (ta < p.n_tiles) {
      if (wave == 0) {
        uint32_t polls = 0;
        int ok = 1;
        for (;;) {
          if (ev_load(&p.events[ta]) >= 1u) break;
          if (++polls > p.spin_limit) { ok = 0; break; }
          __builtin_amdgcn_s_sleep(1);
        }
        if (!ok) mb_flag(p, 1u);
        s_box[0] = ok;          // every lane stores the same value
      }
      __syncthreads();
      const int ok = __builtin_amdgcn_readfirstlane(s_box[0]);
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      __syncthreads();
      if (ok) mb_add_rows(p, ta * p.tile_rows, min(p.M, (ta + 1) * p.tile_rows));
    }
  }
}

// Dynamic schedule: ready queues.  A worker draws a ticket (atomic on the head of its queue),
// waits until that entry of the ring has been published, runs the task; a SwiGLU task then
// publishes its Add task (atomic on the tail, entry write after a release).  Queue x holds
// 2 * n_local tickets.  PER_XCD = false: one queue, device-wide release and acquire;
// PER_XCD = true: workgroup b serves queue b % 8 (its XCD), hand-off through that XCD's L2.
template <bool PER_XCD>
__global__ __launch_bounds__(256) void mb_dynamic_kernel(MicrobenchParams p) {
  __shared__ int s_box[2];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n_q = PER_XCD ? kNumXcd : 1, x = PER_XCD ? (int)(blockIdx.x % kNumXcd) : 0;
  const MbQueue q = mb_queue(p.ring_base, p.n_tiles, n_q, x);
  const uint32_t total = 2u * (uint32_t)q.n_local;
  uint32_t* head = &p.queue[16 * x];
  if (PER_XCD) mb_check_placement(p, wave);
  for (;;) {
    if (wave == 0) {
      int task = -1;                                     // no tickets left
      const uint32_t ticket = wave_atomic_add(head, 1u);
      if (ticket < total) {
        task = -2;                                       // entry never published within the limit
        for (uint32_t polls = 0; polls <= p.spin_limit; ++polls) {
          const uint32_t e = ev_load(&p.queue[q.ring + ticket]);
          if (e != 0) { task = (int)e - 1; break; }
          __builtin_amdgcn_s_sleep(1);
        }
        if (task == -2) mb_flag(p, 1u);
      }
      s_box[0] = task;          // every lane stores the same value
    }
    __syncthreads();
    const int task = __builtin_amdgcn_readfirstlane(s_box[0]);
    __syncthreads();
    if (task == -1) break;
    if (task >= 0) {
      if (PER_XCD) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      else __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      if (task < q.n_local) {
        const int t = task * n_q + x;
        mb_swiglu_rows(p, t * p.tile_rows, min(p.M, (t + 1) * p.tile_rows));
        if (PER_XCD) {
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
          wait_own_stores();
        } else {
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        }
        __syncthreads();
        if (wave == 0) {
          const uint32_t slot = wave_atomic_add(head + 1, 1u);
          // the release fence above ordered this workgroup's rows; every lane stores the same word
          __hip_atomic_store(&p.queue[q.ring + slot], (uint32_t)(q.n_local + task) + 1u, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        }
      } else {
        const int t = (task - q.n_local) * n_q + x;
        mb_add_rows(p, t * p.tile_rows, min(p.M, (t + 1) * p.tile_rows));
      }
    }
  }
}

}  // namespace moe
