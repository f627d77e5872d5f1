// Wave-uniform synchronisation primitives shared by the single-launch schedulers.
#pragma once
#include "common.h"

namespace moe {

constexpr int kNumXcd = 8;   // accelerator dies; workgroups of a launch are dealt to them round-robin by id

// Id of the accelerator die (XCD) this wave runs on: bits 3:0 of the hardware register XCC_ID (number 20).
__device__ __forceinline__ int hw_xcc_id() { return (int)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)); }

// The scheduler's control flow is kept wave-uniform on purpose.  A lane-divergent
// `if (threadIdx.x == 0) { atomic }` at the head of a loop that also contains
// barriers was restructured by the compiler into nested loops in which lanes 1..63
// never left the inner (barrier + ticket read) loop, so no new ticket was ever drawn
// and the kernel spun forever.  Here wave 0 acts as a whole: single-lane atomics are
// issued with the execution mask narrowed inside one assembly statement (the compiler
// does not know that the statement rewrites exec: it must only be reached with all 64
// lanes active, which wave-uniform control flow guarantees), polls are uniform loads,
// and every branch below is scalar.

// This wave's earlier global stores have been acknowledged by the L2 (s_waitcnt vmcnt(0); stores are
// write-through in the L1).  A release between workgroups behind the SAME L2 needs exactly this on
// every storing wave, followed by a workgroup barrier, before the counter moves: a workgroup-scope
// fence alone emits no such wait (a workgroup shares its L1), and the counter's atomic, issued by one
// wave, could then reach the L2 ahead of another wave's data.
__device__ __forceinline__ void wait_own_stores() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// One atomic add of `inc` at p, issued by lane 0 only; returns the old value to all lanes.
__device__ __forceinline__ uint32_t wave_atomic_add(uint32_t* p, uint32_t inc) {
  uint32_t old;
  uint64_t saved_exec;
  asm volatile(
      "s_mov_b64 %1, exec\n\t"
      "s_mov_b64 exec, 1\n\t"
      "global_atomic_add %0, %2, %3, %4 sc0\n\t"
      "s_waitcnt vmcnt(0)\n\t"
      "s_mov_b64 exec, %1"
      : "=&v"(old), "=&s"(saved_exec)
      : "v"(0u), "v"(inc), "s"(p)
      : "memory");
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)old);
}

// One atomic OR of `bits` at p, issued by lane 0 only (no return value needed by the callers).
__device__ __forceinline__ void wave_atomic_or(uint32_t* p, uint32_t bits) {
  uint64_t saved_exec;
  asm volatile(
      "s_mov_b64 %0, exec\n\t"
      "s_mov_b64 exec, 1\n\t"
      "global_atomic_or %1, %2, %3\n\t"
      "s_waitcnt vmcnt(0)\n\t"
      "s_mov_b64 exec, %0"
      : "=&s"(saved_exec)
      : "v"(0u), "v"(bits), "s"(p)
      : "memory");
}

__device__ __forceinline__ uint32_t ev_load(const uint32_t* p) {
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// ---- Placement check ----
// The schedulers hand tiles over between the workgroups of one class (workgroup id % 8) through the L2 they
// share, which is sound only if a class really sits on ONE die.  Workgroups are dealt to the dies round-robin,
// continuing where the previous launch stopped, so class c is die (c + s) % 8 for some shift s as long as
// nothing (a CU mask, another partition mode) disturbs the dealing.  Instead of trusting that, every worker
// records the die it runs on in its class's byte of two mask words and then counts itself; once all workers
// are counted, a class is sound iff its byte has exactly one bit set.
// words[0] = workers counted, words[1..2] = masks (class c: byte c % 4 of word 1 + c / 4); all zero at launch.
// Called by a whole wave (wave-uniform); returns the count before this worker.  poison: record a second die.
__device__ __forceinline__ uint32_t placement_report(uint32_t* words, int cls, bool poison = false) {
  const int xcc = hw_xcc_id();
  const uint32_t bits = (xcc < kNumXcd && !poison) ? (1u << xcc) : 0xFFu;
  wave_atomic_or(&words[1 + (cls >> 2)], bits << ((cls & 3) * 8));   // acknowledged before the count moves
  return wave_atomic_add(&words[0], 1u);
}
__device__ __forceinline__ bool placement_class_ok(const uint32_t* words, int cls) {
  return __builtin_popcount((ev_load(&words[1 + (cls >> 2)]) >> ((cls & 3) * 8)) & 0xFFu) == 1;
}
__device__ __forceinline__ bool placement_all_ok(const uint32_t* words) {
  bool ok = true;
  for (int c = 0; c < kNumXcd; ++c) ok = ok && placement_class_ok(words, c);
  return ok;
}

}  // namespace moe
