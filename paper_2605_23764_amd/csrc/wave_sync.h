// Wave-uniform synchronisation primitives shared by the single-launch schedulers.
#pragma once
#include "common.h"

namespace moe {

constexpr int kNumXcd = 8;   // accelerator dies; workgroup b of a launch runs on XCD b % 8

// The scheduler's control flow is kept wave-uniform on purpose.  A lane-divergent
// `if (threadIdx.x == 0) { atomic }` at the head of a loop that also contains
// barriers was restructured by the compiler into nested loops in which lanes 1..63
// never left the inner (barrier + ticket read) loop, so no new ticket was ever drawn
// and the kernel spun forever.  Here wave 0 acts as a whole: single-lane atomics are
// issued with the execution mask narrowed inside one assembly statement, polls are
// uniform loads, and every branch below is scalar.

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

__device__ __forceinline__ uint32_t ev_load(const uint32_t* p) {
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

}  // namespace moe
