// Barrier among the workgroups of one launch that run on the same accelerator die (XCD).
// MI355X hands the workgroups of a launch to its eight dies in turn, so workgroups i, i + 8,
// i + 16, ... share a die and its L2.  Work that is private to a die (the instances dealt to
// one tag machine, and the cells of those instances) can therefore run as a persistent loop
// with this barrier between dependent phases: every wave drains its stores into the shared L2
// before its workgroup arrives (s_waitcnt vmcnt(0)), so no L2 write-back or invalidation and no
// kernel boundary is needed.  The per-CU L1 is NOT
// invalidated: what crosses the barrier must be data the consumer's CU cannot hold an older copy
// of (rows written once per launch and read only afterwards), or be read past the L1.  The barrier words themselves are accessed at device scope, so the
// barrier completes wherever the workgroups run; every wait is bounded.
#pragma once
#ifndef __HIPCC_RTC__
#include <hip/hip_runtime.h>
#endif
#include <stdint.h>

namespace tdf {

constexpr uint32_t XCDS = 8;

struct alignas(128) DieSync {
  uint32_t count;      // arrivals (monotone: G per barrier)
  uint32_t pad;
  uint32_t xcc_mask;   // dies the workgroups of this group actually ran on
  uint32_t abort;      // a workgroup gave up waiting
};

// HW_REG_XCC_ID (20), bits 3:0: the die this wave runs on
__device__ __forceinline__ uint32_t xcc_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 15u; }

// Called by every thread of each of the G workgroups of a group, `gen` counting the group's
// barriers so far (all workgroups pass the same value).  Returns false if the wait exceeded
// spin_ticks (100 MHz ticks) or another workgroup had given up: the caller then leaves.
__device__ inline bool die_barrier(DieSync* sy, uint32_t G, uint32_t gen, long long spin_ticks, uint32_t* sh_ok) {
  // Release: each wave waits until the die's L2 has acknowledged all its outstanding stores (on this
  // architecture stores count in vmcnt; the workgroup barrier by itself does not wait for them), then
  // the workgroup meets, then one thread announces the arrival.  No L2 write-back is involved.
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (threadIdx.x == 0) {
    bool ok = true;
    // arrive without waiting for the old value; the count itself says when all G have arrived
    __hip_atomic_fetch_add(&sy->count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t full = (gen + 1u) * G;
    const long long t0 = wall_clock64();
    while (__atomic_load_n(&sy->count, __ATOMIC_RELAXED) < full) {
      __builtin_amdgcn_s_sleep(1);
      if (wall_clock64() - t0 > spin_ticks) {
        __atomic_store_n(&sy->abort, 1u, __ATOMIC_RELAXED);
        ok = false;
        break;
      }
    }
    if (__atomic_load_n(&sy->abort, __ATOMIC_RELAXED)) ok = false;
    *sh_ok = ok ? 1u : 0u;
  }
  __syncthreads();
  return *sh_ok != 0;
}

}  // namespace tdf
