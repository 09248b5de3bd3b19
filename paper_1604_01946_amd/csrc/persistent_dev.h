// Device-side helpers shared by the persistent recurrence kernels: bounded waits on step counters, signals,
// write-through stores for data that other workgroups read during the same launch.
#pragma once
#include "persistent.h"

namespace lstm {
namespace {

// ------------------------------------------------------------------ device helpers
template <int NT>
struct BVec;
template <>
struct BVec<1> {
  static __device__ __forceinline__ void ld(const float* p, float (&v)[1]) { v[0] = *p; }
};
template <>
struct BVec<2> {
  static __device__ __forceinline__ void ld(const float* p, float (&v)[2]) {
    const float2 t = *reinterpret_cast<const float2*>(p);
    v[0] = t.x; v[1] = t.y;
  }
};
template <>
struct BVec<4> {
  static __device__ __forceinline__ void ld(const float* p, float (&v)[4]) {
    const floatx4 t = *reinterpret_cast<const floatx4*>(p);
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
  }
};

// Synchronisation protocol.  Exchange data is written with agent-scope (write-through) stores,
// so publishing a step needs no L2 write-back: the producer waits for its stores to be
// acknowledged (vmcnt(0)), the workgroup meets at a barrier, and one thread bumps the step
// counter with an agent-scope atomic.  A consumer polls the counter with agent-scope loads and
// only then issues its first-ever loads of that exchange slot; no cache of its CU or XCD can
// hold those lines (every slot is written once per launch, slots are 128-byte aligned, and
// every workgroup invalidates its caches once when the kernel starts), so no invalidate is
// needed per step either.  `full` (LSTM_FULL_FENCES=1) swaps both sides for the compiler's
// agent-scope release / acquire fences (L2 write-back and invalidate on every step), which is
// several times slower and exists to cross-check the fast protocol.
// A step counter is split into kFlagSub words, each on a cache line of its own (kFlagStride ints
// apart).  Agent-scope atomics from many workgroups on one line are served one after the other by the
// memory side, about 25 ns each (6.4 us for 256 arrivals on one line, measured), so arrivals are spread
// over the lines by slice index and a waiter reads all of them with one load (lane i reads word i).

struct Waiter {
  int* watchdog;  // host-visible word, set when a wait expires
  int limit;
  bool dead;
  int full;
  // Non-blocking read of a counter (per lane: the arrivals on line lane, lanes >= kFlagSub report
  // "enough"); issue it early and hand the value to wait() later so that the round trip of the first
  // poll overlaps other work.
  static __device__ __forceinline__ int peek(int* flag) {
    const int lane = threadIdx.x & 63;
    return lane < kFlagSub ? __hip_atomic_load(flag + lane * kFlagStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : (1 << 30);
  }
  // The same without any branch or lane mask (lane i reads line i % kFlagSub), for reads issued in the
  // middle of pinned straight-line code: the value stays in flight until land() is called on it.
  static __device__ __forceinline__ int peek_all(int* flag) {
    return __hip_atomic_load(flag + (threadIdx.x & (kFlagSub - 1)) * kFlagStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // Marks the point where a peeked value is first needed; nothing that depends on it (and so no wait
  // for it) can be placed earlier.
  static __device__ __forceinline__ void land(int& v) { asm volatile("" : "+v"(v)); }
  // Waits until `target` workgroups (a multiple of kFlagSub, spread evenly) have arrived; `seen` is a
  // value peeked earlier (pass 0 if none, anything >= target to skip the wait).
  __device__ __forceinline__ void wait(int* flag, int target, int seen = 0) {
    const int each = target / kFlagSub;
    if (!dead && !__all(seen >= each)) {
      int spins = 0;
      while (!__all(peek(flag) >= each)) {
        __builtin_amdgcn_s_sleep(1);
        if (++spins > limit) {
          dead = true;
          __hip_atomic_store(watchdog, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
          break;
        }
      }
    }
    acquire();
  }
  // The same for a counter split into NSUB lines with its own arrival count per line.
  template <int NSUB>
  __device__ __forceinline__ void wait_split(int* flags, int target_each) {
    if (!dead) {
      const int lane = threadIdx.x & 63;
      int spins = 0;
      while (true) {
        const int v = lane < NSUB ? __hip_atomic_load(flags + lane * kFlagStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : target_each;
        if (__all(v >= target_each)) break;
        __builtin_amdgcn_s_sleep(1);
        if (++spins > limit) {
          dead = true;
          __hip_atomic_store(watchdog, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
          break;
        }
      }
    }
    acquire();
  }
  __device__ __forceinline__ void acquire() const {
    if (full)
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    else
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
  }
};

// Optional time-stamping of one workgroup's step phases (diagnostic hook lstm_debug_set_trace).
struct Tracer {
  long long* buf;  // [steps][8] wall-clock ticks (100 MHz), null when disabled
  __device__ __forceinline__ void mark(int step, int slot) const {
    if (buf && threadIdx.x == 0) {
      buf[(size_t)step * 8 + slot] = wall_clock64();
      if (slot == 0) buf[(size_t)step * 8 + 7] = clock64();  // shader clock, for the core frequency
    }
  }
};

// Store that other workgroups will read during this launch (write-through past the CU's cache): the exchange tiles
// are staged in LDS and written as whole 128-byte lines, 16 bytes per lane, which the memory side takes far better
// than scattered 4-byte write-through stores.
// A store of more than 8 bytes reads its data registers over several cycles after it has issued,
// and an instruction that overwrites them must keep its distance (two idle cycles on this
// architecture).  The compiler keeps that distance for its own stores but cannot see one inside
// inline assembly, so the idle cycles are part of the statement: without them the last lanes of a
// store were seen to carry the values written by the instructions that followed, once a second
// workgroup on the CU kept the address unit busy.
__device__ __forceinline__ void xstore4(float* p, floatx4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 3" ::"v"(p), "v"(v) : "memory");
}

// Makes a wave-uniform value opaque to the optimiser.  Offsets derived from a loop-invariant value
// are otherwise all computed ahead of the time loop, dozens of scalar registers that then live in
// VGPR lanes and are moved back and forth between the MFMAs of every step.
__device__ __forceinline__ void hide(int& v) { asm volatile("" : "+s"(v)); }

// Waits for every outstanding vector memory operation of the wave.  The counter is shared by loads and
// stores and decrements in issue order, so a later count-based wait for an old load also waits for
// every younger store; the second form tells the compiler (which does not read inline assembly) that
// nothing is outstanding, so registers loaded long ago are not waited for again behind later stores.
__device__ __forceinline__ void drain_vmem() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
}

// All threads have written; make it visible at agent scope and bump the counter once.
__device__ __forceinline__ void signal(int* flag, int full) {
  if (full)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  else
    drain_vmem();
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_fetch_add(flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Counter of NL lines: lane i polls line i % NL; every line must reach `each` arrivals.
template <int NL>
struct PpWaiter {
  int* watchdog;
  int limit;
  bool dead;
  static __device__ __forceinline__ int peek(int* flag) {
    return __hip_atomic_load(flag + (threadIdx.x & (NL - 1)) * kFlagStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  static __device__ __forceinline__ void land(int& v) { asm volatile("" : "+v"(v)); }
  // `seen`: a value peeked earlier.  A wait that has to poll ends with every outstanding memory operation complete.
  __device__ __forceinline__ void wait(int* flag, int each, int seen) {
    if (!dead && !__all(seen >= each)) {
      int spins = 0;
      while (!__all(peek(flag) >= each)) {
        __builtin_amdgcn_s_sleep(1);
        if (++spins > limit) {
          dead = true;
          __hip_atomic_store(watchdog, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
          break;
        }
      }
      drain_vmem();
    }
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
  }
};

struct PpTracer {
  long long* buf;  // [2 chains][T][8]
  int T;
  __device__ __forceinline__ void mark(int c, int step, int slot) const {
    if (buf && threadIdx.x == 0) {
      buf[((size_t)c * T + step) * 8 + slot] = wall_clock64();
      if (slot == 0) buf[((size_t)c * T + step) * 8 + 7] = clock64();
    }
  }
};

// blockIdx -> (layer, slice).  Workgroups are dealt round-robin to the 8 XCDs, each with its
// own L2; keeping a layer on 8/L XCDs lets its exchange reads be served by few L2s.
__device__ __forceinline__ void map_block(int L, int NS, int& l, int& s) {
  const int bid = blockIdx.x;
  if (L <= 8 && 8 % L == 0 && NS % (8 / L) == 0 && (gridDim.x % 8) == 0) {
    const int per = 8 / L, xcd = bid & 7;
    l = xcd / per;
    s = (bid >> 3) * per + (xcd % per);
  } else {
    l = bid / NS;
    s = bid % NS;
  }
}

}  // namespace
}  // namespace lstm
