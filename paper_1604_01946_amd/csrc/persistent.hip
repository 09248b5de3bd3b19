// Persistent recurrence kernels: the whole T-step, L-layer recurrence in ONE
// launch, with the recurrent (and, for layers >= 1, the input) weights resident in registers.
//
// Section 4 of arXiv 1604.01946 names this as unexploited: the parameters are reused by every
// iteration and could live in a lower level of memory, at the price of a capacity limit and of
// assumptions outside the usual programming model (all blocks co-resident, blocks waiting on
// each other).  On gfx950 the register file of one CU is 512 KB, so a workgroup that owns 8
// hidden units keeps its [32 x 2H] slice of [W;R] (128 KB at H=512) in VGPRs as ready-made
// MFMA A operands for the whole sequence.  Co-residency comes from the grid never exceeding the
// number of CUs and from never having two such kernels in flight (see launch_resident); ordering comes from per-(layer, step) counters in device
// memory, released / acquired at agent scope, so that a layer only waits for the cells it
// really depends on -- cell (l, t) needs (l, t-1) and (l-1, t) -- and the layers run as the
// diagonal wavefront of Section 2.4 inside one grid.  Every wait is bounded: when the spin
// limit expires the waiter raises a host-visible word and stops waiting for the rest of the
// kernel, so the grid always drains.
//
// Forward data flow per step of workgroup (l, s):
//   input half     acc  = W_l[rows, :] * h_{l-1,t}      (layers >= 1; layer 0 adds the batched P_0)
//   recurrent half acc += R_l[rows, :] * h_{l,t-1}
//   epilogue       4-way K-split summed through LDS, gates, c_t, h_t; h_t goes to the reserve
//                  and, k-major ([H][BP]), to the exchange buffer the other workgroups read.
// MFMA shape v_mfma_f32_16x16x4_f32: M = 32 weight rows (unit-major, gate-minor; two tiles),
// N = batch, K split over the four waves.  The exchange buffer is k-major so that one 16-byte
// load per lane (4 consecutive batch entries of one k) feeds the B operands of the four batch
// tiles: tile j, column n is batch 4n + j.
//
// Contents, in order: device helpers (waits, signals, write-through stores); pers_fwd_kernel (tiles of 16 batch rows:
// B <= 32, and slices of 16 / 32 rows side by side); pers_fwd32_kernel (slices of 64 rows, 32x32x2 tiles; templated on
// the cell: LSTM, GRU, single gate) with its pack kernels; pers_bwd_kernel and pers_bwd32_kernel, the same pair for
// the backward recurrence; pers_fwdL_kernel / pers_bwdL_kernel (one layer per launch, H = 1024 / 2048, the recurrent
// matrix spread over all CUs); host side: residency checks and launches, which shapes run where, groups of layers
// for stacks deeper than the chip holds, batch slices.
#include "../../include/lstm.h"
#include "schedule.h"
#include "knobs.h"

#include <algorithm>
#include <mutex>
#include <stdlib.h>

namespace lstm {

#define CK(expr, what)                                             \
  do {                                                             \
    if (record((expr), what) != hipSuccess) return LSTM_HIP_ERROR; \
  } while (0)

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
constexpr int kFlagStride = 32;
constexpr int kFlagSub = 8;
constexpr int kFlagInts = kFlagSub * kFlagStride;  // ints per counter

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

struct PersFwdArgs {
  const float* W;     // flat input matrices; layers >= 1 are read
  const float* R;     // [L][4H][H]
  const float* bias;  // [L][4H]
  const float* P0;    // [T][B][4H] input projection of layer 0 (batched GEMM before the launch), unless xin is set
  const float* xin;   // wide kernel, I == H: x in exchange layout, [nsl][T+1][H*64] with slot t+1 = x_t; layer 0 then
                      // multiplies by W_0 itself, step by step, like the layers above it
  const float* c0;    // [L][B][H] or null
  const float* h0;    // [L][B][H] or null: read by the GRU variant of the wide kernel (its cell update needs h_{t-1})
  float* hx;          // [L][T+1][NC][H][BP] exchange, slot t+1 = h_t, slot 0 = h0
  int* flags;         // [L][T+1][NC], slot t+1 counts the slices of layer l that finished step t
  int* watchdog;
  float* res;         // reserve base
  float* y;
  float* hT;
  float* cT;
  int L, T, B, I, H;
  int b0;             // wide kernel: first batch row of this launch (a multiple of 64)
  int nsl;            // wide kernel: batch slices of 64 rows that run side by side in this launch (grid = nsl * L * H/8)
  int has_h0;
  int spin_limit;
  int full_fences;
  long long* trace;
  int trace_block;
  int keep;           // wide kernel: 0 = inference call (no reserve wanted): only y, hT, cT are written
};

// KG: k-groups (of 4) per wave and per operand half = H/16.  NT: batch tiles of 16 per chain.
// NC: batch chains.  The recurrences of different batch rows are independent, so the batch is cut
// into NC chains of 16*NT rows that share the resident weights but have their own exchange slots
// and counters; a workgroup alternates between them, and while one chain's h_t is on its way to
// the other workgroups the matrix cores work on the other chain.
template <int KG, int NT, int NC>
__global__ __launch_bounds__(256) void pers_fwd_kernel(const PersFwdArgs a) {
  constexpr int H = 16 * KG, G = 4 * H, BP = 16 * NT, NS = H / 8;
  constexpr int CPL = (2 * NT + 3) / 4;  // cells finalised per lane and chain
  __shared__ float part[4][2 * NT * 4][64];
  __shared__ __attribute__((aligned(16))) float xs[8 * BP];  // this step's h slice, [unit][batch]
  __shared__ __attribute__((aligned(16))) float ro[6 * BP * 8];  // gates, c, h of the slice: [array][batch][unit]

  // The recurrences of different batch rows are independent: slices of NC*BP rows run side by side as separate groups
  // of workgroups with their own exchange slots and counters (a.nsl of them, the first at batch row a.b0).
  int l, s;
  map_block(a.L, NS * a.nsl, l, s);
  const int sl = s / NS;
  s -= sl * NS;
  const int brow0 = a.b0 + NC * BP * sl;
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, n = lane & 15;
  const int u0 = 8 * s;
  const size_t TB = (size_t)T * B;

  // Register i of a wave covers k-group (i + rot) mod KG: workgroups (and waves) that share an L2
  // walk the exchange slot from different starting points instead of all hitting one channel.
  const int rot = ((int)(blockIdx.x >> 3) + __builtin_amdgcn_readfirstlane(wave)) & (KG - 1);
  // ---- weights -> registers, as MFMA A operands: lane (q, n) holds row n of tile mt at k = kbase + 4*kg + q
  float wR[KG][2], wW[KG][2];
  {
    const float* Rl = a.R + (size_t)l * G * H;
    const float* Wl = a.W + (size_t)4 * H * a.I + (size_t)(l > 0 ? l - 1 : 0) * G * H;
    const int kbase = wave * (H / 4) + q;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const int unit = u0 + 4 * mt + (n >> 2), gate = n & 3;
      const size_t row = ((size_t)gate * H + unit) * H;
#pragma unroll
      for (int i = 0; i < KG; ++i) {
        const int kg = (i + rot) & (KG - 1);
        wR[i][mt] = Rl[row + kbase + 4 * kg];
        wW[i][mt] = (l > 0) ? Wl[row + kbase + 4 * kg] : 0.f;
      }
    }
  }

  // ---- the cells this lane finalises: pair p = (tile mt, tile j) -> unit 4*mt+q, chain-local batch NT*n+j
  int c_unit[CPL], c_lb[CPL], c_p[CPL];
  float c_bias[CPL][4];
  bool c_valid[NC][CPL];
  float c_state[NC][CPL];
#pragma unroll
  for (int ci = 0; ci < CPL; ++ci) {
    const int p = wave + 4 * ci;
    c_p[ci] = p;
    const int mt = p / NT, j = p % NT;
    c_unit[ci] = u0 + 4 * mt + q;
    c_lb[ci] = NT * n + j;
#pragma unroll
    for (int g = 0; g < 4; ++g) c_bias[ci][g] = (p < 2 * NT) ? a.bias[(size_t)l * G + g * H + c_unit[ci]] : 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int bb = brow0 + c * BP + c_lb[ci];
      c_valid[c][ci] = (p < 2 * NT) && (bb < B);
      c_state[c][ci] = (c_valid[c][ci] && a.c0) ? a.c0[((size_t)l * B + bb) * H + c_unit[ci]] : 0.f;
    }
  }

  float* const res_l = a.res + (size_t)l * TB * 6 * H;
  float* const res_gates = res_l;
  float* const res_c = res_l + TB * 4 * H;
  float* const res_h = res_l + TB * 5 * H;
  const size_t boff = (size_t)(wave * (H / 4) + q) * BP + NT * n;  // this lane's B-operand offset inside a slot
  float* const hx = a.hx + (size_t)sl * a.L * (T + 1) * NC * H * BP;
  int* const flags = a.flags + (size_t)sl * a.L * (T + 1) * NC * kFlagInts;
  auto slot = [&](int layer, int st, int c) { return hx + (((size_t)layer * (T + 1) + st) * NC + c) * H * BP; };
  auto flag = [&](int layer, int st, int c) { return flags + (((size_t)layer * (T + 1) + st) * NC + c) * kFlagInts; };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2

  int rv = rot;
  for (int t = 0; t < T; ++t) {
    if (KG >= 32) hide(rv);  // large H: keeps the rotated offsets next to their loads instead of in spilled registers
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (c == 0) tr.mark(t, 0);
      floatx4 acc[2][NT];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[mt][j] = floatx4{0.f, 0.f, 0.f, 0.f};

      // layer 0: fetch the batched input projection early, it is consumed in the epilogue
      float pin[CPL][4];
#pragma unroll
      for (int ci = 0; ci < CPL; ++ci)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          pin[ci][g] = (l == 0 && c_valid[c][ci])
                           ? a.P0[((size_t)t * B + brow0 + c * BP + c_lb[ci]) * G + g * H + c_unit[ci]] : 0.f;

      // Loads are issued in bulk ahead of the MFMAs that consume them (the scheduling barriers keep
      // the compiler from re-serialising them): a step is bound by load latency otherwise.
      const bool do_in = l > 0, do_rec = (t > 0 || a.has_h0);
      // both counters are read at once, without branches, so that their round trips overlap (a counter that
      // does not apply is replaced by one that exists; its value is not used)
      int seen_in = Waiter::peek_all(do_in ? flag(l - 1, t + 1, c) : flag(l, t > 0 ? t : 1, c));
      int seen_rec = Waiter::peek_all(flag(l, t > 0 ? t : 1, c));
      float bi[KG][NT], br[KG][NT];
      if (do_in) {  // input half: h of the layer below at this step
        Waiter::land(seen_in);
        w.wait(flag(l - 1, t + 1, c), NS, seen_in);
        const float* src = slot(l - 1, t + 1, c) + boff;
#pragma unroll
        for (int i = 0; i < KG; ++i) BVec<NT>::ld(src + (size_t)4 * ((i + rv) & (KG - 1)) * BP, bi[i]);
        if (c == 0) tr.mark(t, 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < KG / 2; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wW[i][mt], bi[i][j], acc[mt][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (do_rec) {  // recurrent half: own layer, previous step; its loads fly under the rest of the input half
        Waiter::land(seen_rec);
        if (t > 0) w.wait(flag(l, t, c), NS, seen_rec);
        if (c == 0) tr.mark(t, 2);
        const float* src = slot(l, t, c) + boff;
#pragma unroll
        for (int i = 0; i < KG; ++i) BVec<NT>::ld(src + (size_t)4 * ((i + rv) & (KG - 1)) * BP, br[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (do_in) {
#pragma unroll
        for (int i = KG / 2; i < KG; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wW[i][mt], bi[i][j], acc[mt][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (do_rec) {
#pragma unroll
        for (int i = 0; i < KG; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wR[i][mt], br[i][j], acc[mt][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }

      // ---- 4-way K-split reduction through LDS
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) part[wave][(mt * NT + j) * 4 + r][lane] = acc[mt][j][r];
      if (c == 0) tr.mark(t, 3);
      __syncthreads();
      if (c == 0) tr.mark(t, 4);

      // ---- epilogue: register r of lane (q, n) in tile (mt, j) is (unit 4*mt+q, gate r, batch NT*n+j)
      float o_gate[CPL][4], o_c[CPL], o_h[CPL];
#pragma unroll
      for (int ci = 0; ci < CPL; ++ci) {
        if (c_p[ci] < 2 * NT) {
          float sg[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = c_p[ci] * 4 + r;
            sg[r] = (part[0][row][lane] + part[1][row][lane]) + (part[2][row][lane] + part[3][row][lane]) +
                    pin[ci][r] + c_bias[ci][r];
          }
          o_gate[ci][0] = sigmoidf_dev(sg[0]);
          o_gate[ci][1] = sigmoidf_dev(sg[1]);
          o_gate[ci][2] = sigmoidf_dev(sg[2]);
          o_gate[ci][3] = tanhf_dev(sg[3]);
          o_c[ci] = o_gate[ci][1] * c_state[c][ci] + o_gate[ci][0] * o_gate[ci][3];
          o_h[ci] = o_gate[ci][2] * tanhf_dev(o_c[ci]);
          c_state[c][ci] = o_c[ci];
          xs[(c_unit[ci] - u0) * BP + c_lb[ci]] = c_valid[c][ci] ? o_h[ci] : 0.f;
        }
      }
      __syncthreads();
      if (threadIdx.x < 2 * BP)  // the slice's 8 rows are contiguous in the k-major exchange slot
        xstore4(slot(l, t + 1, c) + (size_t)u0 * BP + 4 * threadIdx.x, *reinterpret_cast<const floatx4*>(xs + 4 * threadIdx.x));
      if (c == 0) tr.mark(t, 5);
      signal(flag(l, t + 1, c) + (s & (kFlagSub - 1)) * kFlagStride, a.full_fences);  // publish h_t (the barrier also protects `part` and `xs`)
      if (c == 0) tr.mark(t, 6);
      // The reserve and the outputs are not read before the kernel ends, so they are written after
      // the signal -- staged through LDS so that each store instruction writes 16-byte runs
      // (scattered 4-byte stores keep the address unit busy for longer than the whole epilogue).
#pragma unroll
      for (int ci = 0; ci < CPL; ++ci) {
        if (c_p[ci] < 2 * NT) {
          const int ul = c_unit[ci] - u0;
#pragma unroll
          for (int g = 0; g < 4; ++g) ro[(g * BP + c_lb[ci]) * 8 + ul] = o_gate[ci][g];
          ro[(4 * BP + c_lb[ci]) * 8 + ul] = o_c[ci];
          ro[(5 * BP + c_lb[ci]) * 8 + ul] = o_h[ci];
        }
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < (12 * BP + 255) / 256; ++i) {
        const int idx = threadIdx.x + 256 * i;  // (array 0..5, chain-local batch row, half of the 8 units)
        const int arr = idx / (2 * BP), lb = (idx >> 1) % BP, hf = idx & 1;
        const int b2 = brow0 + c * BP + lb;
        if (idx < 12 * BP && b2 < B) {
          const floatx4 v = *reinterpret_cast<const floatx4*>(ro + (arr * BP + lb) * 8 + 4 * hf);
          const size_t e = ((size_t)t * B + b2) * H + u0 + 4 * hf;
          if (arr < 4) {
            *reinterpret_cast<floatx4*>(res_gates + ((size_t)t * B + b2) * G + (size_t)arr * H + u0 + 4 * hf) = v;
          } else if (arr == 4) {
            *reinterpret_cast<floatx4*>(res_c + e) = v;
            if (t == T - 1 && a.cT) *reinterpret_cast<floatx4*>(a.cT + ((size_t)l * B + b2) * H + u0 + 4 * hf) = v;
          } else {
            *reinterpret_cast<floatx4*>(res_h + e) = v;
            if (l == a.L - 1) *reinterpret_cast<floatx4*>(a.y + e) = v;
            if (t == T - 1 && a.hT) *reinterpret_cast<floatx4*>(a.hT + ((size_t)l * B + b2) * H + u0 + 4 * hf) = v;
          }
        }
      }
    }
  }
}

// h0 [L][B][H] -> exchange slot 0 of every slice, layer and chain, k-major [H][BP]; rows past the batch are zero.
__global__ void pack_state_kernel(const float* __restrict__ h0, float* __restrict__ hx, int L, int T, int B, int H,
                                  int BP, int NC, int b0, int nsl) {
  const long n = (long)nsl * L * NC * BP * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long)gridDim.x * blockDim.x) {
    const int lb = (int)(e % BP);
    long r = e / BP;
    const int k = (int)(r % H); r /= H;
    const int c = (int)(r % NC); r /= NC;
    const int l = (int)(r % L);
    const int sl = (int)(r / L);
    const int bb = b0 + (sl * NC + c) * BP + lb;
    hx[((((size_t)sl * L + l) * (T + 1)) * NC + c) * H * BP + (size_t)k * BP + lb] =
        bb < B ? h0[((size_t)l * B + bb) * H + k] : 0.f;
  }
}

// ------------------------------------------------------------------ forward, wide-batch variant
// Same decomposition as pers_fwd_kernel (8 hidden units x all batch rows per workgroup) for
// 32 < B <= 64, on v_mfma_f32_32x32x2_f32: with one wave per SIMD the 16x16x4 shape issues at about
// three quarters of the fp32 matrix rate, the 32x32 shape at nearly all of it.  M = 32 weight rows
// ordered gate-major (row = 8*gate + unit) so that, in the D layout, a lane holds all four gates of
// four units; N = two tiles of 32 batch rows (tile j, column n = batch 2n + j).
// Exchange layout of one (layer, step) slot: for k = 4*k4 + 2*m + kk and batch b = 2n + j, element
// ((k4*2 + kk)*32 + n)*4 + 2*m + j -- lane (kk, n) fetches two k-pairs of both tiles with one
// 16-byte load, 1 KB per wave and instruction.
// CELL = 1 runs a GRU on the same machinery (convention of rnn.h: gates r, z, n; the reset gate multiplies the
// recurrent product): the four row groups of a workgroup's tile are then r, z, the input half of n (W_n x, no
// recurrent weights) and the recurrent half of n (R_n h, no input weights) -- a quarter of the MFMA work
// multiplies zeros, everything else is unchanged.  Its reserve is h [T][B][H] followed by r, z, n, R_n h as [T][B][4H].
// CELL = 2 / 3: single-gate RNN with ReLU / tanh: only the first row group carries weights (three quarters of the
// MFMA work multiply zeros -- these small cells are bound by the synchronisation of a step, not by the products);
// the reserve is h [T][B][H].
template <int HH, int CELL>
__global__ __launch_bounds__(256) void pers_fwd32_kernel(const PersFwdArgs a) {
  constexpr int H = HH, NG = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1), G = NG * H, NS = H / 8;  // G: rows of W, R, b and of the projection P0
  constexpr int NK4 = H / 16;  // 4-k groups per wave and operand half
  __shared__ float part[4][32][64];
  __shared__ __attribute__((aligned(16))) float xs[512];  // this step's h slice in exchange order
  __shared__ __attribute__((aligned(16))) float ro[6 * 64 * 8];  // gates, c, h of the slice: [array][batch][unit]

  // The recurrences of different batch rows are independent: slices of 64 rows run side by side as
  // separate groups of workgroups with their own exchange slots and counters.
  int l, s;
  map_block(a.L, NS * a.nsl, l, s);
  const int sl = s / NS;
  s -= sl * NS;
  const int b0 = a.b0 + 64 * sl;
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kk = lane >> 5, n = lane & 31;
  const int u0 = 8 * s;
  const size_t TB = (size_t)T * B;
  const int rot = ((int)(blockIdx.x >> 3) + __builtin_amdgcn_readfirstlane(wave)) & (NK4 - 1);

  // ---- weights -> registers: A operand row rho = lane%32 = (gate rho/8, unit rho%8), k = wave*H/4 + 4*k4 + 2*m + kk
  float wR[NK4][2], wW[NK4][2];
  {
    const float* Rl = a.R + (size_t)l * G * H;
    const float* Wl = l > 0 ? a.W + (size_t)G * a.I + (size_t)(l - 1) * G * H : a.W;  // layer 0: [G][I], read if I == H
    const int grp = n >> 3;
    // matrix row behind tile row group grp: the gate itself (LSTM); r, z, n (input half), n (recurrent half) for the GRU
    const int gate = CELL >= 2 ? 0 : ((CELL == 1 && grp == 3) ? 2 : grp);
    const bool useR = CELL == 0 || (CELL == 1 ? grp != 2 : grp == 0);
    const bool useW = (CELL == 0 || (CELL == 1 ? grp != 3 : grp == 0)) && (l > 0 || a.xin);
    const size_t row = ((size_t)gate * H + u0 + (n & 7)) * H;
#pragma unroll
    for (int i = 0; i < NK4; ++i) {
      const int k4 = (i + rot) & (NK4 - 1);
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        const int k = wave * (H / 4) + 4 * k4 + 2 * m + kk;
        wR[i][m] = useR ? Rl[row + k] : 0.f;
        wW[i][m] = useW ? Wl[row + k] : 0.f;
      }
    }
  }

  // ---- the two cells this lane finalises: wave w takes batch tile j = w%2 and unit pair up = w/2;
  //      D register r of a lane is row 8*(r/4) + 4*kk + r%4 = (gate r/4, unit 4*kk + r%4)
  const int tj = wave & 1, up = wave >> 1;
  const int lb = 2 * n + tj;   // batch row inside this launch's 64
  const int bb = b0 + lb;      // batch row in the tensors
  const bool valid = bb < B;
  int c_unit[2];
  float c_state[2], c_bias[2][4];  // c_state: c_{t-1} (LSTM), h_{t-1} (GRU)
#pragma unroll
  for (int ci = 0; ci < 2; ++ci) {
    c_unit[ci] = u0 + 4 * kk + 2 * up + ci;
    const float* const s0 = CELL == 0 ? a.c0 : (CELL == 1 ? a.h0 : nullptr);
    c_state[ci] = (valid && s0) ? s0[((size_t)l * B + bb) * H + c_unit[ci]] : 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g) c_bias[ci][g] = g < NG ? a.bias[(size_t)l * G + g * H + c_unit[ci]] : 0.f;
  }

  float* const res_l = a.res + (size_t)l * TB * (CELL == 0 ? 6 : (CELL == 1 ? 5 : 1)) * H;
  float* const res_gates = CELL == 0 ? res_l : res_l + TB * H;  // the four saved arrays, [T][B][4H]
  float* const res_c = res_l + TB * 4 * H;                       // LSTM only
  float* const res_h = CELL == 0 ? res_l + TB * 5 * H : res_l;
  float* const hx = a.hx + (size_t)sl * a.L * (T + 1) * H * 64;
  int* const flags = a.flags + (size_t)sl * a.L * (T + 1) * kFlagInts;
  auto slot = [&](int layer, int st) { return hx + ((size_t)layer * (T + 1) + st) * H * 64; };
  auto flag = [&](int layer, int st) { return flags + ((size_t)layer * (T + 1) + st) * kFlagInts; };
  const size_t boff = (size_t)wave * NK4 * 256 + lane * 4;  // this lane's offset inside a slot

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2

  // One 16-byte load of a lane feeds four MFMAs (two k-pairs x two batch tiles).  `rv` is `rot`
  // made opaque once per step (see hide()), so that the rotated offsets are computed next to their
  // loads with a few scalar instructions.
  int rv = rot;
  auto ldx = [&](const float* src, int i) {
    return *reinterpret_cast<const floatx4*>(src + (size_t)((i + rv) & (NK4 - 1)) * 256);
  };

  // ---- everything after the MFMAs of step t: K-split reduction, gates, publish h_t, reserve
  auto finish_step = [&](const floatx16 (&acc)[2], const float (&pin)[2][4], const int t) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) part[wave][j * 16 + r][lane] = acc[j][r];
    tr.mark(t, 3);
    __syncthreads();
    tr.mark(t, 4);
    float o_gate[2][4], o_c[2], o_h[2];
#pragma unroll
    for (int ci = 0; ci < 2; ++ci) {
      float sg[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int row = tj * 16 + 4 * g + 2 * up + ci;
        sg[g] = (part[0][row][lane] + part[1][row][lane]) + (part[2][row][lane] + part[3][row][lane]) +
                pin[ci][g] + c_bias[ci][g];
      }
      if (CELL == 0) {
        o_gate[ci][0] = sigmoidf_dev(sg[0]);
        o_gate[ci][1] = sigmoidf_dev(sg[1]);
        o_gate[ci][2] = sigmoidf_dev(sg[2]);
        o_gate[ci][3] = tanhf_dev(sg[3]);
        o_c[ci] = o_gate[ci][1] * c_state[ci] + o_gate[ci][0] * o_gate[ci][3];
        o_h[ci] = o_gate[ci][2] * tanhf_dev(o_c[ci]);
        c_state[ci] = o_c[ci];
      } else if (CELL >= 2) {
#pragma unroll
        for (int g = 0; g < 4; ++g) o_gate[ci][g] = 0.f;
        o_h[ci] = CELL == 3 ? tanhf_dev(sg[0]) : fmaxf(sg[0], 0.f);
        o_c[ci] = 0.f;
      } else {  // sg: r and z pre-activations, W_n x + b_n, R_n h
        o_gate[ci][0] = sigmoidf_dev(sg[0]);
        o_gate[ci][1] = sigmoidf_dev(sg[1]);
        o_gate[ci][2] = tanhf_dev(sg[2] + o_gate[ci][0] * sg[3]);
        o_gate[ci][3] = sg[3];
        o_h[ci] = (1.f - o_gate[ci][1]) * o_gate[ci][2] + o_gate[ci][1] * c_state[ci];
        o_c[ci] = 0.f;
        c_state[ci] = o_h[ci];
      }
      // unit offset ul = 4*kk + 2*up + ci: k4 block ul/4 = kk, m = up, parity ci; batch (n, tj)
      xs[kk * 256 + (ci * 32 + n) * 4 + 2 * up + tj] = valid ? o_h[ci] : 0.f;
    }
    __syncthreads();
    if (threadIdx.x < 128)  // the slice's 8 units are two contiguous 1 KB blocks of the exchange slot
      xstore4(slot(l, t + 1) + (size_t)(u0 / 4) * 256 + 4 * threadIdx.x, *reinterpret_cast<const floatx4*>(xs + 4 * threadIdx.x));
    tr.mark(t, 5);
    signal(flag(l, t + 1) + (s & (kFlagSub - 1)) * kFlagStride, a.full_fences);  // publish h_t (the barrier also protects `part` and `xs`)
    tr.mark(t, 6);
    // The reserve and the outputs are not read before the kernel ends, so they are written after the
    // signal -- staged through LDS so that each store instruction writes 16-byte runs (scattered
    // 4-byte stores keep the address unit busy for longer than the whole epilogue).  An inference call
    // has nothing to write for the lower layers except the final states.
    if (!(a.keep || l == a.L - 1 || t == T - 1)) return;
#pragma unroll
    for (int ci = 0; ci < 2; ++ci) {
      const int ul = 4 * kk + 2 * up + ci;
#pragma unroll
      for (int g = 0; g < 4; ++g) ro[(g * 64 + lb) * 8 + ul] = o_gate[ci][g];
      ro[(4 * 64 + lb) * 8 + ul] = o_c[ci];
      ro[(5 * 64 + lb) * 8 + ul] = o_h[ci];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int idx = threadIdx.x + 256 * i;  // (array 0..5, batch row, half of the 8 units)
      const int arr = idx >> 7, l2 = (idx >> 1) & 63, hf = idx & 1;
      const int b2 = b0 + l2;
      if (b2 < B) {
        const floatx4 v = *reinterpret_cast<const floatx4*>(ro + (arr * 64 + l2) * 8 + 4 * hf);
        const size_t e = ((size_t)t * B + b2) * H + u0 + 4 * hf;
        if (arr < 4) {
          if (CELL <= 1 && a.keep) *reinterpret_cast<floatx4*>(res_gates + ((size_t)t * B + b2) * 4 * H + (size_t)arr * H + u0 + 4 * hf) = v;
        } else if (arr == 4) {
          if (CELL == 0) {
            if (a.keep) *reinterpret_cast<floatx4*>(res_c + e) = v;
            if (t == T - 1 && a.cT) *reinterpret_cast<floatx4*>(a.cT + ((size_t)l * B + b2) * H + u0 + 4 * hf) = v;
          }
        } else {
          if (a.keep) *reinterpret_cast<floatx4*>(res_h + e) = v;
          if (l == a.L - 1) *reinterpret_cast<floatx4*>(a.y + e) = v;
          if (t == T - 1 && a.hT) *reinterpret_cast<floatx4*>(a.hT + ((size_t)l * B + b2) * H + u0 + 4 * hf) = v;
        }
      }
    }
  };

  if (l == 0 && !a.xin) {
    // ---- layer 0: the input half is the batched projection P_0 (added in the epilogue); its values
    //      for the next step are fetched one step ahead, behind the exchange loads, so that a miss to
    //      HBM never sits in front of a counter poll (loads return in order).
    float pin[2][4];
#pragma unroll
    for (int ci = 0; ci < 2; ++ci)
#pragma unroll
      for (int g = 0; g < 4; ++g) pin[ci][g] = (valid && g < NG) ? a.P0[(size_t)bb * G + g * H + c_unit[ci]] : 0.f;
    for (int t = 0; t < T; ++t) {
      tr.mark(t, 0);
      hide(rv);
      floatx16 acc[2];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
      if (t > 0) w.wait(flag(0, t), NS);  // slot 0 (h0 or zeros) was written before the launch
      tr.mark(t, 2);
      const float* src = slot(0, t) + boff;
      floatx4 br[NK4];
#pragma unroll
      for (int i = 0; i < NK4; ++i) br[i] = ldx(src, i);
      float pnx[2][4];
#pragma unroll
      for (int ci = 0; ci < 2; ++ci)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          pnx[ci][g] = (valid && t + 1 < T && g < NG) ? a.P0[((size_t)(t + 1) * B + bb) * G + g * H + c_unit[ci]] : 0.f;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NK4; ++i)
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wR[i][m], br[i][2 * m + j], acc[j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      finish_step(acc, pin, t);
#pragma unroll
      for (int ci = 0; ci < 2; ++ci)
#pragma unroll
        for (int g = 0; g < 4; ++g) pin[ci][g] = pnx[ci][g];
    }
    return;
  }

  // ---- layers >= 1.  Order of one step, in k-groups of 4:
  //   1. input MFMAs on the first half of h_{l-1,t}, already in registers; the second half is fetched
  //      between them.  This part also covers the time the own layer's h_{t-1} needs to become visible.
  //   2. wait for h_{l,t-1}; input MFMAs on the second half, the recurrent operand fetched between them.
  //   3. recurrent MFMAs; between the first of them the first half of h_{l-1,t+1} is fetched if the
  //      layer below (which normally runs ahead) has published it.  If it has not, the same loads
  //      re-read the current step's slot -- valid memory, values unused -- so that the step is one
  //      straight line of code, and the operand is fetched after a wait at the end of the step.
  // Loads are issued between MFMAs rather than in bulk (a bulk of 32 16-byte loads per wave holds the
  // wave in the address unit for about a microsecond while the matrix cores idle); the scheduling
  // barriers pin that order.  Only half an operand is carried from step to step, which keeps the
  // kernel inside the register file.
  // The layer below is, for layer 0 with I == H, the input sequence itself: x in exchange layout, all
  // of it there before the launch, with one counter that reads "published" for every step.
  constexpr int HK = NK4 / 2;
  const float zero_pin[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  const float* const in_base = l > 0 ? slot(l - 1, 0) : a.xin + (size_t)sl * (T + 1) * H * 64;
  int* const in_flag_base = l > 0 ? flag(l - 1, 0) : a.flags + (size_t)a.nsl * a.L * (T + 1) * kFlagInts;
  const int in_flag_step = l > 0 ? kFlagInts : 0;
  auto in_slot = [&](int st) { return in_base + (size_t)st * H * 64; };
  auto in_flag = [&](int st) { return in_flag_base + (size_t)st * in_flag_step; };
  floatx4 bl[HK];
  w.wait(in_flag(1), NS);
  {
    const float* src = in_slot(1) + boff;
#pragma unroll
    for (int i = 0; i < HK; ++i) bl[i] = ldx(src, i);
    drain_vmem();
  }
  for (int t = 0; t < T; ++t) {
    tr.mark(t, 0);
    hide(rv);
    floatx16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    auto mma4 = [&](const float (&wgt)[2], const floatx4& bv) {
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wgt[m], bv[2 * m + j], acc[j], 0, 0, 0);
    };
    // both counters are read now; the answers arrive under the MFMAs of part 1
    // (slots that do not exist at the ends of the sequence are replaced by ones that do; their values are not used)
    int seen_rec = Waiter::peek_all(flag(l, t > 0 ? t : 1));
    int seen_in = Waiter::peek_all(in_flag(t + 1 < T ? t + 2 : t + 1));
    floatx4 bh[HK], br[NK4];
    {
      const float* src = in_slot(t + 1) + boff;
      tr.mark(t, 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < HK; ++i) {
        bh[i] = ldx(src, HK + i);
        mma4(wW[i], bl[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    Waiter::land(seen_rec);
    w.wait(flag(l, t), NS, t > 0 ? seen_rec : NS);  // h_{l,t-1}; slot 0 (h0 or zeros) was written before the launch
    tr.mark(t, 2);
    {
      const float* src = slot(l, t) + boff;
#pragma unroll
      for (int i = 0; i < HK; ++i) {
        br[2 * i] = ldx(src, 2 * i);
        br[2 * i + 1] = ldx(src, 2 * i + 1);
        mma4(wW[HK + i], bh[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    const bool more = t + 1 < T;
    Waiter::land(seen_in);
    const bool pre = more && __all(seen_in >= NS / kFlagSub) && !w.dead;
    {
      const float* nsrc = in_slot(pre ? t + 2 : t + 1) + boff;
#pragma unroll
      for (int i = 0; i < NK4; ++i) {
        if (i < HK) bl[i] = ldx(nsrc, i);
        mma4(wR[i], br[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    finish_step(acc, zero_pin, t);
    if (more && !pre) {  // the layer below was late: wait for it now, after this step is published
      w.wait(in_flag(t + 2), NS);
      const float* src = in_slot(t + 2) + boff;
#pragma unroll
      for (int i = 0; i < HK; ++i) bl[i] = ldx(src, i);
      drain_vmem();
    }
  }
}

// h0 [L][B][H] (zeros if null) -> exchange slot 0 of every layer in the layout of pers_fwd32_kernel.
__global__ void pack_state32_kernel(const float* __restrict__ h0, float* __restrict__ hx, int L, int T, int B, int H, int b0,
                                    int nsl) {
  const long cnt = (long)nsl * L * 64 * H;  // all 64 batch columns of every slot: rows past the batch hold zeros
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < cnt; e += (long)gridDim.x * blockDim.x) {
    const int k = (int)(e % H), lb = (int)((e / H) % 64), l = (int)((e / ((long)H * 64)) % L);
    const int sl = (int)(e / ((long)H * 64 * L));
    const int k4 = k >> 2, m = (k >> 1) & 1, kk = k & 1, n = lb >> 1, j = lb & 1;
    const int bb = b0 + 64 * sl + lb;
    hx[(((size_t)sl * L + l) * (T + 1)) * H * 64 + ((size_t)(k4 * 2 + kk) * 32 + n) * 4 + 2 * m + j] =
        (h0 && bb < B) ? h0[((size_t)l * B + bb) * H + k] : 0.f;
  }
}

// x [T][B][H] (I == H) -> exchange layout of pers_fwd32_kernel, slots 1..T of xin [nsl][T+1][H*64], rows past the
// batch zero; also sets the counter that stands for "every step of the input is published" (nsl*L*(T+1) counters
// into `flags`).  Block (kb, t, sl) moves the 64 batch rows x 64 inputs [64*kb, 64*kb+64) of one step through LDS:
// whole rows in, one contiguous 16 KB piece of the slot out.
__global__ __launch_bounds__(256) void pack_x32_kernel(const float* __restrict__ x, float* __restrict__ xin, int* flags,
                                                       int L, int T, int B, int H, int b0, int nsl, int ready) {
  __shared__ float tile[64][65];
  const int kb = blockIdx.x, t = blockIdx.y, sl = blockIdx.z;
  if (kb == 0 && t == 0 && sl == 0 && threadIdx.x < kFlagSub)
    flags[(size_t)nsl * L * (T + 1) * kFlagInts + threadIdx.x * kFlagStride] = ready;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int e = threadIdx.x + 256 * i, lb = e >> 6, kc = e & 63;
    const int bb = b0 + 64 * sl + lb;
    tile[lb][kc] = bb < B ? x[((size_t)t * B + bb) * H + 64 * kb + kc] : 0.f;
  }
  __syncthreads();
  float* const dst = xin + ((size_t)sl * (T + 1) + t + 1) * H * 64 + (size_t)kb * 4096;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int o = threadIdx.x + 256 * i;  // 16-byte piece: ((k4*2 + kk)*32 + n), holding (m, j) = (0,0) (0,1) (1,0) (1,1)
    const int n = o & 31, kk = (o >> 5) & 1, k4 = o >> 6;
    floatx4 v;
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = tile[2 * n + (q & 1)][4 * k4 + 2 * (q >> 1) + kk];
    *reinterpret_cast<floatx4*>(dst + 4 * o) = v;
  }
}

// ------------------------------------------------------------------ backward
// Workgroup (l, s) owns hidden units u0..u0+7 of layer l.  Per step t (descending) and batch chain:
//   point-wise   dh_t = dout_t + dh_rec,  gate gradients dA_t (4 x 8 x BP values), dc carry;
//                dA_t goes to the standard [T][B][4H] array (weight-gradient GEMMs) and, k-major
//                ([4H][BP]), to the exchange buffer;
//   GEMM         [dh_rec_{t-1} ; dx_{l,t}] (16 rows) = [R_l[:, units] | W_l[:, units]]^T * dA_t, K = 4H:
//                rows 0-7 stay in registers for the next point-wise step, rows 8-15 are the gradient
//                for the same units of layer l-1 at step t (its dout) and go to dxbuf; for layer 0 they
//                are the gradient of the network input and go to the caller's dx when I == H (the
//                tile rows would otherwise multiply zeros), else a batched GEMM follows the launch.
// Section 2.1's remark on the backward pass (four gate gradients map to one output through the
// stacked matrices) is the K = 4H contraction; wave w takes the K range of gate w.
// Counters: slot t+1 of layer l = "point-wise of step t published" (which, by program order, also
// covers dx of step t+1); slot 0 = "dx of step 0 published".
struct PersBwdArgs {
  const float* W;      // flat input matrices (layer 0's only when dx0 is set)
  const float* R;      // [L][4H][H]
  const float* res;    // reserve written by the forward pass
  const float* c0;     // [L][B][H] or null
  const float* dy;     // [T][B][H]
  const float* dhT;    // [L][B][H] or null
  const float* dcT;    // [L][B][H] or null
  float* dA;           // [L][T][B][4H] gate gradients (standard layout)
  float* dAx;          // [L][T][NC][4H][BP] exchange
  float* dxbuf;        // [L][T][B][H] gradient for the layer below (slice l written by layer l, l >= 1)
  float* dx0;          // [T][B][I] gradient of the network input, written by layer 0 when I == H; else null
  float* dh0;          // [L][B][H] or null
  float* dc0;          // [L][B][H] or null
  float* db;           // [L][4H] bias gradient, zeroed before the launch (wide kernel only), or null
  int* flags;          // [L][T+1][NC]
  int* watchdog;
  int L, T, B, I, H;
  int b0;              // first batch row of this launch (a multiple of the slice height)
  int spin_limit;
  int full_fences;
  long long* trace;
  int trace_block;
  const float* h0;     // [L][B][H] or null: read by the GRU variant of the wide kernel
};

// KGB: k-groups (of 4) per wave = H/4 (wave w covers the rows of gate w).  NT, NC as in the forward kernel.
template <int KGB, int NT, int NC>
__global__ __launch_bounds__(256) void pers_bwd_kernel(const PersBwdArgs a) {
  constexpr int H = 4 * KGB, G = 4 * H, BP = 16 * NT, NS = H / 8;
  __shared__ float part[4][NT * 4][64];
  __shared__ __attribute__((aligned(16))) float xs[32 * BP];  // this step's dA slice, [gate][unit][batch]

  // Slices of NC*BP batch rows side by side, as in the forward kernel: the grid holds one group of L*NS workgroups
  // per slice, the first slice starts at batch row a.b0.
  const int nsl = (int)gridDim.x / (a.L * NS);
  int l, s;
  map_block(a.L, NS * nsl, l, s);
  const int sl = s / NS;
  s -= sl * NS;
  const int brow0 = a.b0 + NC * BP * sl;
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, n = lane & 15;
  const int u0 = 8 * s;
  const size_t TB = (size_t)T * B;

  // ---- weights -> registers: A operand row n (< 8: column u0+n of R_l, >= 8: column u0+n-8 of W_l),
  //      k = wave*H + 4*kg + q
  const int rot = ((int)(blockIdx.x >> 3) * (KGB / 32) + 2 * __builtin_amdgcn_readfirstlane(wave)) & (KGB - 1);
  float wB[KGB];
  {
    const float* Rl = a.R + (size_t)l * G * H;
    const float* Wl = a.W + (size_t)4 * H * a.I + (size_t)(l > 0 ? l - 1 : 0) * G * H;
    const float* src = (n < 8) ? Rl + u0 + n : (l > 0 ? Wl : a.W) + u0 + (n - 8);  // layer 0: its own [4H][I], I == H
    const bool live = (n < 8) || (l > 0) || a.dx0;
#pragma unroll
    for (int i = 0; i < KGB; ++i)
      wB[i] = live ? src[(size_t)(wave * H + 4 * ((i + rot) & (KGB - 1)) + q) * H] : 0.f;
  }

  // ---- the cells this lane owns in the point-wise stage: wave j finalises batch tile j;
  //      lanes q < 2 hold dh_rec of units 4q..4q+3, lanes q >= 2 hold dx of units 4(q-2)..+3
  const int lb = NT * n + wave;                     // chain-local batch row
  const bool fin = wave < NT;                       // this wave finalises a tile
  const int unit0 = u0 + 4 * (q & 1);               // first of the lane's four units
  bool pw[NC], dxl[NC];
  float dc[NC][4], dh_rec[NC][4];
  int seen_up[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int bb = brow0 + c * BP + lb;
    pw[c] = fin && q < 2 && bb < B;                 // lane runs the point-wise stage
    dxl[c] = fin && q >= 2 && bb < B && (l > 0 || a.dx0);
    seen_up[c] = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const size_t se = ((size_t)l * B + bb) * H + unit0 + r;
      dc[c][r] = (pw[c] && a.dcT) ? a.dcT[se] : 0.f;
      dh_rec[c][r] = (pw[c] && a.dhT) ? a.dhT[se] : 0.f;
    }
  }

  const float* const res_l = a.res + (size_t)l * TB * 6 * H;
  const float* const res_gates = res_l;
  const float* const res_c = res_l + TB * 4 * H;
  float* const dA_l = a.dA + (size_t)l * TB * G;
  const bool has_up = l < a.L - 1;
  const float* const dout_base = has_up ? a.dxbuf + (size_t)(l + 1) * TB * H : a.dy;
  float* const dx_out = l > 0 ? a.dxbuf + (size_t)l * TB * H : a.dx0;
  const size_t boff = (size_t)(wave * H + q) * BP + NT * n;
  float* const dAx = a.dAx + (size_t)sl * a.L * T * NC * G * BP;
  int* const flags = a.flags + (size_t)sl * a.L * (T + 1) * NC * kFlagInts;
  auto slot = [&](int t, int c) { return dAx + (((size_t)l * T + t) * NC + c) * G * BP; };
  auto flag = [&](int layer, int st, int c) { return flags + (((size_t)layer * (T + 1) + st) * NC + c) * kFlagInts; };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2

  // Reserve values (and, for the top layer, dy) of the step the point-wise stage handles next.  They do
  // not depend on any counter, so they are fetched one step ahead, behind the exchange loads of the
  // previous step: loads return in order, and a miss to HBM in front of the counter polls would
  // otherwise stall every poll behind it.
  floatx4 gi[NC], gf[NC], go[NC], gg[NC], ct[NC], cp[NC], dpre[NC];
  auto fetch_step = [&](int t, int c) {
    if (pw[c]) {
      const int bb = brow0 + c * BP + lb;
      const size_t e = ((size_t)t * B + bb) * H + unit0;
      const size_t g0 = ((size_t)t * B + bb) * G + unit0;
      gi[c] = *reinterpret_cast<const floatx4*>(res_gates + g0);
      gf[c] = *reinterpret_cast<const floatx4*>(res_gates + g0 + H);
      go[c] = *reinterpret_cast<const floatx4*>(res_gates + g0 + 2 * H);
      gg[c] = *reinterpret_cast<const floatx4*>(res_gates + g0 + 3 * H);
      ct[c] = *reinterpret_cast<const floatx4*>(res_c + e);
      if (t > 0)
        cp[c] = *reinterpret_cast<const floatx4*>(res_c + e - (size_t)B * H);
      else if (a.c0)
        cp[c] = *reinterpret_cast<const floatx4*>(a.c0 + ((size_t)l * B + bb) * H + unit0);
      else
        cp[c] = floatx4{0.f, 0.f, 0.f, 0.f};
      if (!has_up) dpre[c] = *reinterpret_cast<const floatx4*>(a.dy + e);
    }
  };
#pragma unroll
  for (int c = 0; c < NC; ++c) fetch_step(T - 1, c);

  int rv = rot;
  for (int t = T - 1; t >= 0; --t) {
    hide(rv);  // keeps the rotated offsets next to their loads
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (c == 0) tr.mark(t, 0);
      const int bb = brow0 + c * BP + lb;
      // ---- point-wise stage of step t
      floatx4 dA4[4];
      const size_t e = ((size_t)t * B + bb) * H + unit0;
      const size_t g0 = ((size_t)t * B + bb) * G + unit0;
      Waiter::land(seen_up[c]);
      if (has_up) w.wait(flag(l + 1, t, c), NS, seen_up[c]);  // dx of the layer above at step t is published
      if (c == 0) tr.mark(t, 1);
      if (fin && q < 2 && !pw[c]) {  // padded batch columns of the staged tile
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int g = 0; g < 4; ++g) xs[(g * 8 + (unit0 - u0) + r) * BP + lb] = 0.f;
      }
      if (pw[c]) {
        const floatx4 dout = has_up ? *reinterpret_cast<const floatx4*>(dout_base + e) : dpre[c];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float dh = dout[r] + dh_rec[c][r];
          const float tc = tanhf_dev(ct[c][r]);
          const float dcv = dc[c][r] + dh * go[c][r] * (1.f - tc * tc);
          dA4[0][r] = dcv * gg[c][r] * gi[c][r] * (1.f - gi[c][r]);
          dA4[1][r] = dcv * cp[c][r] * gf[c][r] * (1.f - gf[c][r]);
          dA4[2][r] = dh * tc * go[c][r] * (1.f - go[c][r]);
          dA4[3][r] = dcv * gi[c][r] * (1.f - gg[c][r] * gg[c][r]);
          dc[c][r] = dcv * gf[c][r];
#pragma unroll
          for (int g = 0; g < 4; ++g) xs[(g * 8 + (unit0 - u0) + r) * BP + lb] = dA4[g][r];
        }
      }
      __syncthreads();
      {  // per gate the slice's 8 rows are contiguous in the k-major exchange slot
        float* const xo = slot(t, c);
#pragma unroll
        for (int i = 0; i < (8 * BP + 255) / 256; ++i) {
          const int idx = threadIdx.x + 256 * i;
          if (idx < 8 * BP) {
            const int g = idx / (2 * BP), rem = idx % (2 * BP);
            xstore4(xo + (size_t)(g * H + u0) * BP + 4 * rem, *reinterpret_cast<const floatx4*>(xs + 4 * idx));
          }
        }
      }
      if (c == 0) tr.mark(t, 2);
      signal(flag(l, t + 1, c) + (s & (kFlagSub - 1)) * kFlagStride, a.full_fences);
      if (c == 0) tr.mark(t, 3);
      if (pw[c]) {
#pragma unroll
        for (int g = 0; g < 4; ++g) *reinterpret_cast<floatx4*>(dA_l + g0 + (size_t)g * H) = dA4[g];
      }

      // ---- GEMM of step t: needs dA_t of every slice of this layer
      w.wait(flag(l, t + 1, c), NS);
      if (c == 0) tr.mark(t, 4);
      // counter of the layer above for the next point-wise stage, read without a branch and consumed there
      // (the top layer reads its own, already complete counter instead)
      seen_up[c] = Waiter::peek_all(has_up ? flag(l + 1, t > 0 ? t - 1 : 0, c) : flag(l, t + 1, c));
      floatx4 acc[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
      {
        const float* src = slot(t, c) + boff;
        // double-buffered chunks of CH k-groups: the loads of chunk i+1 are in flight under the MFMAs
        // of chunk i (the scheduling barriers keep the compiler from re-serialising them)
        constexpr int CH = (KGB >= 64) ? 32 : 16, NCH = KGB / CH;
        float bv[2][CH][NT];
#pragma unroll
        for (int i = 0; i < CH; ++i) BVec<NT>::ld(src + (size_t)4 * ((i + rv) & (KGB - 1)) * BP, bv[0][i]);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          if (ch + 1 < NCH) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
              BVec<NT>::ld(src + (size_t)4 * (((ch + 1) * CH + i + rv) & (KGB - 1)) * BP, bv[(ch + 1) & 1][i]);
          }
          if (ch == (NCH > 1 ? NCH - 2 : 0) && t > 0) fetch_step(t - 1, c);  // behind this step's last exchange loads
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < CH; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wB[ch * CH + i], bv[ch & 1][i][j], acc[j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[wave][j * 4 + r][lane] = acc[j][r];
      if (c == 0) tr.mark(t, 5);
      __syncthreads();
      if (c == 0) tr.mark(t, 6);
      if (fin) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = wave * 4 + r;
          v[r] = (part[0][row][lane] + part[1][row][lane]) + (part[2][row][lane] + part[3][row][lane]);
        }
        if (q < 2) {
#pragma unroll
          for (int r = 0; r < 4; ++r) dh_rec[c][r] = v[r];
        } else if (dxl[c]) {
          xstore4(dx_out + ((size_t)t * B + bb) * H + unit0, floatx4{v[0], v[1], v[2], v[3]});
        }
      }
      // `part` is next written after the barriers of the next point-wise stage
    }
  }
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    signal(flag(l, 0, c) + (s & (kFlagSub - 1)) * kFlagStride, a.full_fences);  // slot 0: dx of step 0 published
    if (pw[c]) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const size_t se = ((size_t)l * B + brow0 + c * BP + lb) * H + unit0 + r;
        if (a.dh0) a.dh0[se] = dh_rec[c][r];
        if (a.dc0) a.dc0[se] = dc[c][r];
      }
    }
  }
}

// ------------------------------------------------------------------ backward, wide-batch variant
// For 32 < B <= 64 the kernel above is bound by L2->CU bandwidth: every workgroup reads the whole
// dA_t (4H x 64 values per step).  This variant halves that traffic by giving a workgroup 16 hidden
// units of ONE half of the batch: M = 32 rows (16 dh_rec + 16 dx), N = 32 batch rows, which is one
// v_mfma_f32_32x32x2_f32 tile (the fp32 MFMA shape that issues at full rate with one wave per
// SIMD).  Its weight slice is [32 x 4H] = 256 KB at H = 512: the first 128 k-pairs of every wave
// stay in VGPRs, the rest sit in LDS (152 KB of the CU's 160 KB are used).  The two batch halves
// never exchange data, so they are placed on different XCDs.
// Exchange layout of one (layer, step, half) slot: for k = 8*k8 + 2*m + kk and batch row n,
// element ((k8*2 + kk)*32 + n)*4 + m -- lane (kk, n) of a wave fetches the four k-pairs of an
// 8-k group with one 16-byte load, 1 KB per wave and instruction.
// CELL = 1: GRU (see pers_fwd32_kernel).  The four K groups are then the gradients with respect to the r and z
// pre-activations, to W_n x + b_n, and to R_n h; the recurrent rows of the tile have no weights in the third group,
// the input rows none in the fourth, and dh_{t-1} also receives dh_t o z_t directly.  The arrays c0 / dcT / dc0 of
// the arguments are not used; `res` is the GRU reserve, W / R / db have 3H rows.
// CELL = 2 / 3: single-gate RNN (ReLU / tanh): only the first K group is non-zero; `res` holds h alone.
template <int HH, int CELL>
__global__ __launch_bounds__(256) void pers_bwd32_kernel(const PersBwdArgs a, const int NBH) {
  constexpr int H = HH, G = 4 * H, NS2 = H / 16;  // G: width of the gate-gradient arrays (four groups for both cells)
  constexpr int NG = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1), GW = NG * H;  // rows of W, R, db
  constexpr int NB8 = H / 8;                 // 8-k groups per wave (wave w covers the rows of gate w)
  constexpr int KPW = H / 2;                 // k-pairs per wave
  constexpr int RP = KPW < 128 ? KPW : 128;  // k-pairs whose weights live in registers
  constexpr int LP = KPW - RP;               // k-pairs whose weights live in LDS
  constexpr int DEPTH = NB8 < 16 ? NB8 : 16;  // 8-k groups whose exchange loads are in flight ahead of the MFMAs
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* const part = smem;         // [4 waves][16 regs][64 lanes]
  float* const xs = smem + 4096;    // [8 blocks of 8 k][256]: this step's dA slice in exchange order
  float* const wl = smem + 6144;    // [4 waves][LP][64 lanes]

  // blockIdx -> (layer, batch half, slice): one (layer, half) group per 8/(L*NBH) XCDs when that divides
  int l, bh, s2;
  {
    const int bid = blockIdx.x, groups = a.L * NBH;
    if (groups <= 8 && 8 % groups == 0 && NS2 % (8 / groups) == 0 && (gridDim.x % 8) == 0) {
      const int per = 8 / groups, xcd = bid & 7, grp = xcd / per;
      l = grp / NBH;
      bh = grp % NBH;
      s2 = (bid >> 3) * per + (xcd % per);
    } else {
      l = bid / (NS2 * NBH);
      bh = (bid / NS2) % NBH;
      s2 = bid % NS2;
    }
  }
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kk = lane >> 5, n = lane & 31;
  const int u0 = 16 * s2;
  const size_t TB = (size_t)T * B;
  const int rot = ((int)(blockIdx.x >> 3) * (NB8 / 32 > 0 ? NB8 / 32 : 1) + 2 * __builtin_amdgcn_readfirstlane(wave)) & (NB8 - 1);

  // ---- weights: A operand row rho = lane%32 (< 16: column u0+rho of R_l, >= 16: column u0+rho-16 of W_l)
  float wreg[RP];
  {
    const float* Rl = a.R + (size_t)l * GW * H;
    const float* Wl = a.W + (size_t)GW * a.I + (size_t)(l > 0 ? l - 1 : 0) * GW * H;
    const float* src = (n < 16) ? Rl + u0 + n : (l > 0 ? Wl : a.W) + u0 + (n - 16);  // layer 0: its own [GW][I], I == H
    // matrix row block behind K group `wave`: the gate itself (LSTM); GRU: r, z, then n for the input rows only,
    // then n for the recurrent rows only
    const int gate = CELL >= 2 ? 0 : ((CELL == 1 && wave == 3) ? 2 : wave);
    const bool live = ((n < 16) || (l > 0) || a.dx0) &&
                      (CELL == 0 || (CELL == 1 ? (n < 16 ? wave != 2 : wave != 3) : wave == 0));
#pragma unroll
    for (int i = 0; i < KPW; ++i) {
      const int k8 = ((i >> 2) + rot) & (NB8 - 1), m = i & 3;
      const float v = live ? src[(size_t)(gate * H + 8 * k8 + 2 * m + kk) * H] : 0.f;
      if (i < RP)
        wreg[i < RP ? i : 0] = v;
      else
        wl[((size_t)wave * LP + (i - RP)) * 64 + lane] = v;
    }
  }

  // ---- roles: waves 0,1 run the point-wise stage on units u0 + 8*wave + 4*kk + {0..3};
  //      waves 2,3 publish dx of units u0 + 8*(wave-2) + 4*kk + {0..3}; batch row bh*32 + n
  const int bb = a.b0 + bh * 32 + n;  // batch row in the tensors; the exchange slots hold this launch's 64 rows
  const bool pwv = wave < 2 && bb < B;
  const bool dxl = wave >= 2 && bb < B && (l > 0 || a.dx0);
  const int unit0 = u0 + 8 * (wave & 1) + 4 * kk;
  float dc[4], dh_rec[4];  // dc: carried cell gradient (LSTM); the direct term dh_t o z_t (GRU)
  float dbsum[4][4];  // this lane's share of the bias gradient: sum over t of dA_t, per (gate, unit)
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const size_t se = ((size_t)l * B + bb) * H + unit0 + r;
    dc[r] = (CELL == 0 && pwv && a.dcT) ? a.dcT[se] : 0.f;
    dh_rec[r] = (pwv && a.dhT) ? a.dhT[se] : 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g) dbsum[g][r] = 0.f;
  }

  const float* const res_l = a.res + (size_t)l * TB * (CELL == 0 ? 6 : (CELL == 1 ? 5 : 1)) * H;
  const float* const res_gates = CELL == 0 ? res_l : res_l + TB * H;  // the four saved arrays, [T][B][4H] (LSTM, GRU)
  const float* const res_c = CELL == 0 ? res_l + TB * 4 * H : res_l;   // c (LSTM) or h: the state array the step reads
  const float* const s0 = CELL == 0 ? a.c0 : a.h0;
  float* const dA_l = a.dA + (size_t)l * TB * G;
  const bool has_up = l < a.L - 1;
  const float* const dout_base = has_up ? a.dxbuf + (size_t)(l + 1) * TB * H : a.dy;
  float* const dx_out = l > 0 ? a.dxbuf + (size_t)l * TB * H : a.dx0;
  auto slot = [&](int t) { return a.dAx + (((size_t)l * T + t) * NBH + bh) * G * 32; };
  auto flag = [&](int layer, int sl) { return a.flags + (((size_t)layer * (T + 1) + sl) * NBH + bh) * kFlagInts; };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2
  __syncthreads();                                    // LDS weights are in place

  // Reserve values (and, for the top layer, dy) of the step the point-wise stage handles next.  They do
  // not depend on any counter, so they are fetched one step ahead, under the MFMAs of the previous
  // step: loads return in order, and a miss to HBM in front of the counter polls would otherwise
  // stall every poll behind it.
  floatx4 gi, gf, go, gg, ct, cp, dpre;
  auto fetch_step = [&](int t) {
    if (pwv) {
      const size_t e = ((size_t)t * B + bb) * H + unit0;
      const size_t g0 = ((size_t)t * B + bb) * G + unit0;
      if (CELL <= 1) {
        gi = *reinterpret_cast<const floatx4*>(res_gates + g0);
        gf = *reinterpret_cast<const floatx4*>(res_gates + g0 + H);
        go = *reinterpret_cast<const floatx4*>(res_gates + g0 + 2 * H);
        gg = *reinterpret_cast<const floatx4*>(res_gates + g0 + 3 * H);
      }
      if (CELL != 1) ct = *reinterpret_cast<const floatx4*>(res_c + e);  // c_t (LSTM), h_t (single gate)
      if (CELL <= 1) {
        if (t > 0)
          cp = *reinterpret_cast<const floatx4*>(res_c + e - (size_t)B * H);
        else if (s0)
          cp = *reinterpret_cast<const floatx4*>(s0 + ((size_t)l * B + bb) * H + unit0);
        else
          cp = floatx4{0.f, 0.f, 0.f, 0.f};
      }
    }
  };
  // The upstream gradient of step t (dy, or dx of the layer above) is fetched with them when it is there:
  // `t_src` is t if it is published, else a step whose row this lane has already read (valid memory, value unused).
  auto fetch_dout = [&](int t_src) {
    if (pwv) dpre = *reinterpret_cast<const floatx4*>(dout_base + ((size_t)t_src * B + bb) * H + unit0);
  };
  fetch_step(T - 1);
  bool dpre_ok = !has_up;
  if (dpre_ok) fetch_dout(T - 1);

  int seen_up = 0;
  for (int t = T - 1; t >= 0; --t) {
    tr.mark(t, 0);
    // ---- point-wise stage of step t
    floatx4 dA4[4];
    const size_t e = ((size_t)t * B + bb) * H + unit0;
    const size_t g0 = ((size_t)t * B + bb) * G + unit0;
    if (has_up) w.wait(flag(l + 1, t), NS2, seen_up);  // dx of the layer above at step t is published
    tr.mark(t, 1);
    if (wave < 2) {
      floatx4 dout = {0.f, 0.f, 0.f, 0.f};
      if (pwv) dout = dpre_ok ? dpre : *reinterpret_cast<const floatx4*>(dout_base + e);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (pwv) {
          const float dh = dout[r] + dh_rec[r];
          if (CELL == 0) {
            const float tc = tanhf(ct[r]);
            const float dcv = dc[r] + dh * go[r] * (1.f - tc * tc);
            dA4[0][r] = dcv * gg[r] * gi[r] * (1.f - gi[r]);
            dA4[1][r] = dcv * cp[r] * gf[r] * (1.f - gf[r]);
            dA4[2][r] = dh * tc * go[r] * (1.f - go[r]);
            dA4[3][r] = dcv * gi[r] * (1.f - gg[r] * gg[r]);
            dc[r] = dcv * gf[r];
          } else if (CELL >= 2) {  // ct holds h_t
            dA4[0][r] = CELL == 3 ? dh * (1.f - ct[r] * ct[r]) : (ct[r] > 0.f ? dh : 0.f);
            dA4[1][r] = dA4[2][r] = dA4[3][r] = 0.f;
          } else {  // gi, gf, go, gg hold r, z, n, R_n h; cp holds h_{t-1}
            const float dn = dh * (1.f - gf[r]) * (1.f - go[r] * go[r]);
            dA4[0][r] = dn * gg[r] * gi[r] * (1.f - gi[r]);
            dA4[1][r] = dh * (cp[r] - go[r]) * gf[r] * (1.f - gf[r]);
            dA4[2][r] = dn;
            dA4[3][r] = dn * gi[r];
            dc[r] = dh * gf[r];
          }
#pragma unroll
          for (int g = 0; g < 4; ++g) dbsum[g][r] += dA4[g][r];
        }
        // unit u0 + 8*wave + 4*kk + r sits at k%8 = 4*kk + r of block (gate, wave): m = 2*kk + r/2, parity r%2
#pragma unroll
        for (int g = 0; g < 4; ++g)
          xs[(g * 2 + wave) * 256 + ((r & 1) * 32 + n) * 4 + 2 * kk + (r >> 1)] = pwv ? dA4[g][r] : 0.f;
      }
    }
    __syncthreads();
    {  // eight 1 KB blocks (gate x unit-octet), each contiguous in the exchange slot
      float* const xo = slot(t);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int idx = threadIdx.x + 256 * i, blk = idx >> 6, off = idx & 63;
        const int g = blk >> 1, o8 = blk & 1;
        xstore4(xo + ((size_t)(g * H + u0) / 8 + o8) * 256 + off * 4, *reinterpret_cast<const floatx4*>(xs + blk * 256 + off * 4));
      }
    }
    tr.mark(t, 2);
    signal(flag(l, t + 1) + (s2 & (kFlagSub - 1)) * kFlagStride, a.full_fences);
    tr.mark(t, 3);
    if (pwv) {
#pragma unroll
      for (int g = 0; g < 4; ++g) *reinterpret_cast<floatx4*>(dA_l + g0 + (size_t)g * H) = dA4[g];
    }

    // ---- GEMM of step t: needs dA_t of every slice of this layer and batch half
    w.wait(flag(l, t + 1), NS2);
    tr.mark(t, 4);
    // counter of the layer above for the next point-wise stage: read now, looked at under the MFMAs
    // (the top layer reads its own, already complete counter instead, so that this is one straight line)
    seen_up = Waiter::peek_all(has_up ? flag(l + 1, t > 0 ? t - 1 : 0) : flag(l, t + 1));
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    {
      // One 16-byte exchange load feeds the four MFMAs of an 8-k group.  The loads run DEPTH groups
      // ahead of the MFMAs and are issued between them (so is the LDS part of the weights, two groups
      // ahead): issued in bulk they would hold the wave in the address unit while the matrix cores
      // idle.  The scheduling barrier after every group keeps this order.
      const float* src = slot(t) + (size_t)wave * NB8 * 256 + lane * 4;
      floatx4 bv[NB8];
      float al[NB8][4];
      int rv = rot;
      hide(rv);  // keeps the rotated offsets next to their loads
      auto ldb = [&](int g) { bv[g] = *reinterpret_cast<const floatx4*>(src + (size_t)((g + rv) & (NB8 - 1)) * 256); };
      auto ldw = [&](int g) {
        if (g * 4 >= RP) {
#pragma unroll
          for (int m = 0; m < 4; ++m) al[g][m] = wl[((size_t)wave * LP + (g * 4 + m - RP)) * 64 + lane];
        }
      };
#pragma unroll
      for (int g = 0; g < DEPTH; ++g) ldb(g);
      ldw(0);
      if (NB8 > 1) ldw(1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < NB8; ++g) {
        if (g + DEPTH < NB8) ldb(g + DEPTH);
        if (g + 2 < NB8) ldw(g + 2);
        if (g == NB8 - DEPTH) {  // behind the last exchange load of this step
          Waiter::land(seen_up);
          dpre_ok = t > 0 && (!has_up || (__all(seen_up >= NS2 / kFlagSub) && !w.dead));
          if (t > 0) fetch_step(t - 1);
          fetch_dout(dpre_ok ? t - 1 : t);
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const int pr = g * 4 + m;
          const float av = (pr < RP) ? wreg[pr < RP ? pr : 0] : al[g][m];
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[g][m], acc, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) part[(wave * 16 + r) * 64 + lane] = acc[r];
    tr.mark(t, 5);
    __syncthreads();
    tr.mark(t, 6);
    {
      // register r of a lane is row 8*(r/4) + 4*kk + r%4: wave w sums registers 4w..4w+3 = rows 8w+4kk+{0..3}
      float v[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = 4 * wave + r;
        v[r] = (part[(0 * 16 + row) * 64 + lane] + part[(1 * 16 + row) * 64 + lane]) +
               (part[(2 * 16 + row) * 64 + lane] + part[(3 * 16 + row) * 64 + lane]);
      }
      if (wave < 2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) dh_rec[r] = CELL == 1 ? v[r] + dc[r] : v[r];
      } else if (dxl) {
        xstore4(dx_out + ((size_t)t * B + bb) * H + unit0, floatx4{v[0], v[1], v[2], v[3]});
      }
    }
    // `part` and `xs` are next written after the barriers of the next point-wise stage
  }
  signal(flag(l, 0) + (s2 & (kFlagSub - 1)) * kFlagStride, a.full_fences);  // slot 0: dx of step 0 published
  if (pwv) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const size_t se = ((size_t)l * B + bb) * H + unit0 + r;
      if (a.dh0) a.dh0[se] = dh_rec[r];
      if (CELL == 0 && a.dc0) a.dc0[se] = dc[r];
    }
  }
  // Bias gradient (Section 2.6 lists it with the weight update): the per-lane sums over t are added
  // over the 32 batch rows of this workgroup through LDS and then into db.  Each element of db
  // receives exactly one contribution per batch half, and a + b does not depend on which of the
  // two arrives first, so the result is reproducible.
  if (a.db) {
    if (wave < 2) {
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int g = 0; g < 4; ++g) part[(g * 16 + 8 * wave + 4 * kk + r) * 32 + n] = dbsum[g][r];
    }
    __syncthreads();
    if (threadIdx.x < 16 * NG) {
      const int g = threadIdx.x >> 4, ul = threadIdx.x & 15;
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 32; ++i) sum += part[threadIdx.x * 32 + ((i + threadIdx.x) & 31)];
      atomicAdd(a.db + (size_t)l * GW + g * H + u0 + ul, sum);
    }
  }
}

// ------------------------------------------------------------------ one layer, large hidden size
// Section 4 of arXiv 1604.01946 puts the limit of the persistent approach at the capacity of the
// on-chip memory.  On MI355X the 256 CUs together hold 128 MB of registers and 40 MB of LDS, so a
// whole [4H x H] recurrent matrix of H = 2048 (64 MiB) fits: every workgroup keeps the 32 rows of
// 8 hidden units (4 gates x 8 units x H floats = 256 KB) for all T steps, half of it in VGPRs and half
// in LDS, exactly the split of pers_bwd32_kernel.  One launch runs one layer (all CUs are needed for
// it, so the layers cannot overlap); the layer's input projection is a batched GEMM before it, as for
// layer 0 above.  Per step a workgroup multiplies its [32 x H] slice by h_{t-1} ([H x 32 batch rows],
// read from the exchange slot), K split over the four waves, and finalises 8 units x 32 batch rows.
// Exchange layout of a slot (H x 32 floats): for k = wave*H/4 + 8*k8 + 2*m + kk and batch row n,
// element (wave*H/32 + k8)*256 + ((kk*32 + n)*4 + m) -- the 8 units of slice s are one contiguous KB.
struct PersFwdLArgs {
  const float* R;     // [4H][H] of this layer
  const float* bias;  // [4H]
  const float* P;     // [T][B][4H] input projection of this layer
  const float* c0;    // [B][H] or null
  float* hx;          // [T+1][H*32] exchange, slot t+1 = h_t, slot 0 = h0 (or zeros)
  int* flags;         // [T+1][16][kFlagStride]: slot t+1 counts the slices that published h_t, spread over 16 lines
  int* watchdog;
  float* res;         // reserve of this layer
  float* y;           // [T][B][H] or null (top layer only)
  float* hT;          // [B][H] or null
  float* cT;          // [B][H] or null
  int T, B;
  int b0;             // first batch row of this launch (a multiple of 32)
  int nsl;            // batch slices of 32 rows side by side in this launch (grid = nsl * H/8), each with its own
                      // exchange slots and counters
  int spin_limit;
  int full_fences;
  long long* trace;
  int trace_block;
};

// CELL as in pers_fwd32_kernel (0 LSTM, 1 GRU, 2 / 3 single gate with ReLU / tanh).  Only recurrent weights live here
// (the input projection P is a batched product), so the GRU's four row groups are r, z, an empty one and R_n, and P's
// third block (W_n x) is added in the epilogue; the single gate uses the first group alone.
template <int HH, int CELL>
__global__ __launch_bounds__(256) void pers_fwdL_kernel(const PersFwdLArgs a) {
  constexpr int H = HH, NG = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1), G = NG * H, NS = H / 8;  // G: rows of R, bias, P
  constexpr int NB8 = H / 32;                // 8-k groups per wave
  constexpr int KPW = H / 8;                 // k-pairs per wave
  constexpr int RP = KPW < 128 ? KPW : 128;  // k-pairs whose weights live in registers
  constexpr int LP = KPW - RP;               // k-pairs whose weights live in LDS
  constexpr int DEPTH = NB8 < 16 ? NB8 : 16;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* const part = smem;         // [4 waves][16 regs][64 lanes]
  float* const xs = smem + 4096;    // [256]: this step's h slice in exchange order
  float* const ro = smem + 4352;    // [6 arrays][32 batch rows][8 units]
  float* const wl = smem + 6144;    // [4 waves][LP][64 lanes]

  const int sl = blockIdx.x / NS, s = blockIdx.x % NS, u0 = 8 * s;
  const int T = a.T, B = a.B, b0 = a.b0 + 32 * sl;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kk = lane >> 5, n = lane & 31;
  const size_t TB = (size_t)T * B;
  const int rot = ((int)(blockIdx.x >> 3) * (NB8 / 32 > 0 ? NB8 / 32 : 1) + 2 * __builtin_amdgcn_readfirstlane(wave)) & (NB8 - 1);
  float* const hx = a.hx + (size_t)sl * (T + 1) * H * 32;
  int* const flags = a.flags + (size_t)sl * (T + 1) * 16 * kFlagStride;

  // ---- weights: A operand row rho = lane%32 = (gate rho/8, unit rho%8); register / LDS entry i covers
  //      k = wave*H/4 + 8*((i/4 + rot) mod NB8) + 2*(i%4) + kk
  float wreg[RP];
  {
    const int grp = n >> 3;
    const int gate = CELL >= 2 ? 0 : ((CELL == 1 && grp == 3) ? 2 : grp);
    const bool live = CELL == 0 || (CELL == 1 ? grp != 2 : grp == 0);
    const float* src = a.R + ((size_t)gate * H + u0 + (n & 7)) * H + (size_t)wave * (H / 4) + kk;
#pragma unroll
    for (int i = 0; i < KPW; ++i) {
      const int k8 = ((i >> 2) + rot) & (NB8 - 1), m = i & 3;
      const float v = live ? src[8 * k8 + 2 * m] : 0.f;
      if (i < RP)
        wreg[i < RP ? i : 0] = v;
      else
        wl[((size_t)wave * LP + (i - RP)) * 64 + lane] = v;
    }
  }

  // ---- the cell this thread finalises: unit u0 + 4*kk + wave, batch row n (D register 4*gate + wave)
  const int uj = 4 * kk + wave;
  const int bb = b0 + n;  // batch row in the tensors
  const bool valid = bb < B;
  float c_state = (CELL <= 1 && valid && a.c0) ? a.c0[(size_t)bb * H + u0 + uj] : 0.f;  // c_{t-1} (LSTM), h_{t-1} (GRU: a.c0 = h0)
  float c_bias[4], pin[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    c_bias[g] = g < NG ? a.bias[g * H + u0 + uj] : 0.f;
    pin[g] = (valid && g < NG) ? a.P[(size_t)bb * G + g * H + u0 + uj] : 0.f;
  }
  float* const res_gates = CELL == 0 ? a.res : a.res + TB * H;  // the four saved arrays [T][B][4H] (LSTM, GRU)
  float* const res_c = a.res + TB * 4 * H;                       // LSTM only
  float* const res_h = CELL == 0 ? a.res + TB * 5 * H : a.res;
  auto slot = [&](int st) { return hx + (size_t)st * H * 32; };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2
  __syncthreads();                                    // LDS weights are in place

  int rv = rot;
  for (int t = 0; t < T; ++t) {
    tr.mark(t, 0);
    hide(rv);  // keeps the rotated offsets next to their loads
    if (t > 0) w.template wait_split<16>(flags + (size_t)16 * kFlagStride * t, NS / 16);  // slot 0 was written before the launch
    tr.mark(t, 2);
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float pnx[4];
    {
      const float* src = slot(t) + (size_t)wave * NB8 * 256 + lane * 4;
      floatx4 bv[NB8];
      float al[NB8][4];
      auto ldb = [&](int g) { bv[g] = *reinterpret_cast<const floatx4*>(src + (size_t)((g + rv) & (NB8 - 1)) * 256); };
      auto ldw = [&](int g) {
        if (g * 4 >= RP) {
#pragma unroll
          for (int m = 0; m < 4; ++m) al[g][m] = wl[((size_t)wave * LP + (g * 4 + m - RP)) * 64 + lane];
        }
      };
#pragma unroll
      for (int g = 0; g < DEPTH; ++g) ldb(g);
      ldw(0);
      if (NB8 > 1) ldw(1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < NB8; ++g) {
        if (g + DEPTH < NB8) ldb(g + DEPTH);
        if (g + 2 < NB8) ldw(g + 2);
        if (g == NB8 - DEPTH) {  // next step's input projection, behind the last exchange load of this step
#pragma unroll
          for (int q = 0; q < 4; ++q)
            pnx[q] = (valid && t + 1 < T && q < NG) ? a.P[((size_t)(t + 1) * B + bb) * G + q * H + u0 + uj] : 0.f;
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const int pr = g * 4 + m;
          const float av = (pr < RP) ? wreg[pr < RP ? pr : 0] : al[g][m];
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[g][m], acc, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) part[(wave * 16 + r) * 64 + lane] = acc[r];
    tr.mark(t, 3);
    __syncthreads();
    tr.mark(t, 4);
    float sg[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int r = 4 * g + wave;
      sg[g] = (part[(0 * 16 + r) * 64 + lane] + part[(1 * 16 + r) * 64 + lane]) +
              (part[(2 * 16 + r) * 64 + lane] + part[(3 * 16 + r) * 64 + lane]) + pin[g] + c_bias[g];
    }
    float gi, gf, go, gg, cv, hv;
    if (CELL == 0) {
      gi = sigmoidf_dev(sg[0]); gf = sigmoidf_dev(sg[1]); go = sigmoidf_dev(sg[2]); gg = tanhf_dev(sg[3]);
      cv = gf * c_state + gi * gg;
      hv = go * tanhf_dev(cv);
      c_state = cv;
    } else if (CELL == 1) {  // sg: r, z pre-activations; W_n x + b_n (from P: this group has no weights here); R_n h
      gi = sigmoidf_dev(sg[0]); gf = sigmoidf_dev(sg[1]);
      go = tanhf_dev(sg[2] + gi * sg[3]);
      gg = sg[3];
      hv = (1.f - gf) * go + gf * c_state;
      cv = 0.f;
      c_state = hv;
    } else {
      gi = gf = go = gg = cv = 0.f;
      hv = CELL == 3 ? tanhf_dev(sg[0]) : fmaxf(sg[0], 0.f);
    }
    xs[((uj & 1) * 32 + n) * 4 + (uj >> 1)] = valid ? hv : 0.f;
    __syncthreads();
    if (threadIdx.x < 64)
      xstore4(slot(t + 1) + (size_t)s * 256 + 4 * threadIdx.x, *reinterpret_cast<const floatx4*>(xs + 4 * threadIdx.x));
    tr.mark(t, 5);
    signal(flags + ((size_t)16 * (t + 1) + (s & 15)) * kFlagStride, a.full_fences);  // publish h_t (the barrier also protects `part` and `xs`)
    tr.mark(t, 6);
    // reserve and outputs: staged through LDS so that every store instruction writes 16-byte runs
    ro[(0 * 32 + n) * 8 + uj] = gi;
    ro[(1 * 32 + n) * 8 + uj] = gf;
    ro[(2 * 32 + n) * 8 + uj] = go;
    ro[(3 * 32 + n) * 8 + uj] = gg;
    ro[(4 * 32 + n) * 8 + uj] = cv;
    ro[(5 * 32 + n) * 8 + uj] = hv;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = threadIdx.x + 256 * i;  // (array 0..5, batch row, half of the 8 units)
      const int arr = idx >> 6, l2 = (idx >> 1) & 31, hf = idx & 1;
      const int b2 = b0 + l2;
      if (idx < 384 && b2 < B) {
        const floatx4 v = *reinterpret_cast<const floatx4*>(ro + (arr * 32 + l2) * 8 + 4 * hf);
        const size_t e = ((size_t)t * B + b2) * H + u0 + 4 * hf;
        if (arr < 4) {
          if (CELL <= 1) *reinterpret_cast<floatx4*>(res_gates + ((size_t)t * B + b2) * 4 * H + (size_t)arr * H + u0 + 4 * hf) = v;
        } else if (arr == 4) {
          if (CELL == 0) {
            *reinterpret_cast<floatx4*>(res_c + e) = v;
            if (t == T - 1 && a.cT) *reinterpret_cast<floatx4*>(a.cT + (size_t)b2 * H + u0 + 4 * hf) = v;
          }
        } else {
          *reinterpret_cast<floatx4*>(res_h + e) = v;
          if (a.y) *reinterpret_cast<floatx4*>(a.y + e) = v;
          if (t == T - 1 && a.hT) *reinterpret_cast<floatx4*>(a.hT + (size_t)b2 * H + u0 + 4 * hf) = v;
        }
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) pin[g] = pnx[g];
  }
}

// h0 [B][H] of one layer (zeros if null) -> exchange slot 0 of every slice in the layout of pers_fwdL_kernel, all 32 batch columns.
__global__ void pack_stateL_kernel(const float* __restrict__ h0, float* __restrict__ hx, int T, int B, int H, int b0,
                                   int nsl) {
  const long cnt = (long)nsl * 32 * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < cnt; e += (long)gridDim.x * blockDim.x) {
    const int k = (int)(e % H), lb = (int)((e / H) % 32), sl = (int)(e / ((long)H * 32));
    const int bb = b0 + 32 * sl + lb;
    const int wv = k / (H / 4), kr = k % (H / 4), k8 = kr >> 3, m = (kr >> 1) & 3, kk = kr & 1;
    hx[(size_t)sl * (T + 1) * H * 32 + ((size_t)wv * (H / 32) + k8) * 256 + (kk * 32 + lb) * 4 + m] =
        (h0 && bb < B) ? h0[(size_t)bb * H + k] : 0.f;
  }
}

// ------------------------------------------------------------------ one layer, large hidden size, backward
// dh_{t-1} = R^T dA_t has K = 4H, four times the forward product: slicing it by output units would make
// every workgroup read all of dA_t (1 MB per step at H = 2048).  The [4H x H] matrix is therefore cut in
// two dimensions, NBK x NBK tiles of [4*UB gate rows x UB output units] (UB = 128: tiles of 256 KB, half
// in VGPRs, half in LDS; 256 tiles at H = 2048, 64 at H = 1024).  Workgroup (i, j) multiplies the gate
// gradients of unit block i into a partial sum for the output units of block j; the NBK partial sums of a
// block are then added -- always in the order of i, so the result does not depend on arrival order -- by
// the same NBK workgroups, each taking UB/NBK of the block's 128 units (8 at H = 2048, 16 at H = 1024: one
// or two cells per thread), which also run the point-wise stage of the next step for those units and
// publish their gate gradients to the NBK workgroups (j, .) that consume unit block j.
// Per step: 64 KB of dA read and 16 KB of partial sums written per workgroup, two synchronisation
// hops of NBK arrivals each.  The gradient for the layer below is a batched GEMM after the launch.
// The batch runs in slices of 32 rows, each with its own workgroups, exchange buffers and counters; at
// H = 1024 four slices fit side by side on 256 CUs.
// Exchange layouts: dA_t of a unit block: [k8][(kk*32 + n)*4 + m] for k = 8*k8 + 2*m + kk, batch row n,
// where k8 = 4*(unit/8 within the block) + gate and k%8 = unit%8; partial sums: [unit in block][32].
struct PersBwdLArgs {
  const float* R;      // [4H][H] of this layer
  const float* res;    // reserve of this layer
  const float* c0;     // [B][H] or null
  const float* dout;   // [T][B][H]: dy (top layer) or the gradient handed down by the layer above
  const float* dhT;    // [B][H] or null
  const float* dcT;    // [B][H] or null
  float* dA;           // [T][B][4H] gate gradients (standard layout)
  float* X;            // [nsl][T][NBK][4*UB*32] exchange
  float* Pp;           // [nsl][T][NBK][NBK][UB*32] partial sums
  float* dh0;          // [B][H] or null
  float* dc0;          // [B][H] or null
  float* db;           // [4H] or null (must be null when the batch has more than one slice: column sums follow instead)
  int* flagsA;         // [nsl][T][NBK] counters: gate gradients of (step, unit block) published
  int* flagsP;         // [nsl][T][NBK] counters: partial sums of (step, output block) published
  int* watchdog;
  int T, B;
  int b0;              // first batch row of this launch (a multiple of 32)
  int nsl;             // batch slices side by side in this launch (grid = nsl * NBK * NBK)
  int spin_limit;
  int full_fences;
  long long* trace;
  int trace_block;
};

// CELL as in pers_bwd32_kernel: the four K groups of a unit octet are the gradients with respect to the four gate
// pre-activations (LSTM); to the r and z pre-activations, W_n x + b_n and R_n h (GRU: the third has no weights here,
// dh_{t-1} also receives dh_t o z_t); to the one pre-activation (single gate).  For the other cells `res` is that
// cell's reserve, c0 carries h0, dcT / dc0 are unused, R and db have 3H or H rows.
template <int HH, int CELL>
__global__ __launch_bounds__(256) void pers_bwdL_kernel(const PersBwdLArgs a) {
  constexpr int H = HH, G = 4 * H, UB = 128, NBK = H / UB;
  constexpr int NG = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1);  // gate blocks of R and db
  constexpr int UF = UB / NBK;               // units a workgroup finalises: 8 or 16
  constexpr int CPT = UF / 8;                // cells per thread in the point-wise stage
  constexpr int NG8 = 4 * UB / 8;            // 8-k groups of the tile's K = 4*UB
  constexpr int KP = 4 * UB / 2;             // k-pairs; every wave runs all of them for its 32 output units
  constexpr int RP = UF == 16 ? 136 : 128;   // k-pairs with weights in registers (more where the staging arrays are larger)
  constexpr int LP = KP - RP;                // k-pairs with weights in LDS
  constexpr int DEPTH = 16;
  static_assert(NBK % kFlagSub == 0, "arrivals must spread evenly over the counter lines");
  static_assert(UF == 8 || UF == 16, "one or two cells per thread");
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* const stage = smem;              // [UB][32] partial sums of this step; also the bias-gradient reduction
  float* const xsA = smem + 4096;         // [UF/8 octets][4 gates][256] gate gradients of the finalised units, exchange order
  float* const ro = xsA + 1024 * CPT;     // [4 gates][32 batch rows][UF units] the same in standard order
  float* const wl = ro + 128 * UF;        // [4 waves][LP][64 lanes]; 152 KB in all

  const int sl = blockIdx.x / (NBK * NBK), bid = blockIdx.x % (NBK * NBK);
  const int i = bid / NBK, j = bid % NBK;
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kk = lane >> 5, n = lane & 31;
  const size_t TB = (size_t)T * B;
  const int rot = (4 * j + 16 * __builtin_amdgcn_readfirstlane(wave)) & (NG8 - 1);

  // ---- weights: A operand row n = output unit UB*j + 32*wave + n; entry p covers
  //      k = 8*k8 + 2*(p%4) + kk with k8 = (p/4 + rot) mod NG8: gate k8%4, unit UB*i + 8*(k8/4) + k%8
  float wreg[RP];
  {
    const float* col = a.R + UB * j + 32 * wave + n;
#pragma unroll
    for (int p = 0; p < KP; ++p) {
      const int k8 = ((p >> 2) + rot) & (NG8 - 1), m = p & 3;
      const int unit = UB * i + 8 * (k8 >> 2) + 2 * m + kk;
      const int grp = k8 & 3;
      const int gate = CELL >= 2 ? 0 : ((CELL == 1 && grp == 3) ? 2 : grp);
      const bool live = CELL == 0 || (CELL == 1 ? grp != 2 : grp == 0);
      const float v = live ? col[((size_t)gate * H + unit) * H] : 0.f;
      if (p < RP)
        wreg[p < RP ? p : 0] = v;
      else
        wl[((size_t)wave * LP + (p - RP)) * 64 + lane] = v;
    }
  }

  // ---- the cells this thread finalises: units UB*j + UF*i + 8*c + 2*wave + kk (c < CPT), batch row b0 + n
  const int j8 = 2 * wave + kk;
  const int bb = a.b0 + 32 * sl + n;
  const bool valid = bb < B;
  int cu[CPT];
  float dc[CPT], dh_rec[CPT], dbsum[CPT][4];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    cu[c] = UB * j + UF * i + 8 * c + j8;
    dc[c] = (CELL == 0 && valid && a.dcT) ? a.dcT[(size_t)bb * H + cu[c]] : 0.f;  // GRU: the direct term dh_t o z_t
    dh_rec[c] = (valid && a.dhT) ? a.dhT[(size_t)bb * H + cu[c]] : 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g) dbsum[c][g] = 0.f;
  }
  const float* const res_gates = CELL == 0 ? a.res : a.res + TB * H;  // the four saved arrays [T][B][4H] (LSTM, GRU)
  const float* const res_c = CELL == 0 ? a.res + TB * 4 * H : a.res;   // c (LSTM) or h: the state array the step reads
  float* const Xs = a.X + (size_t)sl * T * NBK * (4 * UB * 32);
  float* const Ps = a.Pp + (size_t)sl * T * NBK * NBK * (UB * 32);
  int* const fA = a.flagsA + (size_t)sl * T * NBK * kFlagInts;
  int* const fP = a.flagsP + (size_t)sl * T * NBK * kFlagInts;
  auto slotX = [&](int t, int blk) { return Xs + ((size_t)t * NBK + blk) * (4 * UB * 32); };
  auto slotP = [&](int t, int jb, int ib) { return Ps + (((size_t)t * NBK + jb) * NBK + ib) * (UB * 32); };
  auto flagA = [&](int t, int blk) { return fA + ((size_t)t * NBK + blk) * kFlagInts; };
  auto flagP = [&](int t, int blk) { return fP + ((size_t)t * NBK + blk) * kFlagInts; };

  // reserve values and upstream gradient of the step the point-wise stage handles next: fetched ahead,
  // under the MFMAs, so that no miss to HBM sits in front of a counter poll (loads return in order)
  float fg[CPT][4], fct[CPT], fcp[CPT], fdo[CPT];
  auto fetch_step = [&](int t) {
    if (valid) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const size_t e = ((size_t)t * B + bb) * H + cu[c];
        const size_t g0 = ((size_t)t * B + bb) * G + cu[c];
        if (CELL <= 1) {
#pragma unroll
          for (int g = 0; g < 4; ++g) fg[c][g] = res_gates[g0 + (size_t)g * H];
        }
        if (CELL != 1) fct[c] = res_c[e];  // c_t (LSTM), h_t (single gate)
        if (CELL <= 1) fcp[c] = t > 0 ? res_c[e - (size_t)B * H] : (a.c0 ? a.c0[(size_t)bb * H + cu[c]] : 0.f);
        fdo[c] = a.dout[e];
      }
    }
  };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2

  // point-wise stage of step t for the UF units of this workgroup, and publication of their gate gradients
  auto pointwise_publish = [&](int t) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      float dA4[4] = {0.f, 0.f, 0.f, 0.f};
      if (valid) {
        const float dh = fdo[c] + dh_rec[c];
        if (CELL == 0) {
          const float tc = tanhf_dev(fct[c]);
          const float dcv = dc[c] + dh * fg[c][2] * (1.f - tc * tc);
          dA4[0] = dcv * fg[c][3] * fg[c][0] * (1.f - fg[c][0]);
          dA4[1] = dcv * fcp[c] * fg[c][1] * (1.f - fg[c][1]);
          dA4[2] = dh * tc * fg[c][2] * (1.f - fg[c][2]);
          dA4[3] = dcv * fg[c][0] * (1.f - fg[c][3] * fg[c][3]);
          dc[c] = dcv * fg[c][1];
        } else if (CELL == 1) {  // fg: r, z, n, R_n h; fcp: h_{t-1}
          const float dn = dh * (1.f - fg[c][1]) * (1.f - fg[c][2] * fg[c][2]);
          dA4[0] = dn * fg[c][3] * fg[c][0] * (1.f - fg[c][0]);
          dA4[1] = dh * (fcp[c] - fg[c][2]) * fg[c][1] * (1.f - fg[c][1]);
          dA4[2] = dn;
          dA4[3] = dn * fg[c][0];
          dc[c] = dh * fg[c][1];
        } else {  // fct: h_t
          dA4[0] = CELL == 3 ? dh * (1.f - fct[c] * fct[c]) : (fct[c] > 0.f ? dh : 0.f);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) dbsum[c][g] += dA4[g];
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        xsA[(c * 4 + g) * 256 + (kk * 32 + n) * 4 + wave] = dA4[g];  // k%8 = j8 = 2*wave + kk: m = wave
        ro[(g * 32 + n) * UF + 8 * c + j8] = dA4[g];
      }
    }
    __syncthreads();
    // the unit octets of this workgroup are k8 blocks 4*(UF/8*i + c) + gate of the block's slot: contiguous
#pragma unroll
    for (int c = 0; c < CPT; ++c)
      xstore4(slotX(t, j) + (size_t)(4 * (CPT * i + c)) * 256 + 4 * threadIdx.x,
              *reinterpret_cast<const floatx4*>(xsA + c * 1024 + 4 * threadIdx.x));
    signal(flagA(t, j) + (i & (kFlagSub - 1)) * kFlagStride, a.full_fences);
    // standard layout for the weight-gradient products: (gate, batch row, four of the UF units) per store
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
      const int idx = threadIdx.x + 256 * q;
      const int g = idx / (8 * UF), l2 = (idx / (UF / 4)) & 31, hf = idx % (UF / 4);
      const int b2 = a.b0 + 32 * sl + l2;
      if (b2 < B)
        *reinterpret_cast<floatx4*>(a.dA + ((size_t)t * B + b2) * G + (size_t)g * H + UB * j + UF * i + 4 * hf) =
            *reinterpret_cast<const floatx4*>(ro + (g * 32 + l2) * UF + 4 * hf);
    }
  };

  __syncthreads();  // LDS weights are in place
  fetch_step(T - 1);
  pointwise_publish(T - 1);

  int rv = rot;
  for (int t = T - 1; t >= 0; --t) {
    tr.mark(t, 0);
    hide(rv);
    w.wait(flagA(t, i), NBK);
    tr.mark(t, 1);
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    {
      const float* src = slotX(t, i) + lane * 4;
      floatx4 bv[NG8];
      float al[NG8][4];
      auto ldb = [&](int g) { bv[g] = *reinterpret_cast<const floatx4*>(src + (size_t)((g + rv) & (NG8 - 1)) * 256); };
      auto ldw = [&](int g) {
        if (g * 4 >= RP) {
#pragma unroll
          for (int m = 0; m < 4; ++m) al[g][m] = wl[((size_t)wave * LP + (g * 4 + m - RP)) * 64 + lane];
        }
      };
#pragma unroll
      for (int g = 0; g < DEPTH; ++g) ldb(g);
      ldw(0);
      ldw(1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < NG8; ++g) {
        if (g + DEPTH < NG8) ldb(g + DEPTH);
        if (g + 2 < NG8) ldw(g + 2);
        if (g == NG8 - DEPTH && t > 0) fetch_step(t - 1);  // behind the last exchange load of this step
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const int pr = g * 4 + m;
          const float av = (pr < RP) ? wreg[pr < RP ? pr : 0] : al[g][m];
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[g][m], acc, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // partial sums -> LDS (rows of the D layout) -> one coalesced, write-through 16 KB block
#pragma unroll
    for (int r = 0; r < 16; ++r) stage[(32 * wave + 8 * (r >> 2) + 4 * kk + (r & 3)) * 32 + n] = acc[r];
    tr.mark(t, 2);
    __syncthreads();
    {
      float* const dst = slotP(t, j, i);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int idx = threadIdx.x + 256 * q;
        xstore4(dst + 4 * idx, *reinterpret_cast<const floatx4*>(stage + 4 * idx));
      }
    }
    signal(flagP(t, j) + (i & (kFlagSub - 1)) * kFlagStride, a.full_fences);
    tr.mark(t, 3);
    w.wait(flagP(t, j), NBK);
    tr.mark(t, 4);
#pragma unroll
    for (int c = 0; c < CPT; ++c) {  // dh_rec of this thread's cells: the NBK partial sums in fixed order
      float pv[NBK];
#pragma unroll
      for (int ib = 0; ib < NBK; ++ib) pv[ib] = slotP(t, j, ib)[(UF * i + 8 * c + j8) * 32 + n];
      float sum = 0.f;
#pragma unroll
      for (int ib = 0; ib < NBK; ++ib) sum += pv[ib];
      dh_rec[c] = CELL == 1 ? sum + dc[c] : sum;
    }
    tr.mark(t, 5);
    if (t > 0) pointwise_publish(t - 1);
    tr.mark(t, 6);
  }
  if (valid) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      if (a.dh0) a.dh0[(size_t)bb * H + cu[c]] = dh_rec[c];
      if (CELL == 0 && a.dc0) a.dc0[(size_t)bb * H + cu[c]] = dc[c];
    }
  }
  if (a.db) {  // single slice: this workgroup owns its units for every batch row, plain sums, no atomics
    __syncthreads();
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
      for (int g = 0; g < 4; ++g) stage[(g * UF + 8 * c + j8) * 32 + n] = dbsum[c][g];
    __syncthreads();
    if (threadIdx.x < NG * UF) {
      float sum = 0.f;
#pragma unroll
      for (int q = 0; q < 32; ++q) sum += stage[threadIdx.x * 32 + ((q + threadIdx.x) & 31)];
      a.db[(size_t)(threadIdx.x / UF) * H + UB * j + UF * i + (threadIdx.x % UF)] = sum;
    }
  }
}

// ------------------------------------------------------------------ host state
struct DeviceInfo {
  bool ok = false;
  int cus = 0;
  int coop = 0;
};
std::mutex g_mu;
DeviceInfo g_dev[64];
bool g_dev_init[64];
int* g_watch_host = nullptr;
int* g_watch_dev = nullptr;

bool device_info(DeviceInfo& out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    (void)hipGetLastError();
    return false;
  }
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_dev_init[dev]) {
    DeviceInfo di;
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess) di.cus = v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeCooperativeLaunch, dev) == hipSuccess) di.coop = v;
    (void)hipGetLastError();
    di.ok = di.cus > 0;
    g_dev[dev] = di;
    g_dev_init[dev] = true;
  }
  out = g_dev[dev];
  return out.ok;
}

bool ensure_watchdog() {
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_watch_host) return true;
  void* p = nullptr;
  if (hipHostMalloc(&p, 64, hipHostMallocMapped) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  g_watch_host = reinterpret_cast<int*>(p);
  *g_watch_host = 0;
  void* d = nullptr;
  if (hipHostGetDevicePointer(&d, p, 0) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipHostFree(p);
    g_watch_host = nullptr;
    return false;
  }
  g_watch_dev = reinterpret_cast<int*>(d);
  return true;
}

int spin_limit() { return knobs().spin_limit; }

long long* g_trace_buf = nullptr;
size_t g_trace_bytes = 0;
int g_trace_block = 0;

int full_fences() { return knobs().full_fences ? 1 : 0; }

// All workgroups of a persistent kernel must be resident at once (they wait on each other).  The grid never exceeds
// the number of CUs and every workgroup fits a CU on its own, so an ordinary launch is resident as soon as the CUs it
// needs are free, and every other kernel on the device ends without waiting for anything.  What must not happen is
// two persistent kernels each holding part of the CUs and waiting for the rest: the persistent launches of this
// process are therefore chained, each waits (on the GPU, through an event) for the one before it, whatever their
// streams.  This costs nothing on one stream.  A cooperative launch gives the same guarantee device-wide, also
// against other processes, but measured 0.05-0.15 ms slower per launch on this stack and slows later multi-stream
// work of the process down: LSTM_COOP_LAUNCH=1 selects it.  LSTM_PLAIN_LAUNCH=1 launches without the chain (two
// persistent kernels may then share the CUs when both fit; diagnostics and tests).  A wait that never ends is, in
// every mode, turned into LSTM_INTERNAL by the watchdog.
std::mutex g_launch_mu;
hipEvent_t g_last_launch[16] = {};  // per device: completion of the most recent persistent launch
bool g_last_launch_recorded[16] = {};

// Side stream (default priority) and two events for work that overlaps a persistent launch which leaves CUs idle.
hipStream_t g_side_stream = nullptr;
hipEvent_t g_side_ev[2] = {};
std::mutex g_side_mu;  // held by the call that is using them
bool ensure_side_stream() {
  std::lock_guard<std::mutex> lk(g_launch_mu);
  if (g_side_stream) return true;
  if (hipStreamCreateWithFlags(&g_side_stream, hipStreamNonBlocking) != hipSuccess) {
    g_side_stream = nullptr;
    (void)hipGetLastError();
    return false;
  }
  for (hipEvent_t& ev : g_side_ev)
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      return false;
    }
  return true;
}

// Raises a kernel's dynamic LDS limit once per process (`done` is the caller's flag for that kernel); callers on
// several host threads are serialised.
hipError_t allow_dynamic_lds(const void* fn, size_t smem, bool& done) {
  std::lock_guard<std::mutex> lk(g_launch_mu);
  if (done) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e == hipSuccess) done = true;
  return e;
}

hipError_t launch_resident(const void* fn, int grid, void** params, unsigned smem, hipStream_t s) {
  if (knobs().coop_launch) return hipLaunchCooperativeKernel(fn, dim3(grid), dim3(256), params, smem, s);
  int dev = 0;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (knobs().plain_launch || hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16 ||
      hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
    (void)hipGetLastError();
    return hipLaunchKernel(fn, dim3(grid), dim3(256), params, smem, s);  // (a stream under capture is ordered by its graph)
  }
  std::lock_guard<std::mutex> lk(g_launch_mu);
  hipError_t st = hipSuccess;
  if (!g_last_launch[dev]) {
    st = hipEventCreateWithFlags(&g_last_launch[dev], hipEventDisableTiming);
    g_last_launch_recorded[dev] = false;
  } else if (g_last_launch_recorded[dev]) {
    st = hipStreamWaitEvent(s, g_last_launch[dev], 0);
  }
  if (st != hipSuccess) return st;
  st = hipLaunchKernel(fn, dim3(grid), dim3(256), params, smem, s);
  if (st != hipSuccess) return st;
  g_last_launch_recorded[dev] = true;
  return hipEventRecord(g_last_launch[dev], s);
}

// Batch tiles per chain and number of chains.  One chain is the default: on MI355X two chains
// measured slower at B = 64 (the step is bound by MFMA issue forward and by L2->CU bandwidth
// backward, and half-width 8-byte exchange loads are less efficient); LSTM_CHAINS=2 selects two.
struct BatchPlan {
  int NT, NC;
};
BatchPlan batch_plan(int B) {
  const bool two = knobs().two_chains;
  if (B <= 16) return {1, 1};
  if (B <= 32) return two ? BatchPlan{1, 2} : BatchPlan{2, 1};
  return two ? BatchPlan{2, 2} : BatchPlan{4, 1};
}

template <int KG>
hipError_t launch_fwd(BatchPlan bp, int grid, const PersFwdArgs& a, hipStream_t s) {
  void* params[] = {const_cast<PersFwdArgs*>(&a)};
  const void* fn = nullptr;
  if (bp.NT == 1 && bp.NC == 1) fn = (const void*)pers_fwd_kernel<KG, 1, 1>;
  if (bp.NT == 1 && bp.NC == 2) fn = (const void*)pers_fwd_kernel<KG, 1, 2>;
  if (bp.NT == 2 && bp.NC == 2) fn = (const void*)pers_fwd_kernel<KG, 2, 2>;
  if (bp.NT == 2 && bp.NC == 1) fn = (const void*)pers_fwd_kernel<KG, 2, 1>;
  if (bp.NT == 4 && bp.NC == 1) fn = (const void*)pers_fwd_kernel<KG, 4, 1>;
  if (!fn) return hipErrorInvalidValue;
  return launch_resident(fn, grid, params, 0, s);
}

template <int KGB>
hipError_t launch_bwd(BatchPlan bp, int grid, const PersBwdArgs& a, hipStream_t s) {
  void* params[] = {const_cast<PersBwdArgs*>(&a)};
  const void* fn = nullptr;
  if (bp.NT == 1 && bp.NC == 1) fn = (const void*)pers_bwd_kernel<KGB, 1, 1>;
  if (bp.NT == 1 && bp.NC == 2) fn = (const void*)pers_bwd_kernel<KGB, 1, 2>;
  if (bp.NT == 2 && bp.NC == 2) fn = (const void*)pers_bwd_kernel<KGB, 2, 2>;
  if (bp.NT == 2 && bp.NC == 1) fn = (const void*)pers_bwd_kernel<KGB, 2, 1>;
  if (bp.NT == 4 && bp.NC == 1) fn = (const void*)pers_bwd_kernel<KGB, 4, 1>;
  if (!fn) return hipErrorInvalidValue;
  return launch_resident(fn, grid, params, 0, s);
}

// The wide-batch forward kernel (32x32x2 MFMA, two batch tiles of 32).
// Height of the batch slices (16 or 32 rows) that run side by side on the narrow kernels, or 0 where the batch is
// taken whole (B <= 16, or no room) or by the wide kernels.  While all slices fit the chip in one launch the narrow
// kernels are the faster ones: a step's matrix work per workgroup shrinks with the slice and more CUs share it (one or
// two layers at H = 512, up to four at H = 256; L = 1, H = 512, B = 64, T = 100: forward recurrence 0.40 ms on four
// slices of 16 rows, 0.53 on two of 32, 0.74 on the wide kernel; backward 0.65 against 1.14).  `env` names the
// setting that pins the choice (LSTM_FWD_NARROW / LSTM_BWD_NARROW): 1 = one slice on the narrow kernel (B <= 64), 0 = never slices.
int narrow_slice_rows(const Dims& d, int cell, int pinned) {
  if (cell != 0) return 0;  // the narrow kernels are LSTM kernels
  if (pinned >= 0 || knobs().two_chains) return 0;
  DeviceInfo di;
  if (!device_info(di)) return 0;
  for (int rows = 16; rows <= 32; rows *= 2) {
    const int n = (d.B + rows - 1) / rows;
    if (d.B > rows && (long)d.L * (d.H / 8) * n <= di.cus && n <= 16 / d.L) return rows;  // 16 (slice, layer) counter blocks
  }
  return 0;
}

bool fwd_wide(const Dims& d) {
  if (d.B > 64) return true;  // batches above 64 run as slices of 64 rows, one launch each
  if (knobs().fwd_narrow == 1) return false;
  return d.B > 32;
}

template <int CELL>
hipError_t launch_fwd32(int H, int grid, const PersFwdArgs& a, hipStream_t s) {
  void* params[] = {const_cast<PersFwdArgs*>(&a)};
  const void* fn = H == 512 ? (const void*)pers_fwd32_kernel<512, CELL>
                            : (H == 256 ? (const void*)pers_fwd32_kernel<256, CELL> : (const void*)pers_fwd32_kernel<128, CELL>);
  return launch_resident(fn, grid, params, 0, s);
}

// The wide-batch backward kernel: two batch halves, 16 hidden units per workgroup.
bool bwd_wide(const Dims& d) {
  if (d.B > 64) return true;
  if (knobs().bwd_narrow == 1) return false;
  return d.B > 32;
}

template <int HH, int CELL = 0>
hipError_t launch_bwd32(const PersBwdArgs& a, int nbh, hipStream_t s) {
  constexpr int KPW = HH / 2, LP = KPW > 128 ? KPW - 128 : 0;
  const size_t smem = (6144 + (size_t)4 * LP * 64) * sizeof(float);
  const void* fn = (const void*)pers_bwd32_kernel<HH, CELL>;
  static bool attr_set = false;
  if (hipError_t e = allow_dynamic_lds(fn, smem, attr_set); e != hipSuccess) return e;
  void* params[] = {const_cast<PersBwdArgs*>(&a), &nbh};
  const int grid = a.L * (HH / 16) * nbh;
  return launch_resident(fn, grid, params, (unsigned)smem, s);
}

}  // namespace

int device_cu_count() {
  DeviceInfo di;
  return device_info(di) ? di.cus : 0;
}

void set_trace(void* buf, size_t bytes, int block) {
  g_trace_buf = reinterpret_cast<long long*>(buf);
  g_trace_bytes = buf ? bytes : 0;
  g_trace_block = block;
}

// True once after a persistent kernel's bounded wait has expired: the word is cleared by the report, so the
// call after the one that reports LSTM_INTERNAL runs normally again.
bool take_watchdog() {
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_watch_host || !*g_watch_host) return false;
  *g_watch_host = 0;
  return true;
}

// Everything the persistent path creates lazily, created now for the current device: the host-visible watchdog
// word and the event that chains the persistent launches.  After it no persistent forward call creates anything.
hipError_t setup_persistent() {
  DeviceInfo di;
  (void)device_info(di);
  if (!ensure_watchdog()) return hipErrorOutOfMemory;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 16) return hipSuccess;  // launches on such a device are not chained
  std::lock_guard<std::mutex> lk(g_launch_mu);
  if (!g_last_launch[dev]) {
    e = hipEventCreateWithFlags(&g_last_launch[dev], hipEventDisableTiming);
    if (e != hipSuccess) return e;
    g_last_launch_recorded[dev] = false;
  }
  return hipSuccess;
}

void release_persistent() {
  {
    std::lock_guard<std::mutex> lk(g_launch_mu);
    for (hipEvent_t& ev : g_last_launch)
      if (ev) {
        (void)hipEventDestroy(ev);
        ev = nullptr;
      }
    for (hipEvent_t& ev : g_side_ev)
      if (ev) {
        (void)hipEventDestroy(ev);
        ev = nullptr;
      }
    if (g_side_stream) {
      (void)hipStreamDestroy(g_side_stream);
      g_side_stream = nullptr;
    }
  }
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_watch_host) {
    (void)hipHostFree(g_watch_host);
    g_watch_host = nullptr;
    g_watch_dev = nullptr;
  }
}

// Large hidden sizes: one layer per launch, the layer's recurrent matrix spread over all CUs.
// Largest batch the one-layer kernels take at H = 1024 (slices of 32 rows: two side by side forward, four backward):
// measured faster than the step kernels up to here (108 against 89 TFLOP/s at B = 512).
constexpr int kLargeMaxBatch1024 = 512;
// At H = 2048 one slice of 32 rows fills the chip: larger batches run slice after slice, at a constant 5.8 ms per slice
// and 100 steps, which the step kernels (streaming R once per step for the whole batch) undercut from about 200 rows on.
constexpr int kLargeMaxBatch2048 = 192;

bool persistent_large(const Dims& d, bool backward) {
  if (knobs().no_large_persistent) return false;
  if (!(d.H == 1024 || d.H == 2048)) return false;
  if (d.B > (d.H == 1024 ? kLargeMaxBatch1024 : kLargeMaxBatch2048)) return false;
  DeviceInfo di;
  if (!device_info(di) || !di.coop) return false;
  return (backward ? (d.H / 128) * (d.H / 128) : d.H / 8) <= di.cus;
}

bool persistent_supported(const Dims& d, bool backward) {
  if (persistent_large(d, backward)) return true;
  if (!(d.H == 128 || d.H == 256 || d.H == 512)) return false;
  if (d.B > 2048) return false;  // slices of 64 rows; beyond 2048 rows the GEMM rungs are as fast or faster
  DeviceInfo di;
  if (!device_info(di) || !di.coop) return false;
  return d.H / 8 <= di.cus;  // deeper stacks than the chip holds run as groups of layers (run_forward_persistent)
}

namespace {

template <int HH, int CELL>
hipError_t launch_fwdL(const PersFwdLArgs& a, hipStream_t s) {
  constexpr int KPW = HH / 8, LP = KPW > 128 ? KPW - 128 : 0;
  const size_t smem = (6144 + (size_t)4 * LP * 64) * sizeof(float);
  const void* fn = (const void*)pers_fwdL_kernel<HH, CELL>;
  static bool attr_set = false;
  if (hipError_t e = allow_dynamic_lds(fn, smem, attr_set); e != hipSuccess) return e;
  void* params[] = {const_cast<PersFwdLArgs*>(&a)};
  return launch_resident(fn, a.nsl * (HH / 8), params, (unsigned)smem, s);
}

// Forward pass of the large-H shapes: per layer the batched input projection, then one persistent launch.
// Dispatch over (hidden size, cell) of the one-layer kernels.
hipError_t launch_fwdL_any(int H, int cell, const PersFwdLArgs& k, hipStream_t s) {
  if (H == 2048) {
    return cell == 0 ? launch_fwdL<2048, 0>(k, s) : (cell == 1 ? launch_fwdL<2048, 1>(k, s)
                     : (cell == 2 ? launch_fwdL<2048, 2>(k, s) : launch_fwdL<2048, 3>(k, s)));
  }
  return cell == 0 ? launch_fwdL<1024, 0>(k, s) : (cell == 1 ? launch_fwdL<1024, 1>(k, s)
                   : (cell == 2 ? launch_fwdL<1024, 2>(k, s) : launch_fwdL<1024, 3>(k, s)));
}

// Reserve of one layer in floats per (step, row, unit), and where its hidden states start, for each cell.
inline size_t res_width(int cell) { return cell == 0 ? 6 : (cell == 1 ? 5 : 1); }
inline size_t res_h_offset(int cell, size_t TB, int H) { return cell == 0 ? 5 * TB * H : 0; }
inline int gates_of_cell(int cell) { return cell == 0 ? 4 : (cell == 1 ? 3 : 1); }

int run_forward_persistent_large(const FwdArgs& a, int cell) {
  const Dims& d = a.d;
  const size_t TB = (size_t)d.T * d.B, G = (size_t)gates_of_cell(cell) * d.H, BH = (size_t)d.B * d.H;
  const size_t rstride = res_width(cell) * TB * d.H;
  hipStream_t s = a.stream;
  float* hx = reinterpret_cast<float*>(a.ws + a.w.xchg);
  int* flags = reinterpret_cast<int*>(a.ws + a.w.flags);
  float* P = reinterpret_cast<float*>(a.ws + a.w.P);
  // slices of 32 batch rows side by side while the CUs last (two at H = 1024), the rest in further launches
  DeviceInfo di;
  (void)device_info(di);
  const int slices = (d.B + 31) / 32;
  int cap = di.cus / (d.H / 8);
  if (cap < 1) cap = 1;
  if (cap > 4) cap = 4;
  for (int l = 0; l < d.L; ++l) {
    const int Il = in_dim(d, l);
    const float* in = l == 0 ? a.x : a.reserve + (size_t)(l - 1) * rstride + res_h_offset(cell, TB, d.H);
    const float* Wl = a.W + (l == 0 ? 0 : G * d.I + (size_t)(l - 1) * G * d.H);
    {
      ProfScope ps(LSTM_PHASE_FWD_INPUT_GEMM, s);
      GemmProblem p{in, Wl, P, (int)TB, (int)G, Il, Il, 1, 1, Il, (long)G, 0};
      CK(launch_gemm_group(&p, 1, s), "input projection GEMM");
    }
   for (int s0 = 0; s0 < slices; s0 += cap) {
    const int nsl = slices - s0 < cap ? slices - s0 : cap;
    {
      ProfScope ps(LSTM_PHASE_FWD_PACK, s);
      CK(launch_fill_zero(flags, (size_t)nsl * (d.T + 1) * 16 * kFlagStride * 4, s), "zero step counters");
      hipLaunchKernelGGL(pack_stateL_kernel, dim3((unsigned)((32L * nsl * d.H + 255) / 256)), dim3(256), 0, s,
                         a.h0 ? a.h0 + (size_t)l * BH : nullptr, hx, d.T, d.B, d.H, 32 * s0, nsl);
      CK(hipGetLastError(), "pack h0");
    }
    PersFwdLArgs k;
    k.b0 = 32 * s0; k.nsl = nsl;
    k.R = a.R + (size_t)l * G * d.H; k.bias = a.b + (size_t)l * G; k.P = P;
    const float* state0 = cell == 0 ? a.c0 : (cell == 1 ? a.h0 : nullptr);  // the GRU's cell update reads h_{t-1}
    k.c0 = state0 ? state0 + (size_t)l * BH : nullptr;
    k.hx = hx; k.flags = flags; k.watchdog = g_watch_dev;
    k.res = a.reserve + (size_t)l * rstride;
    k.y = l == d.L - 1 ? a.y : nullptr;
    k.hT = a.hT ? a.hT + (size_t)l * BH : nullptr;
    k.cT = a.cT ? a.cT + (size_t)l * BH : nullptr;
    k.T = d.T; k.B = d.B; k.spin_limit = spin_limit(); k.full_fences = full_fences();
    k.trace = (g_trace_bytes >= (size_t)d.T * 64) ? g_trace_buf : nullptr;
    k.trace_block = g_trace_block;
    ProfScope ps(LSTM_PHASE_FWD_RECURRENCE, s);
    prof_flops(2.0 * G * d.H * std::min(32 * nsl, d.B - 32 * s0) * d.T, "pers_fwdL_kernel");
    CK(launch_fwdL_any(d.H, cell, k, s), "persistent forward launch (large H)");
   }
  }
  return LSTM_OK;
}

template <int HH, int CELL>
hipError_t launch_bwdL(const PersBwdLArgs& a, hipStream_t s) {
  constexpr int NBK = HH / 128, UF = 128 / NBK, LP = 256 - (UF == 16 ? 136 : 128);
  const size_t smem = (4096 + 128 * (size_t)UF + 128 * (size_t)UF + (size_t)4 * LP * 64) * sizeof(float);
  const void* fn = (const void*)pers_bwdL_kernel<HH, CELL>;
  static bool attr_set = false;
  if (hipError_t e = allow_dynamic_lds(fn, smem, attr_set); e != hipSuccess) return e;
  void* params[] = {const_cast<PersBwdLArgs*>(&a)};
  return launch_resident(fn, a.nsl * NBK * NBK, params, (unsigned)smem, s);
}

}  // namespace

int weight_gradients(const BwdArgs& a, const float* dA_all, bool grouped, bool bias_done);

namespace {

// Backward pass of the large-H shapes: per layer (top down) one persistent launch for the recurrence, then
// the batched product that hands the gradient to the layer below; weight gradients at the end.
hipError_t launch_bwdL_any(int H, int cell, const PersBwdLArgs& k, hipStream_t s) {
  if (H == 2048) {
    return cell == 0 ? launch_bwdL<2048, 0>(k, s) : (cell == 1 ? launch_bwdL<2048, 1>(k, s)
                     : (cell == 2 ? launch_bwdL<2048, 2>(k, s) : launch_bwdL<2048, 3>(k, s)));
  }
  return cell == 0 ? launch_bwdL<1024, 0>(k, s) : (cell == 1 ? launch_bwdL<1024, 1>(k, s)
                   : (cell == 2 ? launch_bwdL<1024, 2>(k, s) : launch_bwdL<1024, 3>(k, s)));
}

int run_backward_persistent_large(const BwdArgs& a, int cell, bool* bias_done, LayerGradients* lg) {
  const Dims& d = a.d;
  constexpr int UB = 128;
  const int NBK = d.H / UB;
  const size_t TB = (size_t)d.T * d.B, G = 4 * (size_t)d.H, BH = (size_t)d.B * d.H;
  const size_t GW = (size_t)gates_of_cell(cell) * d.H, rstride = res_width(cell) * TB * d.H;
  hipStream_t s = a.stream;
  // slices of 32 batch rows side by side while the CUs last (four at H = 1024), the rest in further launches
  DeviceInfo di;
  (void)device_info(di);
  const int slices = (d.B + 31) / 32;
  int cap = di.cus / (NBK * NBK);
  if (cap < 1) cap = 1;
  if (cap > 4) cap = 4;
  const int maxsl = slices < cap ? slices : cap;
  float* dA_all = reinterpret_cast<float*>(a.ws + a.w.P);
  float* dxb = reinterpret_cast<float*>(a.ws + a.w.dx);
  float* X = reinterpret_cast<float*>(a.ws + a.w.xchg);
  float* Pp = X + (size_t)maxsl * d.T * NBK * (4 * UB * 32);
  int* flagsA = reinterpret_cast<int*>(a.ws + a.w.flags);
  int* flagsP = flagsA + (size_t)maxsl * d.T * NBK * kFlagInts;
  const bool bias_in_kernel = slices == 1;
  // A launch that occupies at most half of the CUs (H = 1024 with one or two slices) leaves room for the weight
  // gradients of the layer above, which are complete once that layer's recurrence is: they run on a side stream
  // while this layer's recurrence runs (Section 2.6 wants them after the propagation of *their* layer, not of all
  // layers).  The side stream starts them behind the counter reset that precedes the persistent launch, so that the
  // launch gets its CUs first and the products fill the rest.  LSTM_NO_WGRAD_OVERLAP=1 keeps one stream.
  bool overlap = (cell == 0 || lg) && d.L > 1 && 2 * maxsl * NBK * NBK <= di.cus && slices <= cap;
  // The side stream and its two events are process-wide: calls from several host threads take turns from the first
  // fork to the join (the enqueue only; the GPU work of different calls still overlaps as their streams allow).
  std::unique_lock<std::mutex> side_turn(g_side_mu, std::defer_lock);
  {
    hipStreamCaptureStatus cst = hipStreamCaptureStatusNone;
    if (knobs().no_wgrad_overlap || hipStreamIsCapturing(s, &cst) != hipSuccess || cst != hipStreamCaptureStatusNone ||
        !ensure_side_stream())
      overlap = false;
    (void)hipGetLastError();
  }
  if (overlap) side_turn.lock();
  int pending = -1;  // layer whose weight gradients wait for the side stream
  for (int l = d.L - 1; l >= 0; --l) {
    const int Il = in_dim(d, l);
    float* dA = dA_all + (size_t)l * TB * G;
    for (int s0 = 0; s0 < slices; s0 += cap) {
      const int nsl = slices - s0 < cap ? slices - s0 : cap;
      {
        ProfScope ps(LSTM_PHASE_BWD_PACK, s);
        CK(launch_fill_zero(flagsA, (size_t)2 * maxsl * d.T * NBK * kFlagInts * 4, s), "zero step counters");
      }
      if (overlap && pending >= 0) {
        CK(hipEventRecord(g_side_ev[0], s), "fork to the side stream");
        CK(hipStreamWaitEvent(g_side_stream, g_side_ev[0], 0), "side stream wait");
        const int st = cell == 0 ? weight_gradients_layers(a, dA_all, pending, pending + 1, g_side_stream, true, bias_in_kernel)
                                 : lg->fn(lg->ctx, pending, g_side_stream);
        if (st != LSTM_OK) return st;
        pending = -1;
      }
      PersBwdLArgs k;
      k.R = a.R + (size_t)l * GW * d.H;
      k.res = a.reserve + (size_t)l * rstride;
      const float* state0 = cell == 0 ? a.c0 : a.h0;
      k.c0 = state0 ? state0 + (size_t)l * BH : nullptr;
      k.dout = (l == d.L - 1) ? a.dy : dxb + (size_t)(l + 1) * TB * d.H;
      k.dhT = a.dhT ? a.dhT + (size_t)l * BH : nullptr;
      k.dcT = a.dcT ? a.dcT + (size_t)l * BH : nullptr;
      k.dA = dA; k.X = X; k.Pp = Pp;
      k.dh0 = a.dh0 ? a.dh0 + (size_t)l * BH : nullptr;
      k.dc0 = a.dc0 ? a.dc0 + (size_t)l * BH : nullptr;
      k.db = bias_in_kernel ? a.db + (size_t)l * GW : nullptr;
      k.flagsA = flagsA; k.flagsP = flagsP; k.watchdog = g_watch_dev;
      k.T = d.T; k.B = d.B; k.b0 = 32 * s0; k.nsl = nsl; k.spin_limit = spin_limit(); k.full_fences = full_fences();
      k.trace = (g_trace_bytes >= (size_t)d.T * 64) ? g_trace_buf : nullptr;
      k.trace_block = g_trace_block;
      ProfScope ps(LSTM_PHASE_BWD_RECURRENCE, s);
      prof_flops(2.0 * GW * d.H * std::min(32 * nsl, d.B - 32 * s0) * d.T, "pers_bwdL_kernel");
      CK(launch_bwdL_any(d.H, cell, k, s), "persistent backward launch (large H)");
    }
    float* din = l > 0 ? dxb + (size_t)l * TB * d.H : a.dx;
    if (din) {  // the GRU's gradient with respect to W_n x is its third group: the first GW columns are the ones W multiplies
      ProfScope ps(LSTM_PHASE_BWD_INPUT_GEMM, s);
      const float* Wl = a.W + (l == 0 ? 0 : GW * d.I + (size_t)(l - 1) * GW * d.H);
      GemmProblem p{dA, Wl, din, (int)TB, Il, (int)GW, (long)G, 1, Il, 1, Il, 0};
      CK(launch_gemm_group(&p, 1, s), "input-gradient GEMM");
    }
    if (overlap) pending = l;
  }
  if (bias_done) *bias_done = bias_in_kernel;
  if (!overlap) return cell != 0 ? LSTM_OK : weight_gradients(a, dA_all, true, bias_in_kernel);
  // the bottom layer's weight gradients have nothing left to hide behind; then the side stream joins
  const int st = cell == 0 ? weight_gradients_layers(a, dA_all, 0, 1, s, true, bias_in_kernel) : lg->fn(lg->ctx, 0, s);
  if (st != LSTM_OK) return st;
  if (lg) lg->used = true;
  CK(hipEventRecord(g_side_ev[1], g_side_stream), "join record");
  CK(hipStreamWaitEvent(s, g_side_ev[1], 0), "join wait");
  return LSTM_OK;
}

}  // namespace

// Wide persistent kernels for the GRU: hidden sizes and CU budget of the LSTM ones; they also take batches of 32
// rows and fewer (the rows past the batch are zeros), where the LSTM has kernels of its own.
bool gru_persistent_supported(const Dims& d) {
  if (persistent_large(d, false) && persistent_large(d, true)) return true;  // one-layer kernels, H = 1024 / 2048
  if (!(d.H == 128 || d.H == 256 || d.H == 512)) return false;
  if (d.B > 2048) return false;
  DeviceInfo di;
  if (!device_info(di) || !di.coop) return false;
  return d.H / 8 <= di.cus;  // deeper stacks than the chip holds run as groups of layers
}

// cell: 0 = LSTM; 1 = GRU, 2 / 3 = single-gate RNN with ReLU / tanh (wide kernels only: the caller has checked
// gru_persistent_supported; a.c0 / a.cT are null, W, R, b have 3H or H rows and a.reserve is that cell's reserve).
// Layers that fit on the chip together: L * H/8 workgroups, one per CU.
int layers_per_launch(const Dims& d) {
  DeviceInfo di;
  if (!device_info(di)) return 0;
  return di.cus / (d.H / 8);
}

int forward_layers(const FwdArgs& a, int cell);
int backward_layers(const BwdArgs& a, int cell, bool* bias_done, bool with_weight_gradients);

// A stack deeper than the chip holds at once runs as groups of consecutive layers, one group per launch (per batch
// slice group): the hidden states of a group's top layer, all T steps, are the input sequence of the next group --
// the same situation as x for layer 0 (Section 2.3) -- and backward the gradient a group's bottom layer produces for
// its input is the upstream gradient of the group below.
int run_forward_persistent(const FwdArgs& a, int cell) {
  const Dims& d = a.d;
  if (persistent_large(d, false)) {
    if (!ensure_watchdog()) return LSTM_HIP_ERROR;
    return run_forward_persistent_large(a, cell);
  }
  const int per = layers_per_launch(d);
  if (per <= 0) return LSTM_UNSUPPORTED;
  if (d.L <= per) return forward_layers(a, cell);
  const size_t TB = (size_t)d.T * d.B, BH = (size_t)d.B * d.H, G = (size_t)gates_of_cell(cell) * d.H;
  const size_t rstride = res_width(cell) * TB * d.H;
  for (int g0 = 0; g0 < d.L; g0 += per) {
    FwdArgs g = a;
    g.d.L = d.L - g0 < per ? d.L - g0 : per;
    const int top = g0 + g.d.L - 1;
    if (g0 > 0) {
      g.d.I = d.H;
      g.x = a.reserve + (size_t)(g0 - 1) * rstride + res_h_offset(cell, TB, d.H);
      g.W = a.W + G * d.I + (size_t)(g0 - 1) * G * d.H;
    }
    g.R = a.R + (size_t)g0 * G * d.H;
    g.b = a.b + (size_t)g0 * G;
    g.h0 = a.h0 ? a.h0 + (size_t)g0 * BH : nullptr;
    g.c0 = a.c0 ? a.c0 + (size_t)g0 * BH : nullptr;
    g.hT = a.hT ? a.hT + (size_t)g0 * BH : nullptr;
    g.cT = a.cT ? a.cT + (size_t)g0 * BH : nullptr;
    g.reserve = a.reserve + (size_t)g0 * rstride;
    // a group's top layer always leaves its hidden states where the next group reads them (an inference call writes
    // nothing else of the reserve): y of the group is that array
    if (top < d.L - 1) g.y = a.reserve + (size_t)top * rstride + res_h_offset(cell, TB, d.H);
    const int st = forward_layers(g, cell);
    if (st != LSTM_OK) return st;
  }
  return LSTM_OK;
}

int forward_layers(const FwdArgs& a, int cell) {
  const Dims& d = a.d;
  const size_t TB = (size_t)d.T * d.B, G = (cell == 0 ? 4 : (cell == 1 ? 3 : 1)) * (size_t)d.H;
  hipStream_t s = a.stream;
  if (!ensure_watchdog()) return LSTM_HIP_ERROR;
  DeviceInfo di;
  (void)device_info(di);
  const int slice_rows_narrow = narrow_slice_rows(d, cell, knobs().fwd_narrow);
  const bool narrow_slices = slice_rows_narrow > 0;
  const BatchPlan bp = narrow_slices ? BatchPlan{slice_rows_narrow / 16, 1} : batch_plan(d.B);
  const int BP = 16 * bp.NT;
  const bool wide = cell != 0 || (!narrow_slices && fwd_wide(d));
  float* hx = reinterpret_cast<float*>(a.ws + a.w.xchg);
  int* flags = reinterpret_cast<int*>(a.ws + a.w.flags);
  float* P0 = reinterpret_cast<float*>(a.ws + a.w.P);
  // Wide kernel with I == H: layer 0 multiplies by W_0 inside the kernel like the layers above it (its workgroups
  // are otherwise idle half of every step), reading x from a copy in exchange layout that takes the place of the
  // projection in the workspace.  LSTM_FWD_BATCHED_INPUT=1 keeps the batched product of Section 2.3 instead.
  // (Section 2.3 notes that batching the input products pays at some sizes and not at others; here the batched
  // product only wins where nothing would be idle otherwise: one layer, one slice -- by about 4 %.)
  bool x_in_kernel = wide && d.I == d.H && !(d.L == 1 && d.B <= 64);
  if (x_in_kernel) {
    if (knobs().fwd_batched_input) x_in_kernel = false;
    const size_t rows = (size_t)(d.B + 63) / 64 * 64;  // the copy of x: T+1 slots of H x 64 per slice
    if (((size_t)d.T + 1) * rows * d.H > (size_t)d.L * TB * 4 * d.H) x_in_kernel = false;
  }
  if (!x_in_kernel) {
    ProfScope ps(LSTM_PHASE_FWD_INPUT_GEMM, s);
    GemmProblem p{a.x, a.W, P0, (int)TB, (int)G, d.I, d.I, 1, 1, d.I, (long)G, 0};
    CK(launch_gemm_group(&p, 1, s), "input projection GEMM (layer 0)");
  }
  PersFwdArgs k;
  k.xin = x_in_kernel ? P0 : nullptr;
  k.keep = a.inference ? 0 : 1;
  k.W = a.W; k.R = a.R; k.bias = a.b; k.P0 = P0; k.c0 = a.c0; k.h0 = a.h0; k.hx = hx; k.flags = flags; k.watchdog = g_watch_dev;
  k.res = a.reserve; k.y = a.y; k.hT = a.hT; k.cT = a.cT;
  k.L = d.L; k.T = d.T; k.B = d.B; k.I = d.I; k.H = d.H; k.has_h0 = a.h0 != nullptr; k.spin_limit = spin_limit();
  k.full_fences = full_fences();
  k.trace = (g_trace_bytes >= (size_t)d.T * 64) ? g_trace_buf : nullptr;
  k.trace_block = g_trace_block;
  const int grid = d.L * (d.H / 8);
  // Slices of 64 batch rows run side by side in one launch while the CUs last, the rest in further launches.
  int cap = (wide || narrow_slices) && grid > 0 ? di.cus / grid : 1;
  if (cap > 16 / d.L) cap = 16 / d.L;  // the counter region holds 16 (slice, layer) pairs
  if (cap < 1) cap = 1;
  const int slice_rows = narrow_slices ? slice_rows_narrow : 64;
  const int slices = wide ? (d.B + 63) / 64 : (narrow_slices ? (d.B + slice_rows - 1) / slice_rows : 1);
  for (int s0 = 0; s0 < slices; s0 += cap) {
    const int nsl = slices - s0 < cap ? slices - s0 : cap;
    k.b0 = slice_rows * s0;
    k.nsl = nsl;
    {
      ProfScope ps(LSTM_PHASE_FWD_PACK, s);
      CK(launch_fill_zero(flags, (size_t)nsl * d.L * (d.T + 1) * bp.NC * kFlagInts * 4, s), "zero step counters");
      if (wide) {
        const long n = (long)nsl * d.L * 64 * d.H;
        hipLaunchKernelGGL(pack_state32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a.h0, hx, d.L, d.T,
                           d.B, d.H, k.b0, nsl);
        CK(hipGetLastError(), "pack h0");
        if (x_in_kernel) {
          hipLaunchKernelGGL(pack_x32_kernel, dim3(d.H / 64, d.T, nsl), dim3(256), 0, s, a.x, P0, flags, d.L, d.T, d.B, d.H,
                             k.b0, nsl, d.H / 8);
          CK(hipGetLastError(), "pack x");
        }
      } else if (a.h0) {
        const long n = (long)nsl * d.L * bp.NC * BP * d.H;
        hipLaunchKernelGGL(pack_state_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a.h0, hx, d.L, d.T, d.B,
                           d.H, BP, bp.NC, k.b0, nsl);
        CK(hipGetLastError(), "pack h0");
      }
    }
    ProfScope ps(LSTM_PHASE_FWD_RECURRENCE, s);
    {  // recurrent products of every layer, input products of the layers above the first, and layer 0's when x is multiplied in the kernel
      const double rows = std::min(slice_rows * nsl, d.B - k.b0), per = 2.0 * G * rows * d.T;
      prof_flops(per * d.H * (2 * d.L - 1) + (x_in_kernel ? per * d.I : 0.0), wide ? "pers_fwd32_kernel" : "pers_fwd_kernel");
    }
    hipError_t e = hipErrorInvalidValue;
    if (wide) {
      e = cell == 0 ? launch_fwd32<0>(d.H, grid * nsl, k, s)
                    : (cell == 1 ? launch_fwd32<1>(d.H, grid * nsl, k, s)
                                 : (cell == 2 ? launch_fwd32<2>(d.H, grid * nsl, k, s) : launch_fwd32<3>(d.H, grid * nsl, k, s)));
    }
    else if (d.H == 512) e = launch_fwd<32>(bp, grid * nsl, k, s);
    else if (d.H == 256) e = launch_fwd<16>(bp, grid * nsl, k, s);
    else if (d.H == 128) e = launch_fwd<8>(bp, grid * nsl, k, s);
    CK(e, "persistent forward launch");
  }
  return LSTM_OK;
}

// cell as in run_forward_persistent.  For the other cells the function stops after the propagation (gate gradients
// [L][T*B][4H] at the start of the workspace: GRU r, z, n, and n times r; single gate: the first H columns) and
// reports in *bias_done whether db is complete; the caller forms the weight gradients.
int run_backward_persistent(const BwdArgs& a, int cell, bool* bias_done, LayerGradients* lg) {
  const Dims& d = a.d;
  if (persistent_large(d, true)) {
    if (!ensure_watchdog()) return LSTM_HIP_ERROR;
    return run_backward_persistent_large(a, cell, bias_done, lg);
  }
  const int per = layers_per_launch(d);
  if (per <= 0) return LSTM_UNSUPPORTED;
  if (d.L <= per) return backward_layers(a, cell, bias_done, true);
  const size_t TB = (size_t)d.T * d.B, BH = (size_t)d.B * d.H, GW = (size_t)gates_of_cell(cell) * d.H;
  const size_t rstride = res_width(cell) * TB * d.H;
  const int ngroups = (d.L + per - 1) / per;
  bool all_bias = true;
  for (int gi = ngroups - 1; gi >= 0; --gi) {  // top group first
    const int g0 = gi * per;
    BwdArgs g = a;
    g.d.L = d.L - g0 < per ? d.L - g0 : per;
    const int above = g0 + g.d.L;  // first layer of the group above, if any
    // the gradient handed from group to group lives in the hand-over array of the workspace, slot = receiving layer + 1
    float* const handover = reinterpret_cast<float*>(a.ws + a.w.dx);
    if (g0 > 0) {
      g.d.I = d.H;
      g.x = a.reserve + (size_t)(g0 - 1) * rstride + res_h_offset(cell, TB, d.H);
      g.W = a.W + GW * d.I + (size_t)(g0 - 1) * GW * d.H;
      g.dx = handover + (size_t)g0 * TB * d.H;
    }
    if (above < d.L) g.dy = handover + (size_t)above * TB * d.H;
    g.R = a.R + (size_t)g0 * GW * d.H;
    g.h0 = a.h0 ? a.h0 + (size_t)g0 * BH : nullptr;
    g.c0 = a.c0 ? a.c0 + (size_t)g0 * BH : nullptr;
    g.dhT = a.dhT ? a.dhT + (size_t)g0 * BH : nullptr;
    g.dcT = a.dcT ? a.dcT + (size_t)g0 * BH : nullptr;
    g.dh0 = a.dh0 ? a.dh0 + (size_t)g0 * BH : nullptr;
    g.dc0 = a.dc0 ? a.dc0 + (size_t)g0 * BH : nullptr;
    g.db = a.db ? a.db + (size_t)g0 * GW : nullptr;
    g.reserve = a.reserve + (size_t)g0 * rstride;
    g.w.P = a.w.P + (size_t)g0 * TB * 4 * d.H * sizeof(float);   // gate gradients of the group's layers, in place
    g.w.dx = a.w.dx + (size_t)g0 * TB * d.H * sizeof(float);
    bool done = false;
    const int st = backward_layers(g, cell, &done, false);
    if (st != LSTM_OK) return st;
    all_bias = all_bias && done;
  }
  if (bias_done) *bias_done = all_bias;
  if (cell != 0) return LSTM_OK;
  return weight_gradients(a, reinterpret_cast<const float*>(a.ws + a.w.P), true, all_bias);
}

int backward_layers(const BwdArgs& a, int cell, bool* bias_done, bool with_weight_gradients) {
  const Dims& d = a.d;
  const size_t TB = (size_t)d.T * d.B, G = 4 * (size_t)d.H, GW = (cell == 0 ? 4 : (cell == 1 ? 3 : 1)) * (size_t)d.H;
  hipStream_t s = a.stream;
  if (!ensure_watchdog()) return LSTM_HIP_ERROR;
  const int slice_rows_narrow = narrow_slice_rows(d, cell, knobs().bwd_narrow);
  const bool narrow_slices = slice_rows_narrow > 0;
  const BatchPlan bp = narrow_slices ? BatchPlan{slice_rows_narrow / 16, 1} : batch_plan(d.B);
  const bool wide = cell != 0 || (!narrow_slices && bwd_wide(d));
  int* flags = reinterpret_cast<int*>(a.ws + a.w.flags);
  float* dA = reinterpret_cast<float*>(a.ws + a.w.P);
  PersBwdArgs k;
  k.W = a.W; k.R = a.R; k.res = a.reserve; k.c0 = a.c0; k.h0 = a.h0; k.dy = a.dy; k.dhT = a.dhT; k.dcT = a.dcT;
  k.dA = dA; k.dAx = reinterpret_cast<float*>(a.ws + a.w.xchg); k.dxbuf = reinterpret_cast<float*>(a.ws + a.w.dx);
  k.dh0 = a.dh0; k.dc0 = a.dc0; k.flags = flags; k.watchdog = g_watch_dev;
  // With I == H layer 0 is like every other layer: its workgroups also multiply by W_0 (the rows of the
  // MFMA tile that would otherwise hold zeros) and write the gradient of the network input themselves.
  k.dx0 = (a.dx && d.I == d.H) ? a.dx : nullptr;
  k.db = nullptr;
  if (wide && a.db && d.B <= 64) {  // one launch: the wide kernel adds the bias gradient into db itself (two addends per element)
    ProfScope ps(LSTM_PHASE_BIAS_GRAD, s);
    CK(launch_fill_zero(a.db, (size_t)d.L * GW * 4, s), "zero db");
    k.db = a.db;
  }
  k.L = d.L; k.T = d.T; k.B = d.B; k.I = d.I; k.H = d.H; k.spin_limit = spin_limit(); k.full_fences = full_fences();
  k.trace = (g_trace_bytes >= (size_t)d.T * 64) ? g_trace_buf : nullptr;
  k.trace_block = g_trace_block;
  const int grid = d.L * (d.H / 8);
  // slices of 64 batch rows side by side while the CUs last (see run_forward_persistent): for the wide kernel a
  // slice is two more "batch halves" of 32 rows with their own exchange slots and counters
  DeviceInfo di;
  (void)device_info(di);
  int cap = (wide || narrow_slices) && grid > 0 ? di.cus / grid : 1;
  if (cap > 16 / d.L) cap = 16 / d.L;
  if (cap < 1) cap = 1;
  const int slice_rows = narrow_slices ? slice_rows_narrow : 64;
  const int slices = wide ? (d.B + 63) / 64 : (narrow_slices ? (d.B + slice_rows - 1) / slice_rows : 1);
  for (int s0 = 0; s0 < slices; s0 += cap) {
    const int nsl = slices - s0 < cap ? slices - s0 : cap;
    k.b0 = slice_rows * s0;
    {
      ProfScope ps(LSTM_PHASE_BWD_PACK, s);
      CK(launch_fill_zero(flags, (size_t)nsl * d.L * (d.T + 1) * 2 * kFlagInts * 4, s), "zero step counters");
    }
    ProfScope ps(LSTM_PHASE_BWD_RECURRENCE, s);
    {  // dh products of every layer, dx products of the layers above the first, and layer 0's when the kernel writes dx itself
      const double rows = std::min(slice_rows * nsl, d.B - k.b0), per = 2.0 * GW * rows * d.T;
      prof_flops(per * d.H * (2 * d.L - 1) + (k.dx0 ? per * d.I : 0.0), wide ? "pers_bwd32_kernel" : "pers_bwd_kernel");
    }
    hipError_t e = hipErrorInvalidValue;
    if (wide && cell == 1) {
      e = d.H == 512 ? launch_bwd32<512, 1>(k, 2 * nsl, s)
                     : (d.H == 256 ? launch_bwd32<256, 1>(k, 2 * nsl, s) : launch_bwd32<128, 1>(k, 2 * nsl, s));
    } else if (wide && cell == 2) {
      e = d.H == 512 ? launch_bwd32<512, 2>(k, 2 * nsl, s)
                     : (d.H == 256 ? launch_bwd32<256, 2>(k, 2 * nsl, s) : launch_bwd32<128, 2>(k, 2 * nsl, s));
    } else if (wide && cell == 3) {
      e = d.H == 512 ? launch_bwd32<512, 3>(k, 2 * nsl, s)
                     : (d.H == 256 ? launch_bwd32<256, 3>(k, 2 * nsl, s) : launch_bwd32<128, 3>(k, 2 * nsl, s));
    }
    else if (wide && d.H == 512) e = launch_bwd32<512>(k, 2 * nsl, s);
    else if (wide && d.H == 256) e = launch_bwd32<256>(k, 2 * nsl, s);
    else if (wide && d.H == 128) e = launch_bwd32<128>(k, 2 * nsl, s);
    else if (d.H == 512) e = launch_bwd<128>(bp, grid * nsl, k, s);
    else if (d.H == 256) e = launch_bwd<64>(bp, grid * nsl, k, s);
    else if (d.H == 128) e = launch_bwd<32>(bp, grid * nsl, k, s);
    CK(e, "persistent backward launch");
  }
  if (a.dx && !k.dx0) {  // layer 0's input gradient: all T steps in one product
    ProfScope ps(LSTM_PHASE_BWD_INPUT_GEMM, s);
    GemmProblem p{dA, a.W, a.dx, (int)TB, d.I, (int)GW, (long)G, 1, d.I, 1, d.I, 0};
    CK(launch_gemm_group(&p, 1, s), "input-gradient GEMM (layer 0)");
  }
  if (bias_done) *bias_done = k.db != nullptr;
  if (cell != 0 || !with_weight_gradients) return LSTM_OK;
  return weight_gradients(a, dA, true, k.db != nullptr);
}

}  // namespace lstm
