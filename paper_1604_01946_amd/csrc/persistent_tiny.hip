// Persistent recurrence for a single sequence (B = 1), H = 128 / 256 / 512, LSTM: pers_fwd_tiny_kernel and
// pers_bwd_tiny_kernel.
//
// With one batch row a step is a matrix-vector product of a few microseconds' worth of nothing: the time goes into the
// hop from workgroup to workgroup (Section 4 of arXiv 1604.01946 names the cost of keeping the weights on chip:
// workgroups that wait on each other).  The kernels for wider batches pay per step: store, wait for its
// acknowledgement, workgroup barrier, atomic counter, poll of the counter by every consumer, fetch of the data, matrix
// instructions with a K-split reduction through LDS and another barrier -- about 3 us forward and 4 us backward.  Here
// the hop is as short as the memory system allows:
//   * the data is its own flag: every exchange slot is filled with a pattern that no result can have (a NaN with a
//     payload that arithmetic never produces; a result that happens to carry it is published as the default NaN)
//     before the launch, a producer stores its values with one write-through store and does nothing else, a consumer
//     re-reads the slot with agent-scope loads until no lane sees the pattern.  No acknowledgement, no counter.
//   * a wave owns two hidden units with all their weights over the whole K (lane i holds a few k each; the wave
//     multiplies with vector FMAs and adds up across its lanes), so no wave waits for another one's arithmetic.
//   * the H / 64 waves of a workgroup poll 1 / (H / 64) of the slot each and hand their shares to each other through
//     LDS (one barrier per step): every word of a slot is asked for once per workgroup, not once per wave.
//   * nothing that has to be waited for is issued between a step's poll and its publishing store except what that
//     store needs: the reserve values of later steps are requested right behind a poll (which has waited for
//     everything in flight anyway) and consumed two steps on, in registers that take turns instead of being copied.
// Measured at H = 256 (one or two layers, T = 500): 1.3 us per forward step and 1.4 us per backward step, of which
// about 0.4 us are the wave's own arithmetic (matrix-vector product, lane reduction, gates), the rest the store
// becoming visible and one poll round.
// Section 2.4's wavefront over layers is the same polling: layer l reads the slot of layer l-1 (forward) or the
// hand-over gradient of layer l+1 (backward).  Every poll is bounded (watchdog as in the other persistent kernels).
#include "../../include/lstm.h"
#include "persistent_dev.h"

#include <algorithm>

namespace lstm {
namespace {

constexpr unsigned kEmpty = 0x7FA5C3E1u;  // "not written yet"

__device__ __forceinline__ float poll_load(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish(float* p, float v) {
  unsigned b = __float_as_uint(v);
  if (b == kEmpty) b = 0x7FC00000u;
  __hip_atomic_store(reinterpret_cast<unsigned*>(p), b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The 16-byte request of the backward kernel is inline assembly (there is no 16-byte atomic load to ask the compiler
// for), so the wait for it is written out as well, tied to the value it covers.  Every word is its own flag: a request
// that is served while the producer is writing is simply partly empty.
__device__ __forceinline__ floatx4 request4(const float* p) {
  floatx4 v;
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
  return v;
}
__device__ __forceinline__ void landed(floatx4& v) { asm volatile("s_waitcnt vmcnt(0)" : "+v"(v)::"memory"); }
__device__ __forceinline__ void publish4(float* p, floatx4 v) {
#pragma unroll
  for (int c = 0; c < 4; ++c)
    if (__float_as_uint(v[c]) == kEmpty) v[c] = __uint_as_float(0x7FC00000u);
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}

// Polls: one round after the other, without a pause (measured over the 500 steps of a forward pass at H = 256 with
// every wave polling whole slots: 0.80 ms; with s_sleep 1 between rounds 0.94; with two rounds in flight half a round
// trip apart, so as to notice a value sooner, 1.12: the polls get in each other's way).  What a round costs grows with
// the bytes that all waves together ask the memory for, not with the number or the width of the requests (a backward
// step at H = 256 with every wave polling the whole 4 KB slot took 2.1 us as 16 one-word requests and as 4 four-word
// requests alike; the forward step with 2 KB took 1.3): the waves of a workgroup poll a share of the slot each and
// hand the shares to each other through LDS.
struct TinyWaiter {
  int* watchdog;
  int limit;
  bool dead;
  __device__ __forceinline__ bool give_up(int& spins) {
    if (dead) return true;
    if (++spins > limit) {
      dead = true;
      __hip_atomic_store(watchdog, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      return true;
    }
    return false;
  }
  // One value per lane.
  __device__ __forceinline__ float poll1(const float* p) {
    int spins = 0;
    while (true) {
      const float v = poll_load(p);
      if (__all(__float_as_uint(v) != kEmpty) || give_up(spins)) return v;
    }
  }
  // Two values per lane.
  __device__ __forceinline__ void poll2(const float* pa, float& va, const float* pb, float& vb) {
    int spins = 0;
    while (true) {
      va = poll_load(pa);
      vb = poll_load(pb);
      if (__all(__float_as_uint(va) != kEmpty && __float_as_uint(vb) != kEmpty) || give_up(spins)) return;
    }
  }
  // Four consecutive values per lane.  If pe is given, every round also reads *pe, which is handed back as the last
  // round saw it (possibly still empty): a value that is due later and costs nothing to look at now.
  __device__ __forceinline__ float poll4_peek(const float* pa, floatx4& va, const float* pe) {
    int spins = 0;
    while (true) {
      va = request4(pa);
      float ve = __uint_as_float(kEmpty);
      if (pe) ve = poll_load(pe);
      landed(va);
      bool ok = true;
#pragma unroll
      for (int c = 0; c < 4; ++c) ok = ok && __float_as_uint(va[c]) != kEmpty;
      if (__all(ok) || give_up(spins)) return ve;
    }
  }
};

// Time stamps of one workgroup's first wave, eight per step (the time-stamped instance only).
template <bool TRACE>
struct TinyTracer {
  long long* buf;  // [T][8]
  __device__ __forceinline__ void mark(int step, int slot) const {
    if (TRACE && buf && threadIdx.x == 0) {
      buf[(size_t)step * 8 + slot] = wall_clock64();
      if (slot == 0) buf[(size_t)step * 8 + 7] = clock64();
    }
  }
};

// Sums of N = 4 or 8 per-lane partial values over the 64 lanes, the N sums computed together: in every stage half of
// the lanes hand their part of one value to the other half and take over the other value, so that after log2(N)
// stages each lane carries one value, and the remaining stages add up the lanes that carry the same one.  The sum of
// value r ends up in every lane whose bits 5, 4 (, 3) spell r from the low bit up: lane of_value(r).  All of it stays
// in the vector ALU: the halves of the wave and the rows of 16 lanes are exchanged with v_permlane32_swap /
// v_permlane16_swap (after the swap of x and y, x + y holds x's sum in one half and y's in the other), the rest are
// DPP moves within a row.
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float merge32(float x, float y) {
  const uintx2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float merge16(float x, float y) {
  const uintx2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(y), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
template <int N>
__device__ __forceinline__ float reduce_lanes(const float (&a)[N], int lane) {
  static_assert(N == 4 || N == 8, "four or eight values");
  float b[N / 2];
#pragma unroll
  for (int m = 0; m < N / 2; ++m) b[m] = merge32(a[2 * m], a[2 * m + 1]);
  float c[N / 4];
#pragma unroll
  for (int m = 0; m < N / 4; ++m) c[m] = merge16(b[2 * m], b[2 * m + 1]);
  float d;
  if (N == 8) {
    const bool hi = lane & 8;
    d = (hi ? c[N / 4 - 1] : c[0]) + dpp_move<0x128>(hi ? c[0] : c[N / 4 - 1]);  // row_ror:8
  } else {
    d = c[0] + dpp_move<0x140>(c[0]);  // row_mirror: the other half of the row (used last: see below)
  }
  // within the remaining 8 (N = 8) or 16 (N = 4) lanes: quads, then the other quad of the half row; for N = 4 the
  // mirror above has already folded the two half rows (every lane pairs with one of the other half)
  d += dpp_move<0xB1>(d);   // quad_perm [1,0,3,2]
  d += dpp_move<0x4E>(d);   // quad_perm [2,3,0,1]
  d += dpp_move<0x141>(d);  // row_half_mirror
  return d;
}
template <int N>
__device__ __forceinline__ constexpr int of_value(int r) {
  return ((r & 1) << 5) | (((r >> 1) & 1) << 4) | (N == 8 ? (((r >> 2) & 1) << 3) : 0);
}
__device__ __forceinline__ float lane_value(float v, int src_lane) {
  return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), src_lane));
}

// ------------------------------------------------------------------ forward
// Workgroup (l, q) of H / 64 waves: wave w owns units u0 = 2 * (q * H / 64 + w), u0 + 1 of layer l (32 workgroups per
// layer); rows r = 4*j + gate of the stacked matrices (j: which of the two units).  Exchange: hx [L][T+1][H], slot t+1 =
// h_t, slot 0 = h0 (or zeros), everything else the empty pattern before the launch.  Wave w polls words 64 w ... of the
// two operands.  Layer 0 takes its input product from the batched projection P0 [T][4H] (Section 2.3).
constexpr int kTinyGroups = 32;  // workgroups per layer

template <int HH, bool TRACE>
__global__ __launch_bounds__(HH) void pers_fwd_tiny_kernel(const PersFwdArgs a) {
  constexpr int H = HH, G = 4 * H, NI = H / 64, NW = H / 64;
  __shared__ __align__(16) float xs[2][2][H];  // [step parity][x, h][word]
  int l, q;
  map_block(a.L, kTinyGroups, l, q);
  const int T = a.T, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int u0 = 2 * (q * NW + wave);

  // value m of a lane: word (64 * (m / VW) + lane) * VW + m % VW of the operand (read from LDS VW words at a time)
  constexpr int VW = NI < 4 ? NI : 4;
  float wW[8][NI], wR[8][NI];
  {
    const float* Rl = a.R + (size_t)l * G * H;
    const float* Wl = a.W + (size_t)G * a.I + (size_t)(l > 0 ? l - 1 : 0) * G * H;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const size_t row = ((size_t)(r & 3) * H + u0 + (r >> 2)) * H;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int k = (64 * (i / VW) + lane) * VW + i % VW;
        wR[r][i] = Rl[row + k];
        wW[r][i] = l > 0 ? Wl[row + k] : 0.f;
      }
    }
  }
  // lanes 0 and 1 finalise the two units (every lane runs the arithmetic; only they store)
  const int j = lane & 1, uj = u0 + j;
  const bool fin = lane < 2;
  float bias[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) bias[g] = a.bias[(size_t)l * G + g * H + uj];
  float c_state = a.c0 ? a.c0[(size_t)l * H + uj] : 0.f;

  float* const res_l = a.res + (size_t)l * T * 6 * H;
  float* const res_c = res_l + (size_t)T * 4 * H;
  float* const res_h = res_l + (size_t)T * 5 * H;
  auto slot = [&](int layer, int st) { return a.hx + ((size_t)layer * (T + 1) + st) * H; };
  TinyWaiter w{a.watchdog, a.spin_limit, false};
  const TinyTracer<TRACE> tr{(int)blockIdx.x == a.trace_block ? a.trace : nullptr};

  // Loads return in the order of their issue, so an ordinary load requested just before a poll holds up the poll's
  // first round: the input product of step t + 1 is requested behind the poll of step t and taken over behind the
  // poll of step t + 1, which has waited for everything in flight anyway.
  float pin[4], pin_next[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) pin_next[g] = l == 0 ? a.P0[g * H + uj] : 0.f;
  for (int t = 0; t < T; ++t) {
    const int par = t & 1, mine = 64 * wave + lane;
    tr.mark(t, 0);
    float vx = 0.f, vh;  // (layer 0 has no input operand in the exchange)
    if (l > 0) w.poll2(slot(l - 1, t + 1) + mine, vx, slot(l, t) + mine, vh);
    else vh = w.poll1(slot(l, t) + mine);
    tr.mark(t, 1);
    xs[par][0][mine] = vx;
    xs[par][1][mine] = vh;
    // (one barrier per step: the buffer written two steps on is the one every wave has read before it arrived here)
    __syncthreads();
    tr.mark(t, 2);
#pragma unroll
    for (int g = 0; g < 4; ++g) pin[g] = pin_next[g];
    if (l == 0 && t + 1 < T) {
#pragma unroll
      for (int g = 0; g < 4; ++g) pin_next[g] = a.P0[(size_t)(t + 1) * G + g * H + uj];
    }
    float xi[NI], hr[NI];
#pragma unroll
    for (int i = 0; i < NI / VW; ++i) {
      typedef float vec __attribute__((ext_vector_type(VW)));
      const vec qx = *reinterpret_cast<const vec*>(&xs[par][0][(64 * i + lane) * VW]);
      const vec qh = *reinterpret_cast<const vec*>(&xs[par][1][(64 * i + lane) * VW]);
#pragma unroll
      for (int c = 0; c < VW; ++c) {
        xi[i * VW + c] = qx[c];
        hr[i * VW + c] = qh[c];
      }
    }
    float acc[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < NI; ++i) s = fmaf(wW[r][i], xi[i], fmaf(wR[r][i], hr[i], s));
      acc[r] = s;
    }
    const float d = reduce_lanes<8>(acc, lane);
    float sg[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float s0 = lane_value(d, of_value<8>(g)), s1 = lane_value(d, of_value<8>(4 + g));
      sg[g] = (j ? s1 : s0) + pin[g] + bias[g];
    }
    const float gi = sigmoidf_dev(sg[0]), gf = sigmoidf_dev(sg[1]), go = sigmoidf_dev(sg[2]), gc = tanhf_dev(sg[3]);
    const float cn = gf * c_state + gi * gc;
    const float hn = go * tanhf_dev(cn);
    c_state = cn;
    tr.mark(t, 3);
    if (fin) {
      publish(slot(l, t + 1) + uj, hn);
      float* const rg = res_l + (size_t)t * G + uj;
      rg[0] = gi;
      rg[H] = gf;
      rg[2 * H] = go;
      rg[3 * H] = gc;
      res_c[(size_t)t * H + uj] = cn;
      res_h[(size_t)t * H + uj] = hn;
      if (l == a.L - 1) a.y[(size_t)t * H + uj] = hn;
      if (t == T - 1) {
        if (a.hT) a.hT[(size_t)l * H + uj] = hn;
        if (a.cT) a.cT[(size_t)l * H + uj] = cn;
      }
    }
  }
}

// hx [L][T+1][H]: slot 0 <- h0 (zeros if null), the rest <- the empty pattern
__global__ void tiny_prepare_fwd_kernel(float* __restrict__ hx, const float* __restrict__ h0, int L, int T, int H) {
  const long n = (long)L * (T + 1) * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long)gridDim.x * blockDim.x) {
    const int k = (int)(e % H), st = (int)((e / H) % (T + 1)), l = (int)(e / ((long)H * (T + 1)));
    float v = __uint_as_float(kEmpty);
    if (st == 0) {  // (an initial state that carries the empty pattern would never be seen as written)
      v = h0 ? h0[(size_t)l * H + k] : 0.f;
      if (__float_as_uint(v) == kEmpty) v = __uint_as_float(0x7FC00000u);
    }
    hx[e] = v;
  }
}

__global__ void tiny_fill_empty_kernel(float* __restrict__ p, long n) {
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long)gridDim.x * blockDim.x)
    p[e] = __uint_as_float(kEmpty);
}

// ------------------------------------------------------------------ backward
// Wave (l, p): units u0 = 2p, 2p + 1: four output rows over K = 4H -- dh_{t-1} of the two units (columns of R_l) and
// the gradient dx_t for the same two units of the layer below (columns of W_l; layer 0: of the network input when
// I == H and it is wanted).  Exchange: dAx [L][T][H][4] gate gradients (the four gates of a unit side by side: one
// 16-byte store publishes them), dxbuf [L][T][H] hand-over gradients (slice l written by layer l >= 1, read by layer
// l-1), both the empty pattern before the launch.  The bias gradient of a unit is
// the sum over t of its gate gradients, which its lane carries along: no reduction, no atomic.
template <int HH, bool TRACE>
__global__ __launch_bounds__(HH) void pers_bwd_tiny_kernel(const PersBwdArgs a) {
  constexpr int H = HH, G = 4 * H, NI = G / 64, NW = H / 64;
  __shared__ __align__(16) float ds[2][G];  // [step parity][word of the slot]
  int l, q;
  map_block(a.L, kTinyGroups, l, q);
  const int T = a.T, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int u0 = 2 * (q * NW + wave);

  float wR[2][NI], wW[2][NI];
  {
    const float* Rl = a.R + (size_t)l * G * H + u0;
    const float* Wl = (l > 0 ? a.W + (size_t)G * a.I + (size_t)(l - 1) * G * H : a.W) + u0;  // layer 0: [G][I], I == H
    const bool live = l > 0 || a.dx0;
    // value m of a lane: gate m % 4 of unit 64 * (m / 4) + lane (read from LDS four words at a time)
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const size_t k = ((size_t)(i & 3) * H + 64 * (i >> 2) + lane) * H;
        wR[jj][i] = Rl[k + jj];
        wW[jj][i] = live ? Wl[k + jj] : 0.f;
      }
  }
  const int j = lane & 1, uj = u0 + j;
  const bool fin = lane < 2;
  const size_t se = (size_t)l * H + uj;
  float dc = a.dcT ? a.dcT[se] : 0.f;
  float dh_rec = a.dhT ? a.dhT[se] : 0.f;
  float dbsum[4] = {0.f, 0.f, 0.f, 0.f};

  const float* const res_l = a.res + (size_t)l * T * 6 * H;
  const float* const res_c = res_l + (size_t)T * 4 * H;
  float* const dA_l = a.dA + (size_t)l * T * G;
  const bool has_up = l < a.L - 1;
  auto dslot = [&](int layer, int t) { return a.dAx + ((size_t)layer * T + t) * G; };
  auto xslot = [&](int layer, int t) { return a.dxbuf + ((size_t)layer * T + t) * H; };
  TinyWaiter w{a.watchdog, a.spin_limit, false};
  const TinyTracer<TRACE> tr{(int)blockIdx.x == a.trace_block ? a.trace : nullptr};

  // Reserve values (and dy) of one step for this lane's unit, and what the point-wise stage makes of them before the
  // incoming gradient is known.  Loads return in the order of their issue, so an ordinary load requested just before
  // a poll holds up the poll's first round: the values of step t - 3 are requested behind the poll of step t, and
  // those of step t - 1 are worked up while step t's own gate gradients are on their way.  The two sets of registers
  // take turns (the loop runs two steps per iteration) so that no value is copied at the end of an iteration, which
  // would wait for everything in flight.
  struct Saved {
    float gi, gf, go, gg, ct, cp, dy;
  };
  struct Ready {
    float k_c, k_i, k_f, k_o, k_g, gf, dy;  // dc += dh * k_c; d = dc * k_i, dc * k_f, dh * k_o, dc * k_g; dc *= gf
  };
  auto fetch = [&](int t) {
    Saved v;
    const float* const rg = res_l + (size_t)t * G + uj;
    v.gi = rg[0];
    v.gf = rg[H];
    v.go = rg[2 * H];
    v.gg = rg[3 * H];
    v.ct = res_c[(size_t)t * H + uj];
    v.cp = t > 0 ? res_c[(size_t)(t - 1) * H + uj] : (a.c0 ? a.c0[se] : 0.f);
    v.dy = has_up ? 0.f : a.dy[(size_t)t * H + uj];
    return v;
  };
  auto work_up = [&](const Saved& v) {
    Ready k;
    const float tc = tanhf_dev(v.ct);
    k.k_c = v.go * (1.f - tc * tc);
    k.k_i = v.gg * v.gi * (1.f - v.gi);
    k.k_f = v.cp * v.gf * (1.f - v.gf);
    k.k_o = tc * v.go * (1.f - v.go);
    k.k_g = v.gi * (1.f - v.gg * v.gg);
    k.gf = v.gf;
    k.dy = v.dy;
    return k;
  };
  Ready k = work_up(fetch(T - 1));
  Saved ra = fetch(T > 1 ? T - 2 : 0), rb = fetch(T > 2 ? T - 3 : 0);
  // hand-over gradient of the step about to start, looked at during the previous step's poll (empty: not there yet)
  float seen = __uint_as_float(kEmpty);

  // step t; rx: the reserve values of step t - 1 on entry, of step t - 3 on exit
  auto step = [&](int t, Saved& rx) {
    // ---- point-wise stage of step t
    tr.mark(t, 0);
    float dout = k.dy;
    if (has_up) dout = __all(__float_as_uint(seen) != kEmpty) ? seen : w.poll1(xslot(l + 1, t) + uj);
    tr.mark(t, 1);
    const float dh = dout + dh_rec;
    const float dcv = dc + dh * k.k_c;
    const float d[4] = {dcv * k.k_i, dcv * k.k_f, dh * k.k_o, dcv * k.k_g};
    dc = dcv * k.gf;
    if (fin) {
      publish4(dslot(l, t) + 4 * uj, floatx4{d[0], d[1], d[2], d[3]});
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        dA_l[(size_t)t * G + g * H + uj] = d[g];
        dbsum[g] += d[g];
      }
    }
    if (t > 0) k = work_up(rx);
    // ---- dh_{t-1} and dx_t: needs dA_t of every unit of the layer
    // (wave w polls words 256 w ... of the slot)
    const int par = t & 1, mine = 256 * wave + 4 * lane;
    tr.mark(t, 2);
    // A poll round that comes back partly empty costs more than its own time: it is in the way of the stores it is
    // waiting for.  Every wave publishes at about the same moment, so the first round is held back until those stores
    // are about to be visible (measured at H = 256: 1.72 us per step with no pause, 1.57 with 192 cycles, 1.44 with
    // 512, 1.57 with 1024; the forward kernel has its stores to the reserve in this place and gains nothing).
    __builtin_amdgcn_s_sleep(8);
    floatx4 share;
    seen = w.poll4_peek(dslot(l, t) + mine, share, has_up && t > 0 ? xslot(l + 1, t - 1) + uj : nullptr);
    tr.mark(t, 3);
    *reinterpret_cast<floatx4*>(&ds[par][mine]) = share;
    __syncthreads();  // (one barrier per step is enough: see the forward kernel)
    tr.mark(t, 4);
    if (t > 2) rx = fetch(t - 3);
    float da[NI];
#pragma unroll
    for (int i = 0; i < NI / 4; ++i) {
      const floatx4 qd = *reinterpret_cast<const floatx4*>(&ds[par][(64 * i + lane) * 4]);
#pragma unroll
      for (int c = 0; c < 4; ++c) da[i * 4 + c] = qd[c];
    }
    float acc[4];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        s0 = fmaf(wR[jj][i], da[i], s0);
        s1 = fmaf(wW[jj][i], da[i], s1);
      }
      acc[jj] = s0;
      acc[2 + jj] = s1;
    }
    const float r = reduce_lanes<4>(acc, lane);
    const float h0v = lane_value(r, of_value<4>(0)), h1v = lane_value(r, of_value<4>(1));
    const float x0v = lane_value(r, of_value<4>(2)), x1v = lane_value(r, of_value<4>(3));
    dh_rec = j ? h1v : h0v;
    const float dxv = j ? x1v : x0v;
    tr.mark(t, 5);
    if (fin) {
      if (l > 0) publish(xslot(l, t) + uj, dxv);
      else if (a.dx0) a.dx0[(size_t)t * a.I + uj] = dxv;
    }
  };
  int t = T - 1;
  for (; t >= 1; t -= 2) {
    step(t, ra);
    step(t - 1, rb);
  }
  if (t == 0) step(0, ra);
  if (fin) {
    if (a.dh0) a.dh0[se] = dh_rec;
    if (a.dc0) a.dc0[se] = dc;
    if (a.db) {
#pragma unroll
      for (int g = 0; g < 4; ++g) a.db[(size_t)l * G + g * H + uj] = dbsum[g];
    }
  }
}

}  // namespace

hipError_t launch_fwd_tiny(int H, const PersFwdArgs& a, hipStream_t s) {
  const long n = (long)a.L * (a.T + 1) * H;
  hipLaunchKernelGGL(tiny_prepare_fwd_kernel, dim3((unsigned)std::min<long>((n + 255) / 256, 1024)), dim3(256), 0, s, a.hx, a.h0, a.L,
                     a.T, H);
  const void* fn = H == 512 ? (const void*)pers_fwd_tiny_kernel<512, false>
                            : (H == 256 ? (const void*)pers_fwd_tiny_kernel<256, false> : (const void*)pers_fwd_tiny_kernel<128, false>);
  if (a.trace)
    fn = H == 512 ? (const void*)pers_fwd_tiny_kernel<512, true>
                  : (H == 256 ? (const void*)pers_fwd_tiny_kernel<256, true> : (const void*)pers_fwd_tiny_kernel<128, true>);
  void* params[] = {const_cast<PersFwdArgs*>(&a)};
  return launch_resident(fn, a.L * kTinyGroups, params, 0, s, H);
}

hipError_t launch_bwd_tiny(int H, const PersBwdArgs& a, hipStream_t s) {
  const long n1 = (long)a.L * a.T * 4 * H, n2 = (long)a.L * a.T * H;
  hipLaunchKernelGGL(tiny_fill_empty_kernel, dim3((unsigned)std::min<long>((n1 + 255) / 256, 1024)), dim3(256), 0, s, a.dAx, n1);
  hipLaunchKernelGGL(tiny_fill_empty_kernel, dim3((unsigned)std::min<long>((n2 + 255) / 256, 1024)), dim3(256), 0, s, a.dxbuf, n2);
  const void* fn = H == 512 ? (const void*)pers_bwd_tiny_kernel<512, false>
                            : (H == 256 ? (const void*)pers_bwd_tiny_kernel<256, false> : (const void*)pers_bwd_tiny_kernel<128, false>);
  if (a.trace)
    fn = H == 512 ? (const void*)pers_bwd_tiny_kernel<512, true>
                  : (H == 256 ? (const void*)pers_bwd_tiny_kernel<256, true> : (const void*)pers_bwd_tiny_kernel<128, true>);
  void* params[] = {const_cast<PersBwdArgs*>(&a)};
  return launch_resident(fn, a.L * kTinyGroups, params, 0, s, H);
}

}  // namespace lstm
