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
//     before the launch, a producer stores its values with a write-through store and does nothing else, a consumer
//     re-reads the slot with agent-scope loads until no lane sees the pattern.  No acknowledgement, no counter.
//   * a wave owns two hidden units with all their weights over the whole K (lane i holds k = i, i + 64, ...; the wave
//     multiplies with vector FMAs and adds up across its lanes), so no wave waits for another one of its
//     workgroup: there is no barrier and no LDS in a step, and a workgroup is a single wave.
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

struct TinyWaiter {
  int* watchdog;
  int limit;
  bool dead;
  // Reads NA values per lane from pa and NB from pb (element 64*i + lane) until none of them is the empty pattern.
  // One round after the other, without a pause (measured over the 500 steps of a forward pass at H = 256: 0.80 ms;
  // with s_sleep 1 between rounds 0.94; with two rounds in flight half a round trip apart, so as to notice a value
  // sooner, 1.12: the polls of 256 waves on the same lines get in each other's way).
  template <int NA, int NB>
  __device__ __forceinline__ void poll(const float* pa, float (&va)[NA], const float* pb, float (&vb)[NB]) {
    const int lane = threadIdx.x & 63;
    int spins = 0;
    while (true) {
#pragma unroll
      for (int i = 0; i < NA; ++i) va[i] = poll_load(pa + 64 * i + lane);
#pragma unroll
      for (int i = 0; i < NB; ++i) vb[i] = poll_load(pb + 64 * i + lane);
      bool ok = true;
#pragma unroll
      for (int i = 0; i < NA; ++i) ok = ok && __float_as_uint(va[i]) != kEmpty;
#pragma unroll
      for (int i = 0; i < NB; ++i) ok = ok && __float_as_uint(vb[i]) != kEmpty;
      if (__all(ok) || dead) return;
      if (++spins > limit) {
        dead = true;
        __hip_atomic_store(watchdog, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        return;
      }
    }
  }
  template <int NA>
  __device__ __forceinline__ void poll1n(const float* pa, float (&va)[NA]) {
    const int lane = threadIdx.x & 63;
    int spins = 0;
    while (true) {
#pragma unroll
      for (int i = 0; i < NA; ++i) va[i] = poll_load(pa + 64 * i + lane);
      bool ok = true;
#pragma unroll
      for (int i = 0; i < NA; ++i) ok = ok && __float_as_uint(va[i]) != kEmpty;
      if (__all(ok) || dead) return;
      if (++spins > limit) {
        dead = true;
        __hip_atomic_store(watchdog, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        return;
      }
    }
  }
  // One value per lane (the same few addresses in every lane).
  __device__ __forceinline__ float poll1(const float* p) {
    int spins = 0;
    while (true) {
      const float v = poll_load(p);
      if (__all(__float_as_uint(v) != kEmpty) || dead) return v;
      if (++spins > limit) {
        dead = true;
        __hip_atomic_store(watchdog, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        return v;
      }
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
// Wave (l, p): units u0 = 2p, 2p + 1 of layer l; rows r = 4*j + gate of the stacked matrices (j: which of the two
// units).  Exchange: hx [L][T+1][H], slot t+1 = h_t, slot 0 = h0 (or zeros), everything else the empty pattern before
// the launch.  Layer 0 takes its input product from the batched projection P0 [T][4H] (Section 2.3).
template <int HH>
__global__ __launch_bounds__(64) void pers_fwd_tiny_kernel(const PersFwdArgs a) {
  constexpr int H = HH, G = 4 * H, NI = H / 64, NP = H / 2;
  int l, p;
  map_block(a.L, NP, l, p);
  const int T = a.T, lane = threadIdx.x & 63;
  const int u0 = 2 * p;

  float wW[8][NI], wR[8][NI];
  {
    const float* Rl = a.R + (size_t)l * G * H;
    const float* Wl = a.W + (size_t)G * a.I + (size_t)(l > 0 ? l - 1 : 0) * G * H;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const size_t row = ((size_t)(r & 3) * H + u0 + (r >> 2)) * H;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        wR[r][i] = Rl[row + 64 * i + lane];
        wW[r][i] = l > 0 ? Wl[row + 64 * i + lane] : 0.f;
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

  for (int t = 0; t < T; ++t) {
    float pin[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) pin[g] = l == 0 ? a.P0[(size_t)t * G + g * H + uj] : 0.f;
    float xi[NI], hr[NI];
    // (layer 0 has no input operand in the exchange: it reads its own recurrent slot twice; those weights are zero)
    w.poll(l > 0 ? slot(l - 1, t + 1) : slot(l, t), xi, slot(l, t), hr);
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
// I == H and it is wanted).  Exchange: dAx [L][T][4H] gate gradients, dxbuf [L][T][H] hand-over gradients (slice l
// written by layer l >= 1, read by layer l-1), both the empty pattern before the launch.  The bias gradient of a unit is
// the sum over t of its gate gradients, which its lane carries along: no reduction, no atomic.
template <int HH>
__global__ __launch_bounds__(64) void pers_bwd_tiny_kernel(const PersBwdArgs a) {
  constexpr int H = HH, G = 4 * H, NI = G / 64, NP = H / 2;
  int l, p;
  map_block(a.L, NP, l, p);
  const int T = a.T, lane = threadIdx.x & 63;
  const int u0 = 2 * p;

  float wR[2][NI], wW[2][NI];
  {
    const float* Rl = a.R + (size_t)l * G * H + u0;
    const float* Wl = (l > 0 ? a.W + (size_t)G * a.I + (size_t)(l - 1) * G * H : a.W) + u0;  // layer 0: [G][I], I == H
    const bool live = l > 0 || a.dx0;
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const size_t k = (size_t)(64 * i + lane) * H;
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

  float gi, gf, go, gg, ct, cp, dy = 0.f;
  auto fetch = [&](int t) {  // reserve values (and dy) of step t for this lane's unit
    const float* const rg = res_l + (size_t)t * G + uj;
    gi = rg[0];
    gf = rg[H];
    go = rg[2 * H];
    gg = rg[3 * H];
    ct = res_c[(size_t)t * H + uj];
    cp = t > 0 ? res_c[(size_t)(t - 1) * H + uj] : (a.c0 ? a.c0[se] : 0.f);
    if (!has_up) dy = a.dy[(size_t)t * H + uj];
  };
  fetch(T - 1);

  for (int t = T - 1; t >= 0; --t) {
    // ---- point-wise stage of step t
    const float dout = has_up ? w.poll1(xslot(l + 1, t) + uj) : dy;
    const float dh = dout + dh_rec;
    const float tc = tanhf_dev(ct);
    const float dcv = dc + dh * go * (1.f - tc * tc);
    float d[4];
    d[0] = dcv * gg * gi * (1.f - gi);
    d[1] = dcv * cp * gf * (1.f - gf);
    d[2] = dh * tc * go * (1.f - go);
    d[3] = dcv * gi * (1.f - gg * gg);
    dc = dcv * gf;
    if (fin) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        publish(dslot(l, t) + g * H + uj, d[g]);
        dA_l[(size_t)t * G + g * H + uj] = d[g];
        dbsum[g] += d[g];
      }
    }
    if (t > 0) fetch(t - 1);  // under the hop
    // ---- dh_{t-1} and dx_t: needs dA_t of every unit of the layer
    float da[NI];
    w.poll1n(dslot(l, t), da);
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
    if (fin) {
      if (l > 0) publish(xslot(l, t) + uj, dxv);
      else if (a.dx0) a.dx0[(size_t)t * a.I + uj] = dxv;
    }
  }
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
  const void* fn = H == 512 ? (const void*)pers_fwd_tiny_kernel<512>
                            : (H == 256 ? (const void*)pers_fwd_tiny_kernel<256> : (const void*)pers_fwd_tiny_kernel<128>);
  void* params[] = {const_cast<PersFwdArgs*>(&a)};
  return launch_resident(fn, a.L * (H / 2), params, 0, s, 64);
}

hipError_t launch_bwd_tiny(int H, const PersBwdArgs& a, hipStream_t s) {
  const long n1 = (long)a.L * a.T * 4 * H, n2 = (long)a.L * a.T * H;
  hipLaunchKernelGGL(tiny_fill_empty_kernel, dim3((unsigned)std::min<long>((n1 + 255) / 256, 1024)), dim3(256), 0, s, a.dAx, n1);
  hipLaunchKernelGGL(tiny_fill_empty_kernel, dim3((unsigned)std::min<long>((n2 + 255) / 256, 1024)), dim3(256), 0, s, a.dxbuf, n2);
  const void* fn = H == 512 ? (const void*)pers_bwd_tiny_kernel<512>
                            : (H == 256 ? (const void*)pers_bwd_tiny_kernel<256> : (const void*)pers_bwd_tiny_kernel<128>);
  void* params[] = {const_cast<PersBwdArgs*>(&a)};
  return launch_resident(fn, a.L * (H / 2), params, 0, s, 64);
}

}  // namespace lstm
