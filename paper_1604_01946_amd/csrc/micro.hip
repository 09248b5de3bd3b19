// A whole pass in one workgroup: lstm_micro_fwd_kernel / lstm_micro_bwd_kernel, for networks so small that a launch
// per step costs more than the step (H = 8 / 16 / 32, I <= 64, B <= 8: a step is a few thousand multiply-adds,
// a launch a few microseconds).  Section 3.1 of arXiv 1604.01946 names the two extremes: one large product per
// step at the top of the range, launch overhead at the bottom.  Here one launch runs all layers and steps of a pass
// (the backward one the weight gradients of Section 2.6 as well); the weights of the layer at hand live in the
// registers of the workgroup's 512 threads, the step's vectors in LDS, two barriers per step.
//
// A step is shorter than one trip to memory, so nothing inside the loop over the steps waits for memory: what the
// steps read (inputs; in the backward pass the gates, cell states, hidden states and incoming gradients as well) is
// brought into LDS for as many steps at a time as fit, in one batch of requests, and what they write is stored and
// not waited for (the barriers inside the loop order LDS only).
//
// Forward.  The K = I_l + H columns of [W_l | R_l] are padded to KP = 64 or 96 and cut into 8 parts; thread (rows, part p)
// keeps the part of R = 1 or 2 adjacent rows of the 4H stacked gate rows in registers for all T steps.  The products
// with [x_t | h_{t-1}] are added up over the part, then over the 8 neighbouring lanes; lane p then applies the gate's
// non-linearity for batch row p, so that the B values of a row are spread over the lanes.  Cells: one per thread.
//
// Backward.  The same (rows, part) layout accumulates dW_l, dR_l (one register per weight) and db_l over the steps;
// for dh_{t-1} and dx_t a second layout holds the transposed slice: thread (column q of [W_l | R_l], part rs of the
// 4H rows).  Every sum is added in a fixed order: repeatable bit for bit.
#include <algorithm>
#include <cstdint>

#include "../../include/lstm.h"
#include "internal.h"
#include "knobs.h"
#include "persistent.h"
#include "schedule.h"

namespace lstm {
namespace {

constexpr int kMicroMaxI = 64, kMicroMaxB = 8;
constexpr int kMicroK = 96;              // columns of [W_l | R_l], padded: I_l + H <= 64 + 32
constexpr int kMicroStaged = 24576;      // floats of LDS for the staged steps (96 KB)
constexpr int kMicroThreads = 512;

struct MicroFwdArgs {
  const float *x, *h0, *c0, *W, *R, *b;
  float *y, *hT, *cT, *res;
  int L, T, B, I;
  int C;  // steps staged at a time
};

struct MicroBwdArgs {
  const float *x, *h0, *c0, *W, *R, *res, *dy, *dhT, *dcT;
  float *dx, *dh0, *dc0, *dW, *dR, *db;
  float* hand;  // [2][T][B][H]: gradient handed from a layer to the one below (the two halves take turns)
  int L, T, B, I;
  int C;
};

template <int CTRL>
__device__ __forceinline__ float dpp_get(float v) {  // the value of another lane of the row (every lane active)
  return __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), CTRL, 0xf, 0xf, false));
}

// Sum over the aligned group of N = 4 or 8 neighbouring lanes; every lane of the group gets it, added in one order.
template <int N>
__device__ __forceinline__ float sum_lanes(float v) {
  v += dpp_get<0xB1>(v);               // quad_perm [1,0,3,2]
  v += dpp_get<0x4E>(v);               // quad_perm [2,3,0,1]
  if (N == 8) v += dpp_get<0x141>(v);  // row_half_mirror: the other quad of the eight
  return v;
}

// Barrier that orders the workgroup's LDS traffic only: stores to device memory stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ bool aligned16_dev(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// NS pieces of device memory, one after the other in LDS, in units of 16 bytes: piece k ends at end[k]; a piece
// without a source is filled with zeros.  All requests of a batch (U per thread) are issued before the first is used.
template <int NS>
struct Segs {
  const float4* src[NS];
  int end[NS];
};

template <int NS, int U>
__device__ __forceinline__ void stage_segs(float4* dst, const Segs<NS>& s, int tid) {
  const int total = s.end[NS - 1];
  for (int base = 0; base < total; base += kMicroThreads * U) {
    float4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = base + u * kMicroThreads + tid;
      const float4* sp = s.src[0];
      int st = 0;
#pragma unroll
      for (int k = 1; k < NS; ++k)
        if (idx >= s.end[k - 1]) {
          sp = s.src[k];
          st = s.end[k - 1];
        }
      v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (idx < total && sp) v[u] = sp[idx - st];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = base + u * kMicroThreads + tid;
      if (idx < total) dst[idx] = v[u];
    }
  }
}

template <int U>
__device__ __forceinline__ void stage_scalar(float* dst, const float* src, int n, int tid) {
  for (int base = 0; base < n; base += kMicroThreads * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = base + u * kMicroThreads + tid;
      v[u] = idx < n ? src[idx] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = base + u * kMicroThreads + tid;
      if (idx < n) dst[idx] = v[u];
    }
  }
}

// Layout shared by the forward product and the weight gradients: thread (rg, p) = (tid / 8, tid % 8) has rows
// rg R .. rg R + R - 1 and columns p KSL .. p KSL + KSL - 1.
template <int H, int KP>
struct RowPart {
  static constexpr int G = 4 * H;
  static constexpr int R = G * 8 > kMicroThreads ? G * 8 / kMicroThreads : 1;
  static constexpr int NRG = G / R;  // row groups: the threads from NRG * 8 on have no rows
  static constexpr int KSL = KP / 8;
  static_assert(KSL % 4 == 0 && NRG * 8 <= kMicroThreads, "a part is read four columns at a time");
};

struct MicroLds {
  float* act;     // [8][KP]: [x_t | h_{t-1} | 0] per batch row
  float* gates;   // [8][4H]: forward: the activated gates of the step; backward: the gate gradients
  float* dhs;     // [8][H]: backward: dh_{t-1} from the recurrent product
  float4* staged4;
};

template <int H, int KP>
__device__ __forceinline__ void micro_fwd_layer(const MicroFwdArgs& a, const int l, const MicroLds& m) {
  using S = RowPart<H, KP>;
  constexpr int G = S::G, R = S::R, KSL = S::KSL;
  float* const sx = reinterpret_cast<float*>(m.staged4);  // [C][B][I_l]: inputs of the staged steps
  const int tid = threadIdx.x, rg = tid >> 3, p = tid & 7;
  const bool rows = rg < S::NRG;
  const int T = a.T, B = a.B;
  const size_t TB = (size_t)T * B;
  const int Il = l == 0 ? a.I : H, K = Il + H, BI = B * Il, BH = B * H;
  const float* Wl = a.W + (l == 0 ? 0 : (size_t)G * a.I + (size_t)(l - 1) * G * H);
  const float* Rl = a.R + (size_t)l * G * H;
  float* const res_l = a.res + (size_t)l * TB * 6 * H;
  float* const res_c = res_l + TB * 4 * H;
  float* const res_h = res_l + TB * 5 * H;
  const float* const in = l == 0 ? a.x : a.res + (size_t)(l - 1) * TB * 6 * H + TB * 5 * H;
  float wv[R][KSL], bias[R];
#pragma unroll
  for (int j = 0; j < R; ++j) {
    const int r = rg * R + j;
#pragma unroll
    for (int i = 0; i < KSL; ++i) {
      const int k = p * KSL + i;
      wv[j][i] = !rows ? 0.f : (k < Il ? Wl[r * Il + k] : (k < K ? Rl[r * H + (k - Il)] : 0.f));
    }
    bias[j] = rows ? a.b[(size_t)l * G + r] : 0.f;
  }
  const bool cell = tid < BH;  // one cell per thread: batch row tid / H, unit tid % H
  float c_state = (cell && a.c0) ? a.c0[(size_t)l * BH + tid] : 0.f;
  const float h0v = (cell && a.h0) ? a.h0[(size_t)l * BH + tid] : 0.f;
  const int xo = tid < BI ? (tid / Il) * KP + tid % Il : -1;  // where this thread's element of x_t goes in act
  // The first layer's weights, states and first staged steps are all requested before anything waits: one trip.
  if (l > 0) __syncthreads();  // the layer before has finished with the LDS arrays, and its hidden states are written
  for (int e = tid; e < kMicroMaxB * KP; e += kMicroThreads) m.act[e] = 0.f;
  const bool vec = (BI & 3) == 0 && aligned16_dev(in);
  for (int t0 = 0; t0 < T; t0 += a.C) {
    const int c = min(a.C, T - t0), n = c * BI;
    if (t0 > 0) __syncthreads();  // the steps before have finished with sx
    if (vec) {
      Segs<1> s;
      s.src[0] = reinterpret_cast<const float4*>(in + (size_t)t0 * BI);
      s.end[0] = n >> 2;
      stage_segs<1, 8>(m.staged4, s, tid);
    } else {
      stage_scalar<8>(sx, in + (size_t)t0 * BI, n, tid);
    }
    __syncthreads();
    if (t0 == 0 && cell) m.act[(tid / H) * KP + Il + tid % H] = h0v;
    if (xo >= 0) m.act[xo] = sx[tid];
    lds_barrier();
    for (int tt = 0; tt < c; ++tt) {
      const int t = t0 + tt;
      float z[R];  // lane p keeps the sums of batch row p
#pragma unroll
      for (int j = 0; j < R; ++j) z[j] = 0.f;
#pragma unroll 1
      for (int bb = 0; bb < B; ++bb) {
        float acc[R];
#pragma unroll
        for (int j = 0; j < R; ++j) acc[j] = 0.f;
        const float4* ap = reinterpret_cast<const float4*>(m.act + bb * KP + p * KSL);
#pragma unroll
        for (int i = 0; i < KSL / 4; ++i) {
          const float4 v = ap[i];
#pragma unroll
          for (int j = 0; j < R; ++j) {
            acc[j] = fmaf(wv[j][4 * i], v.x, acc[j]);
            acc[j] = fmaf(wv[j][4 * i + 1], v.y, acc[j]);
            acc[j] = fmaf(wv[j][4 * i + 2], v.z, acc[j]);
            acc[j] = fmaf(wv[j][4 * i + 3], v.w, acc[j]);
          }
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
          const float sum = sum_lanes<8>(acc[j]);
          z[j] = p == bb ? sum : z[j];
        }
      }
#pragma unroll
      for (int j = 0; j < R; ++j) {
        const int r = rg * R + j;
        const float zz = z[j] + bias[j];
        const float g = r >= 3 * H ? tanhf_dev(zz) : sigmoidf_dev(zz);
        if (rows && p < B) m.gates[p * G + r] = g;
      }
      lds_barrier();
      if (cell) {
        const int bb = tid / H, u = tid % H;
        const float* const gp = m.gates + bb * G + u;
        const float gi = gp[0], gf = gp[H], go = gp[2 * H], gc = gp[3 * H];
        const float cn = gf * c_state + gi * gc;
        const float hn = go * tanhf_dev(cn);
        c_state = cn;
        m.act[bb * KP + Il + u] = hn;
        float* const rgp = res_l + ((size_t)t * B + bb) * G + u;
        rgp[0] = gi;
        rgp[H] = gf;
        rgp[2 * H] = go;
        rgp[3 * H] = gc;
        const size_t eo = (size_t)t * BH + tid;
        res_c[eo] = cn;
        res_h[eo] = hn;
        if (l == a.L - 1) a.y[eo] = hn;
        if (t == T - 1) {
          if (a.hT) a.hT[(size_t)l * BH + tid] = hn;
          if (a.cT) a.cT[(size_t)l * BH + tid] = cn;
        }
      }
      if (tt + 1 < c && xo >= 0) m.act[xo] = sx[(tt + 1) * BI + tid];
      lds_barrier();
    }
  }
}

template <int HH>
__global__ __launch_bounds__(kMicroThreads) void lstm_micro_fwd_kernel(const MicroFwdArgs a) {
  extern __shared__ float4 staged4[];
  __shared__ __align__(16) float act[kMicroMaxB * kMicroK];
  __shared__ __align__(16) float gates[kMicroMaxB * 4 * HH];
  const MicroLds m{act, gates, nullptr, staged4};
  for (int l = 0; l < a.L; ++l) {
    if ((l == 0 ? a.I : HH) + HH <= 64) micro_fwd_layer<HH, 64>(a, l, m);
    else micro_fwd_layer<HH, 96>(a, l, m);
  }
}

template <int H, int KP>
__device__ __forceinline__ void micro_bwd_layer(const MicroBwdArgs& a, const int l, const MicroLds& m) {
  using S = RowPart<H, KP>;
  constexpr int G = S::G, R = S::R, KSL = S::KSL;
  // second layout: thread (q, rs) = (tid / TQ, tid % TQ) has column q and rows rs RSL .. rs RSL + RSL - 1
  constexpr int KQ = KP == 64 ? 64 : 128, TQ = kMicroThreads / KQ, RSL = G / TQ;
  static_assert(RSL % 4 == 0 && (TQ == 4 || TQ == 8), "a slice of rows is read four at a time");
  float* const staged = reinterpret_cast<float*>(m.staged4);
  const int tid = threadIdx.x, rg = tid >> 3, p = tid & 7;
  const bool rows = rg < S::NRG;
  const int q = tid / TQ, rs = tid % TQ;
  const int T = a.T, B = a.B;
  const int BH = B * H, BG = B * G;
  const size_t TB = (size_t)T * B;
  const int Il = l == 0 ? a.I : H, K = Il + H, BI = B * Il;
  const size_t woff = l == 0 ? 0 : (size_t)G * a.I + (size_t)(l - 1) * G * H;
  const float* Wl = a.W + woff;
  const float* Rl = a.R + (size_t)l * G * H;
  const float* const res_l = a.res + (size_t)l * TB * 6 * H;
  const float* const res_c = res_l + TB * 4 * H;
  const float* const res_h = res_l + TB * 5 * H;
  const float* const in = l == 0 ? a.x : a.res + (size_t)(l - 1) * TB * 6 * H + TB * 5 * H;
  const float* const dout = l == a.L - 1 ? a.dy : a.hand + (size_t)((l + 1) & 1) * TB * H;
  float* const dxo = l > 0 ? a.hand + (size_t)(l & 1) * TB * H : a.dx;  // layer 0: the caller's, or null
  float wt[RSL];
#pragma unroll
  for (int i = 0; i < RSL; ++i) {
    const int row = rs * RSL + i;
    wt[i] = q < Il ? Wl[row * Il + q] : (q < K ? Rl[row * H + (q - Il)] : 0.f);
  }
  float gw[R][KSL], gb[R];
#pragma unroll
  for (int j = 0; j < R; ++j) {
    gb[j] = 0.f;
#pragma unroll
    for (int i = 0; i < KSL; ++i) gw[j][i] = 0.f;
  }
  const bool cell = tid < BH;
  float dc = (cell && a.dcT) ? a.dcT[(size_t)l * BH + tid] : 0.f;
  const float dhv = (cell && a.dhT) ? a.dhT[(size_t)l * BH + tid] : 0.f;
  const int xo = tid < BI ? (tid / Il) * KP + tid % Il : -1;
  // The top layer's weights, states and first staged steps are all requested before anything waits: one trip.
  if (l < a.L - 1) __syncthreads();  // the layer above has finished with the LDS arrays, and has written `hand`
  for (int e = tid; e < kMicroMaxB * KP; e += kMicroThreads) m.act[e] = 0.f;
  const bool vec = (BI & 3) == 0 && aligned16_dev(in);
  for (int t1 = T; t1 > 0;) {
    const int t0 = max(0, t1 - a.C), c = t1 - t0;
    // staged steps t0 .. t1 - 1, in floats: gates [c][B][4H] | c_{t0-1 ..} [c+1][B][H] | h_{t0-1 ..} [c][B][H] |
    // incoming gradients [c][B][H] | inputs [c][B][I_l]
    const int oc = c * BG, oh = oc + (c + 1) * BH, od = oh + c * BH, ox = od + c * BH;
    Segs<7> s;
    s.src[0] = reinterpret_cast<const float4*>(res_l + (size_t)t0 * BG);
    s.end[0] = oc >> 2;
    s.src[1] = reinterpret_cast<const float4*>(t0 > 0 ? res_c + (size_t)(t0 - 1) * BH : (a.c0 ? a.c0 + (size_t)l * BH : nullptr));
    s.end[1] = s.end[0] + (BH >> 2);
    s.src[2] = reinterpret_cast<const float4*>(res_c + (size_t)t0 * BH);
    s.end[2] = oh >> 2;
    s.src[3] = reinterpret_cast<const float4*>(t0 > 0 ? res_h + (size_t)(t0 - 1) * BH : (a.h0 ? a.h0 + (size_t)l * BH : nullptr));
    s.end[3] = s.end[2] + (BH >> 2);
    s.src[4] = reinterpret_cast<const float4*>(res_h + (size_t)t0 * BH);
    s.end[4] = od >> 2;
    s.src[5] = reinterpret_cast<const float4*>(dout + (size_t)t0 * BH);
    s.end[5] = ox >> 2;
    s.src[6] = reinterpret_cast<const float4*>(in + (size_t)t0 * BI);
    s.end[6] = s.end[5] + (vec ? (c * BI) >> 2 : 0);
    if (t1 < T) __syncthreads();  // the steps before have finished with the staged arrays
    stage_segs<7, 8>(m.staged4, s, tid);
    if (!vec) stage_scalar<8>(staged + ox, in + (size_t)t0 * BI, c * BI, tid);
    __syncthreads();
    if (t1 == T && cell) m.dhs[tid] = dhv;  // read back by this thread only, in the point-wise stage below
    for (int tt = c - 1; tt >= 0; --tt) {
      const int t = t0 + tt;
      // ---- point-wise stage: gate gradients of step t; [x_t | h_{t-1}] for the weight gradients
      if (cell) {
        const int bb = tid / H, u = tid % H;
        const float* const gp = staged + (tt * B + bb) * G + u;
        const float gi = gp[0], gf = gp[H], go = gp[2 * H], gc = gp[3 * H];
        const float ct = staged[oc + (tt + 1) * BH + tid], cp = staged[oc + tt * BH + tid];
        const float dh = staged[od + tt * BH + tid] + m.dhs[tid];
        const float tc = tanhf_dev(ct);
        const float dcv = dc + dh * go * (1.f - tc * tc);
        float* const dA = m.gates + bb * G + u;
        dA[0] = dcv * gc * gi * (1.f - gi);
        dA[H] = dcv * cp * gf * (1.f - gf);
        dA[2 * H] = dh * tc * go * (1.f - go);
        dA[3 * H] = dcv * gi * (1.f - gc * gc);
        dc = dcv * gf;
        m.act[bb * KP + Il + u] = staged[oh + tt * BH + tid];
      }
      if (xo >= 0) m.act[xo] = staged[ox + tt * BI + tid];
      lds_barrier();
      // ---- dx_t (columns of W_l) and dh_{t-1} (columns of R_l): lane rs writes batch rows rs, rs + TQ
#pragma unroll 1
      for (int bb = 0; bb < B; ++bb) {
        float acc = 0.f;
        const float4* dp = reinterpret_cast<const float4*>(m.gates + bb * G + rs * RSL);
#pragma unroll
        for (int i = 0; i < RSL / 4; ++i) {
          const float4 v = dp[i];
          acc = fmaf(wt[4 * i], v.x, acc);
          acc = fmaf(wt[4 * i + 1], v.y, acc);
          acc = fmaf(wt[4 * i + 2], v.z, acc);
          acc = fmaf(wt[4 * i + 3], v.w, acc);
        }
        const float v = sum_lanes<TQ>(acc);
        // (dhs is read by the point-wise stage of the next step only: the barrier below orders the two)
        if ((bb & (TQ - 1)) == rs && q < K) {
          if (q >= Il) m.dhs[bb * H + (q - Il)] = v;
          else if (dxo) dxo[((size_t)t * B + bb) * Il + q] = v;
        }
      }
      // ---- weight and bias gradients of the thread's rows
#pragma unroll 1
      for (int bb = 0; bb < B; ++bb) {
        {
          float d[R];
#pragma unroll
          for (int j = 0; j < R; ++j) {
            d[j] = rows ? m.gates[bb * G + rg * R + j] : 0.f;
            gb[j] += d[j];
          }
          const float4* ap = reinterpret_cast<const float4*>(m.act + bb * KP + p * KSL);
#pragma unroll
          for (int i = 0; i < KSL / 4; ++i) {
            const float4 v = ap[i];
#pragma unroll
            for (int j = 0; j < R; ++j) {
              gw[j][4 * i] = fmaf(d[j], v.x, gw[j][4 * i]);
              gw[j][4 * i + 1] = fmaf(d[j], v.y, gw[j][4 * i + 1]);
              gw[j][4 * i + 2] = fmaf(d[j], v.z, gw[j][4 * i + 2]);
              gw[j][4 * i + 3] = fmaf(d[j], v.w, gw[j][4 * i + 3]);
            }
          }
        }
      }
      lds_barrier();
    }
    t1 = t0;
  }
  if (cell) {
    if (a.dh0) a.dh0[(size_t)l * BH + tid] = m.dhs[tid];
    if (a.dc0) a.dc0[(size_t)l * BH + tid] = dc;
  }
  if (rows) {
    float* const dWl = a.dW + woff;
    float* const dRl = a.dR + (size_t)l * G * H;
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int r = rg * R + j;
#pragma unroll
      for (int i = 0; i < KSL; ++i) {
        const int k = p * KSL + i;
        if (k < Il) dWl[r * Il + k] = gw[j][i];
        else if (k < K) dRl[r * H + (k - Il)] = gw[j][i];
      }
      if (p == 0) a.db[(size_t)l * G + r] = gb[j];
    }
  }
}

template <int HH>
__global__ __launch_bounds__(kMicroThreads) void lstm_micro_bwd_kernel(const MicroBwdArgs a) {
  extern __shared__ float4 staged4[];
  __shared__ __align__(16) float act[kMicroMaxB * kMicroK];
  __shared__ __align__(16) float gates[kMicroMaxB * 4 * HH];
  __shared__ float dhs[kMicroMaxB * HH];
  const MicroLds m{act, gates, dhs, staged4};
  for (int l = a.L - 1; l >= 0; --l) {
    if ((l == 0 ? a.I : HH) + HH <= 64) micro_bwd_layer<HH, 64>(a, l, m);
    else micro_bwd_layer<HH, 96>(a, l, m);
  }
}

// Steps staged at a time: as many as fit into kMicroStaged floats of LDS.
int fwd_chunk(const Dims& d) { return std::min(d.T, kMicroStaged / (d.B * std::max(d.I, d.H))); }
int bwd_step_floats(const Dims& d) { return d.B * (4 * d.H + 3 * d.H + std::max(d.I, d.H)); }
int bwd_chunk(const Dims& d) { return std::min(d.T, (kMicroStaged - d.B * d.H) / bwd_step_floats(d)); }

template <int HH>
hipError_t launch_fwd_t(const MicroFwdArgs& a, size_t lds, hipStream_t s) {
  static bool attr_set = false;
  const void* fn = reinterpret_cast<const void*>(&lstm_micro_fwd_kernel<HH>);
  if (hipError_t e = allow_dynamic_lds(fn, kMicroStaged * sizeof(float), attr_set); e != hipSuccess) return e;
  hipLaunchKernelGGL(lstm_micro_fwd_kernel<HH>, dim3(1), dim3(kMicroThreads), lds, s, a);
  return hipGetLastError();
}

template <int HH>
hipError_t launch_bwd_t(const MicroBwdArgs& a, size_t lds, hipStream_t s) {
  static bool attr_set = false;
  const void* fn = reinterpret_cast<const void*>(&lstm_micro_bwd_kernel<HH>);
  if (hipError_t e = allow_dynamic_lds(fn, kMicroStaged * sizeof(float), attr_set); e != hipSuccess) return e;
  hipLaunchKernelGGL(lstm_micro_bwd_kernel<HH>, dim3(1), dim3(kMicroThreads), lds, s, a);
  return hipGetLastError();
}

}  // namespace

// Shapes that run as one workgroup per pass.  The kernels take H = 8 / 16 / 32 with I <= 64 and B <= 8 (LSTM_MICRO=2:
// all of those); by default only where they were measured faster than the persistent kernels on the hidden size
// padded to 128.  Those overlap the layers and cost about 6.6 us per step, forward and backward together, for up to
// four layers; here the layers run one after the other at about 1.1 + 0.34 B us per layer and step:
// L (3 + B) <= 20 is where the two meet.  LSTM_MICRO=0 keeps every shape on the other kernels.
bool micro_shape(const Dims& d) {
  const int level = knobs().micro;
  if (level == 0 || !(d.H == 8 || d.H == 16 || d.H == 32) || d.I > kMicroMaxI || d.B > kMicroMaxB) return false;
  return level == 2 || d.L * (3 + d.B) <= 20;
}

hipError_t launch_micro_forward(const FwdArgs& f) {
  const Dims& d = f.d;
  if (!micro_shape(d)) return hipErrorInvalidValue;
  const int C = fwd_chunk(d);
  MicroFwdArgs a{f.x, f.h0, f.c0, f.W, f.R, f.b, f.y, f.hT, f.cT, f.reserve, d.L, d.T, d.B, d.I, C};
  const size_t lds = ((size_t)C * d.B * std::max(d.I, d.H) * sizeof(float) + 15) & ~(size_t)15;
  double fl = 0.0;
  for (int l = 0; l < d.L; ++l) fl += 2.0 * 4 * d.H * ((l == 0 ? d.I : d.H) + d.H) * d.B * d.T;
  prof_flops(fl, "lstm_micro_fwd_kernel");
  switch (d.H) {
    case 8: return launch_fwd_t<8>(a, lds, f.stream);
    case 16: return launch_fwd_t<16>(a, lds, f.stream);
    case 32: return launch_fwd_t<32>(a, lds, f.stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_micro_backward(const BwdArgs& g) {
  const Dims& d = g.d;
  if (!micro_shape(d)) return hipErrorInvalidValue;
  const int C = bwd_chunk(d);
  MicroBwdArgs a{g.x, g.h0, g.c0, g.W, g.R, g.reserve, g.dy, g.dhT, g.dcT, g.dx, g.dh0, g.dc0, g.dW, g.dR, g.db,
                 reinterpret_cast<float*>(g.ws + g.w.dx), d.L, d.T, d.B, d.I, C};
  const size_t lds = ((size_t)C * bwd_step_floats(d) + (size_t)d.B * d.H) * sizeof(float);
  double fl = 0.0;
  for (int l = 0; l < d.L; ++l) fl += 2.0 * 2.0 * 4 * d.H * ((l == 0 ? d.I : d.H) + d.H) * d.B * d.T;
  prof_flops(fl, "lstm_micro_bwd_kernel");
  switch (d.H) {
    case 8: return launch_bwd_t<8>(a, lds, g.stream);
    case 16: return launch_bwd_t<16>(a, lds, g.stream);
    case 32: return launch_bwd_t<32>(a, lds, g.stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace lstm
