// A whole pass in one workgroup: lstm_micro_fwd_kernel / lstm_micro_bwd_kernel, for networks so small that a launch
// per step costs more than the step (H = 8 / 16 / 32, I <= 64, B <= 8: a step is a few thousand multiply-adds,
// a launch a few microseconds).  Section 3.1 of arXiv 1604.01946 names the two extremes: one large product per
// step at the top of the range, launch overhead at the bottom.  Here one launch runs all layers and steps of a pass
// (the backward one the weight gradients of Section 2.6 as well); the weights of the layer at hand live in the
// registers of the workgroup's 256 threads, the step's vectors in LDS, two barriers per step.
//
// A step is shorter than one trip to memory, so nothing inside the loop over the steps waits for memory: what the
// steps read (inputs; in the backward pass the gates, cell states, hidden states and incoming gradients as well) is
// brought into LDS for as many steps at a time as fit, in one batch of requests, and what they write is stored and
// not waited for (the barriers inside the loop order LDS only).
//
// Forward.  Thread (row r, part p): r = one of the 4H stacked gate rows, p = one of TPR = 256 / 4H slices of the
// K = I_l + H columns (padded to 96): the slice of [W_l | R_l] row r stays in registers for all T steps, the products
// with [x_t | h_{t-1}] are added up over the slice and then over the TPR neighbouring lanes.  Cells: one or two per thread.
//
// Backward.  The same (row, part) layout accumulates dW_l, dR_l (one register per weight) and db_l over the steps;
// for dh_{t-1} and dx_t a second layout holds the transposed slice: thread (column q of [W_l | R_l], half pc of the
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

template <int N>
__device__ __forceinline__ float sum_lanes(float v) {  // over N neighbouring lanes (N a power of two <= 8), fixed order
  if (N > 1) v += __shfl_xor(v, 1);
  if (N > 2) v += __shfl_xor(v, 2);
  if (N > 4) v += __shfl_xor(v, 4);
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
  for (int base = 0; base < total; base += 256 * U) {
    float4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = base + u * 256 + tid;
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
      const int idx = base + u * 256 + tid;
      if (idx < total) dst[idx] = v[u];
    }
  }
}

template <int U>
__device__ __forceinline__ void stage_scalar(float* dst, const float* src, int n, int tid) {
  for (int base = 0; base < n; base += 256 * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = base + u * 256 + tid;
      v[u] = idx < n ? src[idx] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = base + u * 256 + tid;
      if (idx < n) dst[idx] = v[u];
    }
  }
}

template <int HH>
__global__ __launch_bounds__(256) void lstm_micro_fwd_kernel(const MicroFwdArgs a) {
  constexpr int H = HH, G = 4 * H, TPR = 256 / G, KS = kMicroK / TPR;
  static_assert(KS % 4 == 0 && KS * TPR == kMicroK, "a thread's slice is read four columns at a time");
  extern __shared__ float4 staged4[];
  float* const sx = reinterpret_cast<float*>(staged4);   // [C][B][I_l]: inputs of the staged steps
  __shared__ __align__(16) float act[kMicroMaxB][kMicroK];  // [x_t | h_{t-1} | 0] per batch row
  __shared__ float pre[kMicroMaxB][G];                      // gate pre-activations
  float* const actf = &act[0][0];
  const int tid = threadIdx.x, r = tid / TPR, p = tid % TPR;
  const int T = a.T, B = a.B;
  const size_t TB = (size_t)T * B;
  for (int l = 0; l < a.L; ++l) {
    const int Il = l == 0 ? a.I : H, K = Il + H, BI = B * Il;
    const float* Wl = a.W + (l == 0 ? 0 : (size_t)G * a.I + (size_t)(l - 1) * G * H);
    const float* Rl = a.R + (size_t)l * G * H;
    float* const res_l = a.res + (size_t)l * TB * 6 * H;
    float* const res_c = res_l + TB * 4 * H;
    float* const res_h = res_l + TB * 5 * H;
    const float* const in = l == 0 ? a.x : a.res + (size_t)(l - 1) * TB * 6 * H + TB * 5 * H;
    float wv[KS];
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      const int k = p * KS + i;
      wv[i] = k < Il ? Wl[(size_t)r * Il + k] : (k < K ? Rl[(size_t)r * H + (k - Il)] : 0.f);
    }
    const float bias = a.b[(size_t)l * G + r];
    float c_state[2];
    int xo[2];  // where this thread's one or two elements of x_t go in act (-1: none)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int e = tid + 256 * j;
      c_state[j] = (e < B * H && a.c0) ? a.c0[(size_t)l * B * H + e] : 0.f;
      xo[j] = e < BI ? (e / Il) * kMicroK + e % Il : -1;
    }
    __syncthreads();  // the layer before has finished with the LDS arrays, and its hidden states are written
    for (int e = tid; e < kMicroMaxB * kMicroK; e += 256) actf[e] = 0.f;
    __syncthreads();
    for (int e = tid; e < B * H; e += 256) act[e / H][Il + e % H] = a.h0 ? a.h0[(size_t)l * B * H + e] : 0.f;
    const bool vec = (BI & 3) == 0 && aligned16_dev(in);
    for (int t0 = 0; t0 < T; t0 += a.C) {
      const int c = min(a.C, T - t0), n = c * BI;
      __syncthreads();  // the steps before have finished with sx
      if (vec) {
        Segs<1> s;
        s.src[0] = reinterpret_cast<const float4*>(in + (size_t)t0 * BI);
        s.end[0] = n >> 2;
        stage_segs<1, 8>(staged4, s, tid);
      } else {
        stage_scalar<8>(sx, in + (size_t)t0 * BI, n, tid);
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (xo[j] >= 0) actf[xo[j]] = sx[tid + 256 * j];
      lds_barrier();
      for (int tt = 0; tt < c; ++tt) {
        const int t = t0 + tt;
        float acc[kMicroMaxB];
#pragma unroll
        for (int bb = 0; bb < kMicroMaxB; ++bb) {
          acc[bb] = 0.f;
          if (bb < B) {
            const float4* ap = reinterpret_cast<const float4*>(&act[bb][p * KS]);
#pragma unroll
            for (int i = 0; i < KS / 4; ++i) {
              const float4 v = ap[i];
              acc[bb] = fmaf(wv[4 * i], v.x, acc[bb]);
              acc[bb] = fmaf(wv[4 * i + 1], v.y, acc[bb]);
              acc[bb] = fmaf(wv[4 * i + 2], v.z, acc[bb]);
              acc[bb] = fmaf(wv[4 * i + 3], v.w, acc[bb]);
            }
          }
        }
#pragma unroll
        for (int bb = 0; bb < kMicroMaxB; ++bb) {
          const float v = sum_lanes<TPR>(acc[bb]);
          if (p == 0 && bb < B) pre[bb][r] = v + bias;
        }
        lds_barrier();
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int e = tid + 256 * j;
          if (e < B * H) {
            const int bb = e / H, u = e % H;
            const float gi = sigmoidf_dev(pre[bb][u]), gf = sigmoidf_dev(pre[bb][H + u]);
            const float go = sigmoidf_dev(pre[bb][2 * H + u]), gc = tanhf_dev(pre[bb][3 * H + u]);
            const float cn = gf * c_state[j] + gi * gc;
            const float hn = go * tanhf_dev(cn);
            c_state[j] = cn;
            act[bb][Il + u] = hn;
            float* const rg = res_l + ((size_t)t * B + bb) * G + u;
            rg[0] = gi;
            rg[H] = gf;
            rg[2 * H] = go;
            rg[3 * H] = gc;
            const size_t eo = ((size_t)t * B + bb) * H + u;
            res_c[eo] = cn;
            res_h[eo] = hn;
            if (l == a.L - 1) a.y[eo] = hn;
            if (t == T - 1) {
              if (a.hT) a.hT[(size_t)l * B * H + e] = hn;
              if (a.cT) a.cT[(size_t)l * B * H + e] = cn;
            }
          }
        }
        if (tt + 1 < c) {
#pragma unroll
          for (int j = 0; j < 2; ++j)
            if (xo[j] >= 0) actf[xo[j]] = sx[(tt + 1) * BI + tid + 256 * j];
        }
        lds_barrier();
      }
    }
  }
}

template <int HH>
__global__ __launch_bounds__(256) void lstm_micro_bwd_kernel(const MicroBwdArgs a) {
  constexpr int H = HH, G = 4 * H, TPR = 256 / G, KS = kMicroK / TPR;
  constexpr int TPC = 2, RS = G / TPC;  // columns padded to 128: two threads per column, half the rows each
  static_assert(KS % 4 == 0 && RS % 4 == 0 && kMicroK <= 256 / TPC, "slices are read four elements at a time");
  extern __shared__ float4 staged4[];
  float* const staged = reinterpret_cast<float*>(staged4);
  __shared__ __align__(16) float act[kMicroMaxB][kMicroK];  // [x_t | h_{t-1} | 0]
  __shared__ __align__(16) float dAs[kMicroMaxB][G];        // gate gradients of step t
  __shared__ float dhs[kMicroMaxB][H];                      // dh_{t-1} from the recurrent product
  float* const actf = &act[0][0];
  const int tid = threadIdx.x, r = tid / TPR, p = tid % TPR;
  const int q = tid / TPC, pc = tid % TPC;
  const int T = a.T, B = a.B;
  const int BH = B * H, BG = B * G;
  const size_t TB = (size_t)T * B;
  for (int l = a.L - 1; l >= 0; --l) {
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
    // transposed slice: column q of [W_l | R_l], rows pc RS ... pc RS + RS - 1
    float wt[RS];
#pragma unroll
    for (int i = 0; i < RS; ++i) {
      const int row = pc * RS + i;
      wt[i] = q < Il ? Wl[(size_t)row * Il + q] : (q < K ? Rl[(size_t)row * H + (q - Il)] : 0.f);
    }
    float gw[KS];  // gradient of the slice of row r
#pragma unroll
    for (int i = 0; i < KS; ++i) gw[i] = 0.f;
    float gb = 0.f;
    float dc[2];
    int xo[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int e = tid + 256 * j;
      dc[j] = (e < BH && a.dcT) ? a.dcT[(size_t)l * BH + e] : 0.f;
      xo[j] = e < BI ? (e / Il) * kMicroK + e % Il : -1;
    }
    __syncthreads();  // the layer above has finished with the LDS arrays
    for (int e = tid; e < kMicroMaxB * kMicroK; e += 256) actf[e] = 0.f;
    for (int e = tid; e < BH; e += 256) dhs[e / H][e % H] = a.dhT ? a.dhT[(size_t)l * BH + e] : 0.f;
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
      __syncthreads();  // the steps before have finished with the staged arrays; the layer above has written `hand`
      stage_segs<7, 8>(staged4, s, tid);
      if (!vec) stage_scalar<8>(staged + ox, in + (size_t)t0 * BI, c * BI, tid);
      __syncthreads();
      for (int tt = c - 1; tt >= 0; --tt) {
        const int t = t0 + tt;
        // ---- point-wise stage: gate gradients of step t; [x_t | h_{t-1}] for the weight gradients
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int e = tid + 256 * j;
          if (e < BH) {
            const int bb = e / H, u = e % H;
            const float* const rg = staged + (tt * B + bb) * G + u;
            const float gi = rg[0], gf = rg[H], go = rg[2 * H], gc = rg[3 * H];
            const float ct = staged[oc + (tt + 1) * BH + e], cp = staged[oc + tt * BH + e];
            const float dh = staged[od + tt * BH + e] + dhs[bb][u];
            const float tc = tanhf_dev(ct);
            const float dcv = dc[j] + dh * go * (1.f - tc * tc);
            dAs[bb][u] = dcv * gc * gi * (1.f - gi);
            dAs[bb][H + u] = dcv * cp * gf * (1.f - gf);
            dAs[bb][2 * H + u] = dh * tc * go * (1.f - go);
            dAs[bb][3 * H + u] = dcv * gi * (1.f - gc * gc);
            dc[j] = dcv * gf;
            act[bb][Il + u] = staged[oh + tt * BH + e];
          }
          if (xo[j] >= 0) actf[xo[j]] = staged[ox + tt * BI + e];
        }
        lds_barrier();
        // ---- dx_t (columns of W_l) and dh_{t-1} (columns of R_l)
        {
          float out[kMicroMaxB];
#pragma unroll
          for (int bb = 0; bb < kMicroMaxB; ++bb) {
            float acc = 0.f;
            if (bb < B) {
              const float4* dp = reinterpret_cast<const float4*>(&dAs[bb][pc * RS]);
#pragma unroll
              for (int i = 0; i < RS / 4; ++i) {
                const float4 v = dp[i];
                acc = fmaf(wt[4 * i], v.x, acc);
                acc = fmaf(wt[4 * i + 1], v.y, acc);
                acc = fmaf(wt[4 * i + 2], v.z, acc);
                acc = fmaf(wt[4 * i + 3], v.w, acc);
              }
            }
            out[bb] = sum_lanes<TPC>(acc);
          }
          // (dhs is read by the point-wise stage of the next step only: the barrier below orders the two)
          if (pc == 0 && q < K) {
#pragma unroll
            for (int bb = 0; bb < kMicroMaxB; ++bb)
              if (bb < B) {
                if (q >= Il) dhs[bb][q - Il] = out[bb];
                else if (dxo) dxo[((size_t)t * B + bb) * Il + q] = out[bb];
              }
          }
        }
        // ---- weight and bias gradients of row r
#pragma unroll
        for (int bb = 0; bb < kMicroMaxB; ++bb)
          if (bb < B) {
            const float d = dAs[bb][r];
            const float4* ap = reinterpret_cast<const float4*>(&act[bb][p * KS]);
#pragma unroll
            for (int i = 0; i < KS / 4; ++i) {
              const float4 v = ap[i];
              gw[4 * i] = fmaf(d, v.x, gw[4 * i]);
              gw[4 * i + 1] = fmaf(d, v.y, gw[4 * i + 1]);
              gw[4 * i + 2] = fmaf(d, v.z, gw[4 * i + 2]);
              gw[4 * i + 3] = fmaf(d, v.w, gw[4 * i + 3]);
            }
            if (p == 0) gb += d;
          }
        lds_barrier();
      }
      t1 = t0;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int e = tid + 256 * j;
      if (e < BH) {
        if (a.dh0) a.dh0[(size_t)l * BH + e] = dhs[e / H][e % H];
        if (a.dc0) a.dc0[(size_t)l * BH + e] = dc[j];
      }
    }
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      const int k = p * KS + i;
      if (k < Il) a.dW[woff + (size_t)r * Il + k] = gw[i];
      else if (k < K) a.dR[(size_t)l * G * H + (size_t)r * H + (k - Il)] = gw[i];
    }
    if (p == 0) a.db[(size_t)l * G + r] = gb;
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
  hipLaunchKernelGGL(lstm_micro_fwd_kernel<HH>, dim3(1), dim3(256), lds, s, a);
  return hipGetLastError();
}

template <int HH>
hipError_t launch_bwd_t(const MicroBwdArgs& a, size_t lds, hipStream_t s) {
  static bool attr_set = false;
  const void* fn = reinterpret_cast<const void*>(&lstm_micro_bwd_kernel<HH>);
  if (hipError_t e = allow_dynamic_lds(fn, kMicroStaged * sizeof(float), attr_set); e != hipSuccess) return e;
  hipLaunchKernelGGL(lstm_micro_bwd_kernel<HH>, dim3(1), dim3(256), lds, s, a);
  return hipGetLastError();
}

}  // namespace

// Shapes that run as one workgroup per pass.  The kernels take H = 8 / 16 / 32 with I <= 64 and B <= 8 (LSTM_MICRO=2:
// all of those); by default only where they were measured faster than the other kernels: one layer (the layers run one
// after the other here, while the persistent kernels, on the hidden size padded to 128, overlap them).
// LSTM_MICRO=0 keeps every shape on the other kernels.
bool micro_shape(const Dims& d) {
  const int level = knobs().micro;
  if (level == 0 || !(d.H == 8 || d.H == 16 || d.H == 32) || d.I > kMicroMaxI || d.B > kMicroMaxB) return false;
  return level == 2 || d.L == 1;
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
