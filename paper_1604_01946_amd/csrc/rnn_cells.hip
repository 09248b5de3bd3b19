// Single-gate RNN (ReLU / tanh) and GRU on the cell-independent rungs of the ladder of
// arXiv 1604.01946: input products batched over time (Section 2.3), the gates of a step grouped into
// one recurrent product (Section 2.1; the GRU's three), one fused point-wise kernel per step
// (Section 2.2.2), weight gradients as large products after propagation (Section 2.6).
#include "../../include/lstm.h"
#include "../../include/rnn.h"
#include "schedule.h"
#include "knobs.h"
#include <algorithm>

namespace lstm {

// persistent.hip: the wide persistent kernels also run the GRU (weights on chip for all T steps, Section 4)
bool gru_persistent_supported(const Dims& d);
int run_forward_persistent(const FwdArgs& a, int cell);
int run_backward_persistent(const BwdArgs& a, int cell, bool* bias_done, LayerGradients* lg);

#define CK(expr, what)                                             \
  do {                                                             \
    if (record((expr), what) != hipSuccess) return LSTM_HIP_ERROR; \
  } while (0)

namespace {

inline int gates_of(int cell) { return cell == RNN_CELL_GRU ? 3 : ((cell == RNN_CELL_RELU || cell == RNN_CELL_TANH) ? 1 : 0); }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Forward point-wise stage of one step: P = W x_t (without bias), Q = R h_{t-1}, both [B][G].
// GRU saves r, z, n and Q_n for the backward pass (sv: [B][4H]).
__global__ void cell_fwd_kernel(int cell, const float* __restrict__ P, const float* __restrict__ Q,
                                const float* __restrict__ bias, const float* __restrict__ hp, float* __restrict__ h,
                                float* __restrict__ y, float* __restrict__ sv, int B, int H) {
  const long cnt = (long)B * H;
  const int G = (cell == RNN_CELL_GRU ? 3 : 1) * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < cnt; e += (long)gridDim.x * blockDim.x) {
    const int u = (int)(e % H);
    const long row = e / H;
    const float* p = P + row * G;
    const float* q = Q + row * G;
    float out;
    if (cell == RNN_CELL_GRU) {
      const float r = sigmoidf_dev(p[u] + bias[u] + q[u]);
      const float z = sigmoidf_dev(p[H + u] + bias[H + u] + q[H + u]);
      const float qn = q[2 * H + u];
      const float n = tanhf_dev(p[2 * H + u] + bias[2 * H + u] + r * qn);
      out = (1.f - z) * n + z * (hp ? hp[e] : 0.f);
      float* s4 = sv + row * 4 * H;
      s4[u] = r; s4[H + u] = z; s4[2 * H + u] = n; s4[3 * H + u] = qn;
    } else {
      const float a = p[u] + bias[u] + q[u];
      out = cell == RNN_CELL_TANH ? tanhf_dev(a) : fmaxf(a, 0.f);
    }
    h[e] = out;
    if (y) y[e] = out;
  }
}

// Backward point-wise stage of one step: dh = dout + carry; writes the gradients with respect to
// W x + b (da, [B][G]) and to R h_{t-1} (dq, [B][G]; the same array for the single-gate cells) and the
// part of dh_{t-1} that does not pass through R (direct, [B][H]; zero for the single-gate cells).
__global__ void cell_bwd_kernel(int cell, const float* __restrict__ dout, const float* __restrict__ carry,
                                const float* __restrict__ h, const float* __restrict__ hp, const float* __restrict__ sv,
                                float* __restrict__ da, float* __restrict__ dq, float* __restrict__ direct, int B, int H) {
  const long cnt = (long)B * H;
  const int G = (cell == RNN_CELL_GRU ? 3 : 1) * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < cnt; e += (long)gridDim.x * blockDim.x) {
    const int u = (int)(e % H);
    const long row = e / H;
    const float dh = dout[e] + (carry ? carry[e] : 0.f);
    if (cell == RNN_CELL_GRU) {
      const float* s4 = sv + row * 4 * H;
      const float r = s4[u], z = s4[H + u], n = s4[2 * H + u], qn = s4[3 * H + u];
      const float hprev = hp ? hp[e] : 0.f;
      const float dn_pre = dh * (1.f - z) * (1.f - n * n);
      const float daz = dh * (hprev - n) * z * (1.f - z);
      const float dar = dn_pre * qn * r * (1.f - r);
      float* a3 = da + row * G;
      float* q3 = dq + row * G;
      a3[u] = dar; a3[H + u] = daz; a3[2 * H + u] = dn_pre;
      q3[u] = dar; q3[H + u] = daz; q3[2 * H + u] = dn_pre * r;
      direct[e] = dh * z;
    } else {
      const float hv = h[e];
      da[row * G + u] = dh * (cell == RNN_CELL_TANH ? (1.f - hv * hv) : (hv > 0.f ? 1.f : 0.f));
      direct[e] = 0.f;
    }
  }
}

struct RnnWs {
  size_t P, Q, da, dq, dx0, dx1, carry0, carry1, dbpart, total;
};

RnnWs rnn_ws(int cell, const Dims& d) {
  const size_t TB = (size_t)d.T * d.B, G = (size_t)gates_of(cell) * d.H, BH = (size_t)d.B * d.H;
  RnnWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  w.P = take(TB * G * 4);
  w.Q = take((size_t)d.B * G * 4);
  w.da = take(TB * G * 4);
  w.dq = take(TB * G * 4);
  w.dx0 = take(TB * d.H * 4);
  w.dx1 = take(TB * d.H * 4);
  w.carry0 = take(BH * 4);
  w.carry1 = take(BH * 4);
  w.dbpart = take(64 * G * 4);
  w.total = off;
  return w;
}

// reserve of layer l: hidden states [T][B][H], then (GRU) r, z, n, R_n h [T][B][4H]
inline size_t res_layer_floats(int cell, const Dims& d) {
  return (size_t)d.T * d.B * d.H * (cell == RNN_CELL_GRU ? 5 : 1);
}

// Shapes the persistent GRU kernels may take (device limits are checked at run time): their workspace is the LSTM
// library's, so the buffer must hold either layout.
inline bool gru_persistent_shape(int cell, const Dims& d) {
  if (gates_of(cell) == 0) return false;
  // one-layer kernels: up to the batch where the step-by-step path with its large products measured faster (the
  // single gate leaves three quarters of the persistent kernels' tiles empty, so its break-even comes earlier)
  const bool gru = cell == RNN_CELL_GRU;
  if (d.H == 1024) return d.B <= (gru ? 512 : 256);
  if (d.H == 2048) return d.B <= (gru ? 320 : 96);  // GRU: 105 TFLOP/s at any number of slices; step by step 99 at 256 rows, 105 at 384, 120 at 512
  // H <= 512: the rate on chip does not depend on the batch (slices of 64 rows, one after the other once the chip is
  // full), the step-by-step path gains with it; measured break-even (L = 4; TFLOP/s on chip / step by step at the
  // limit): GRU H = 512 92 / 92 at 2048 rows, H = 256 57 / 43 at 2048, H = 128 31 / 14 at 2048; single gate H = 512
  // 31 / 29 at 512 rows, H = 256 22 / 19 at 2048, H = 128 11 / 5.5 at 2048
  if (d.H == 512) return d.B <= (gru ? 2048 : 512);
  if (d.H == 256) return d.B <= (gru ? 4096 : 2048);
  return d.H == 128 && d.B <= 8192;
}
// cell selector of the templated persistent kernels
inline int kernel_cell(int cell) { return cell == RNN_CELL_GRU ? 1 : (cell == RNN_CELL_RELU ? 2 : 3); }
inline size_t ws_total(int cell, const Dims& d) {
  const size_t own = rnn_ws(cell, d).total;
  if (!gru_persistent_shape(cell, d)) return own;
  const size_t pers = ws_layout(d, true).total;
  return pers > own ? pers : own;
}
inline bool use_persistent(int cell, const Dims& d) {
  if (!gru_persistent_shape(cell, d) || !gru_persistent_supported(d)) return false;
  return !knobs().rnn_no_persistent;
}

inline int ew_grid(long cnt) { return (int)((cnt + 255) / 256 < 2048 ? (cnt + 255) / 256 : 2048); }

int forward_impl(int cell, const Dims& d, const float* x, const float* h0, const float* W, const float* R, const float* b,
                 float* y, float* hT, float* reserve, char* ws, hipStream_t s) {
  const int gates = gates_of(cell), H = d.H, B = d.B;
  const size_t TB = (size_t)d.T * B, G = (size_t)gates * H, BH = (size_t)B * H;
  if (use_persistent(cell, d)) {
    const FwdArgs a{d, x, h0, nullptr, W, R, b, y, hT, nullptr, reserve, ws, ws_layout(d, true), s};
    return run_forward_persistent(a, kernel_cell(cell));
  }
  const RnnWs w = rnn_ws(cell, d);
  float* P = reinterpret_cast<float*>(ws + w.P);
  float* Q = reinterpret_cast<float*>(ws + w.Q);
  size_t woff = 0;
  for (int l = 0; l < d.L; ++l) {
    const int Il = in_dim(d, l);
    float* hl = reserve + (size_t)l * res_layer_floats(cell, d);
    float* svl = hl + TB * H;
    const float* in = l == 0 ? x : reserve + (size_t)(l - 1) * res_layer_floats(cell, d);
    const float* Wl = W + woff;
    const float* Rl = R + (size_t)l * G * H;
    woff += G * Il;
    {  // Section 2.3: the layer's input products for all steps in one GEMM
      GemmProblem p{in, Wl, P, (int)TB, (int)G, Il, Il, 1, 1, Il, (long)G, 0};
      CK(launch_gemm_group(&p, 1, s), "input projection GEMM");
    }
    for (int t = 0; t < d.T; ++t) {
      const float* hp = t ? hl + (size_t)(t - 1) * BH : (h0 ? h0 + (size_t)l * BH : nullptr);
      float* ht = hl + (size_t)t * BH;
      if (hp) {  // Section 2.1: all gates of the step in one recurrent product
        GemmProblem p{hp, Rl, Q, B, (int)G, H, H, 1, 1, H, (long)G, 0};
        CK(launch_gemm_group(&p, 1, s), "recurrent GEMM");
      } else {
        CK(launch_fill_zero(Q, (size_t)B * G * 4, s), "zero recurrent term");
      }
      hipLaunchKernelGGL(cell_fwd_kernel, dim3(ew_grid((long)BH)), dim3(256), 0, s, cell, P + (size_t)t * B * G, Q,
                         b + (size_t)l * G, hp, ht, (l == d.L - 1) ? y + (size_t)t * BH : nullptr,
                         cell == RNN_CELL_GRU ? svl + (size_t)t * B * 4 * H : nullptr, B, H);
      CK(hipGetLastError(), "point-wise forward");
    }
    if (hT) CK(launch_ew(EW_COPY, hT + (size_t)l * BH, H, hl + (size_t)(d.T - 1) * BH, H, nullptr, 0, B, H, s), "copy hT");
  }
  return LSTM_OK;
}

// Backward on the persistent kernels: propagation in one launch (per group of batch slices), then the weight
// gradients as grouped products over all steps (Section 2.6) from the gate gradients it left in the workspace:
// [L][T*B][4H]; GRU: the gradients with respect to the r and z pre-activations, W_n x + b_n, and R_n h; single gate:
// the gradient of the pre-activation in the first H columns.
int backward_persistent(int cell, const Dims& d, const float* x, const float* h0, const float* W, const float* R,
                        const float* reserve, const float* dy, const float* dhT, float* dx, float* dh0, float* dW,
                        float* dR, float* db, char* ws, hipStream_t s) {
  const int H = d.H, B = d.B;
  const bool gru = cell == RNN_CELL_GRU;
  const size_t TB = (size_t)d.T * B, G = (size_t)gates_of(cell) * H, G4 = 4 * (size_t)H, BH = (size_t)B * H;
  const WsLayout w = ws_layout(d, true);
  const BwdArgs a{d, x, h0, nullptr, W, R, reserve, dy, dhT, nullptr, dx, dh0, nullptr, dW, dR, db, ws, w, s};
  const float* dA_all = reinterpret_cast<const float*>(ws + w.P);
  // The gradient products of layer l (Section 2.6: large products once the layer's propagation is complete) are
  // appended to two groups: the sums over steps, and the initial-state terms that accumulate onto them.
  auto add_layer = [&](int l, GemmProblem* main_g, int& nm, GemmProblem* init_g, int& ni, hipStream_t st) -> int {
    const int Il = in_dim(d, l);
    const float* dA = dA_all + (size_t)l * TB * G4;
    const float* hl = reserve + (size_t)l * res_layer_floats(cell, d);
    const float* in = l == 0 ? x : reserve + (size_t)(l - 1) * res_layer_floats(cell, d);
    float* dWl = dW + (l == 0 ? 0 : G * d.I + (size_t)(l - 1) * G * H);
    float* dRl = dR + (size_t)l * G * H;
    main_g[nm++] = GemmProblem{dA, in, dWl, (int)G, Il, (int)TB, 1, (long)G4, Il, 1, Il, 0};
    // dR: GRU rows r, z from the first two groups, rows n from the fourth (the gradient of R_n h); single gate: the first
    const int m1 = gru ? 2 * H : H;
    if (d.T > 1) {
      main_g[nm++] = GemmProblem{dA + (size_t)B * G4, hl, dRl, m1, H, (int)(TB - B), 1, (long)G4, H, 1, H, 0};
      if (gru)
        main_g[nm++] = GemmProblem{dA + (size_t)B * G4 + 3 * H, hl, dRl + (size_t)2 * H * H, H, H, (int)(TB - B), 1, (long)G4, H, 1, H, 0};
    }
    if (h0) {
      const int acc = d.T > 1 ? 1 : 0;
      init_g[ni++] = GemmProblem{dA, h0 + (size_t)l * BH, dRl, m1, H, B, 1, (long)G4, H, 1, H, acc};
      if (gru)
        init_g[ni++] = GemmProblem{dA + 3 * H, h0 + (size_t)l * BH, dRl + (size_t)2 * H * H, H, H, B, 1, (long)G4, H, 1, H, acc};
    } else if (d.T == 1) {
      CK(launch_fill_zero(dRl, G * H * 4, st), "zero dR");
    }
    return LSTM_OK;
  };
  auto flush = [&](GemmProblem* main_g, int& nm, GemmProblem* init_g, int& ni, hipStream_t st) -> int {
    if (nm) CK(launch_gemm_group(main_g, nm, st), "weight-gradient GEMMs");
    if (ni) CK(launch_gemm_group(init_g, ni, st), "weight-gradient GEMMs (initial state term)");
    nm = ni = 0;
    return LSTM_OK;
  };
  // One layer on a stream of the caller's choice: the one-layer kernels run it under the next layer's recurrence
  // where CUs are idle.
  auto layer_products = [&](int l, hipStream_t st) -> int {
    GemmProblem main_g[3], init_g[2];
    int nm = 0, ni = 0;
    const int rc = add_layer(l, main_g, nm, init_g, ni, st);
    return rc != LSTM_OK ? rc : flush(main_g, nm, init_g, ni, st);
  };
  using Fn = decltype(layer_products);
  LayerGradients lg{[](void* ctx, int l, hipStream_t st) { return (*static_cast<Fn*>(ctx))(l, st); }, &layer_products, false};
  bool bias_done = false;
  const int st = run_backward_persistent(a, kernel_cell(cell), &bias_done, &lg);
  if (st != LSTM_OK) return st;
  if (!lg.used) {  // all layers in grouped launches
    GemmProblem main_g[kMaxGemmGroup], init_g[kMaxGemmGroup];
    int nm = 0, ni = 0;
    for (int l = 0; l < d.L; ++l) {
      if (nm + 3 > kMaxGemmGroup || ni + 2 > kMaxGemmGroup) {
        const int rc = flush(main_g, nm, init_g, ni, s);
        if (rc != LSTM_OK) return rc;
      }
      const int rc = add_layer(l, main_g, nm, init_g, ni, s);
      if (rc != LSTM_OK) return rc;
    }
    const int rc = flush(main_g, nm, init_g, ni, s);
    if (rc != LSTM_OK) return rc;
  }
  if (!bias_done) {  // column sums over all four groups, of which db takes the leading ones
    float* part = reinterpret_cast<float*>(ws + w.dbpart);
    float* sums = reinterpret_cast<float*>(ws + w.scratch);
    for (int l = 0; l < d.L; ++l) {
      CK(launch_colsum(dA_all + (size_t)l * TB * G4, (int)TB, (int)G4, part, sums, s), "bias gradient");
      CK(launch_ew(EW_COPY, db + (size_t)l * G, (long)G, sums, (long)G4, nullptr, 0, 1, (int)G, s), "bias gradient");
    }
  }
  return LSTM_OK;
}

int backward_impl(int cell, const Dims& d, const float* x, const float* h0, const float* W, const float* R,
                  const float* reserve, const float* dy, const float* dhT, float* dx, float* dh0, float* dW, float* dR,
                  float* db, char* ws, hipStream_t s) {
  const int gates = gates_of(cell), H = d.H, B = d.B;
  const size_t TB = (size_t)d.T * B, G = (size_t)gates * H, BH = (size_t)B * H;
  if (use_persistent(cell, d)) return backward_persistent(cell, d, x, h0, W, R, reserve, dy, dhT, dx, dh0, dW, dR, db, ws, s);
  const RnnWs w = rnn_ws(cell, d);
  float* da = reinterpret_cast<float*>(ws + w.da);
  float* dq = cell == RNN_CELL_GRU ? reinterpret_cast<float*>(ws + w.dq) : da;
  float* dxb[2] = {reinterpret_cast<float*>(ws + w.dx0), reinterpret_cast<float*>(ws + w.dx1)};
  float* carry[2] = {reinterpret_cast<float*>(ws + w.carry0), reinterpret_cast<float*>(ws + w.carry1)};
  float* dbpart = reinterpret_cast<float*>(ws + w.dbpart);
  for (int l = d.L - 1; l >= 0; --l) {
    const int Il = in_dim(d, l);
    const float* hl = reserve + (size_t)l * res_layer_floats(cell, d);
    const float* svl = hl + TB * H;
    const float* in = l == 0 ? x : reserve + (size_t)(l - 1) * res_layer_floats(cell, d);
    size_t woff = 0;
    for (int q = 0; q < l; ++q) woff += G * in_dim(d, q);
    const float* Wl = W + woff;
    const float* Rl = R + (size_t)l * G * H;
    const float* dout = (l == d.L - 1) ? dy : dxb[(l + 1) & 1];
    const float* cin = dhT ? dhT + (size_t)l * BH : nullptr;
    int cur = 0;
    for (int t = d.T - 1; t >= 0; --t) {
      const float* hp = t ? hl + (size_t)(t - 1) * BH : (h0 ? h0 + (size_t)l * BH : nullptr);
      float* nxt = carry[cur];
      hipLaunchKernelGGL(cell_bwd_kernel, dim3(ew_grid((long)BH)), dim3(256), 0, s, cell, dout + (size_t)t * BH, cin,
                         hl + (size_t)t * BH, hp, cell == RNN_CELL_GRU ? svl + (size_t)t * B * 4 * H : nullptr,
                         da + (size_t)t * B * G, dq + (size_t)t * B * G, nxt, B, H);
      CK(hipGetLastError(), "point-wise backward");
      // dh_{t-1} = direct + dq_t R  (the stacked gates map to one output, Section 2.1)
      GemmProblem p{dq + (size_t)t * B * G, Rl, nxt, B, H, (int)G, (long)G, 1, H, 1, H, 1};
      CK(launch_gemm_group(&p, 1, s), "recurrent backward GEMM");
      cin = nxt;
      cur ^= 1;
    }
    if (dh0) CK(launch_ew(EW_COPY, dh0 + (size_t)l * BH, H, cin, H, nullptr, 0, B, H, s), "copy dh0");
    float* din = l > 0 ? dxb[l & 1] : dx;
    if (din) {
      GemmProblem p{da, Wl, din, (int)TB, Il, (int)G, (long)G, 1, Il, 1, Il, 0};
      CK(launch_gemm_group(&p, 1, s), "input-gradient GEMM");
    }
    // Section 2.6: weight gradients as large products once the layer's propagation is complete
    float* dWl = dW + woff;
    float* dRl = dR + (size_t)l * G * H;
    GemmProblem g[2];
    int ng = 0;
    g[ng++] = GemmProblem{da, in, dWl, (int)G, Il, (int)TB, 1, (long)G, Il, 1, Il, 0};
    if (d.T > 1) g[ng++] = GemmProblem{dq + (size_t)B * G, hl, dRl, (int)G, H, (int)(TB - B), 1, (long)G, H, 1, H, 0};
    CK(launch_gemm_group(g, ng, s), "weight-gradient GEMMs");
    if (h0) {
      GemmProblem p{dq, h0 + (size_t)l * BH, dRl, (int)G, H, B, 1, (long)G, H, 1, H, d.T > 1 ? 1 : 0};
      CK(launch_gemm_group(&p, 1, s), "weight-gradient GEMM (initial state term)");
    } else if (d.T == 1) {
      CK(launch_fill_zero(dRl, G * H * 4, s), "zero dR");
    }
    CK(launch_colsum(da, (int)TB, (int)G, dbpart, db + (size_t)l * G, s), "bias gradient");
  }
  return LSTM_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Hidden sizes without persistent kernels run zero-padded to the next size that has them, as for the LSTM
// (padded_hidden): a padded unit has pre-activations 0 and initial state 0, so the GRU keeps it at
// h = (1 - 1/2) tanh(0) + 1/2 * 0 = 0 and the single gate at act(0) = 0, nothing reads it, and its gradients are 0.
inline Dims rnn_padded_rule(int cell, const Dims& d) {  // what the environment does not switch off
  // between 512 and 1024 these cells gain more than the LSTM does (their step-by-step path is one GEMM and one
  // point-wise kernel per step): 2.5-3 times at every size measured
  if (d.H > 512 && d.H < 1024 && gru_persistent_shape(cell, Dims{d.L, d.T, d.B, d.I, 1024}))
    return Dims{d.L, d.T, d.B, d.I, 1024};
  // between 1024 and 2048 likewise, with few rows (GRU, L = 4, T = 100, as given -> at 2048: B = 32 44-68 -> 19 ms, B = 64
  // 48-78 -> 37.5, B = 128 82 (H = 1536) -> 75 but 55 (H = 1152) as given; single gate: B = 64 26-39 -> 24, B = 96 from 1536 on)
  if (d.H > 1024 && d.H < 2048) {
    const bool pad = cell == RNN_CELL_GRU ? (d.B <= 64 || (d.B <= 128 && d.H >= 1472)) : (d.B <= 64 || (d.B <= 96 && d.H >= 1536));
    const Dims p{d.L, d.T, d.B, d.I, 2048};
    return (pad && gru_persistent_shape(cell, p)) ? p : d;
  }
  // the LSTM's rule, but only where these cells' persistent kernels take the padded shape (their batch limits are lower)
  const Dims p{d.L, d.T, d.B, d.I, padded_hidden_rule(d)};
  return (p.H == d.H || gru_persistent_shape(cell, p)) ? p : d;
}
inline Dims rnn_padded_dims(int cell, const Dims& d) {
  return (knobs().rnn_no_persistent || knobs().no_pad) ? d : rnn_padded_rule(cell, d);
}

struct RnnPad {
  size_t W, R, b, h0, y, hT, dy, dhT, dh0, dW, dR, db, inner, total;  // byte offsets
};
RnnPad rnn_pad_layout(int cell, const Dims& d, const Dims& p) {
  RnnPad q;
  size_t off = 0;
  auto take = [&](size_t floats) {
    size_t o = off;
    off = (off + floats * sizeof(float) + 255) / 256 * 256;
    return o;
  };
  const size_t G = (size_t)gates_of(cell) * p.H, nW = G * d.I + (size_t)(d.L - 1) * G * p.H, nR = (size_t)d.L * G * p.H;
  const size_t nS = (size_t)d.L * d.B * p.H, nY = (size_t)d.T * d.B * p.H;
  q.W = take(nW); q.R = take(nR); q.b = take(d.L * G);
  q.h0 = take(nS); q.y = take(nY); q.hT = take(nS);
  q.dy = take(nY); q.dhT = take(nS); q.dh0 = take(nS);
  q.dW = take(nW); q.dR = take(nR); q.db = take(d.L * G);
  q.inner = off;
  q.total = off + ws_total(cell, p);
  return q;
}

int pad_rnn_parameters(int cell, const Dims& d, int Hp, const float* W, const float* R, const float* b, float* Wp, float* Rp,
                       float* bp, hipStream_t s) {
  const long ng = gates_of(cell);
  const size_t G = (size_t)ng * d.H, Gp = (size_t)ng * Hp;
  CK(launch_resize(Wp, W, ng, Hp, d.I, d.H, d.I, s), "pad W (layer 0)");
  CK(launch_resize(Wp + Gp * d.I, W + G * d.I, ng * (d.L - 1), Hp, Hp, d.H, d.H, s), "pad W");
  CK(launch_resize(Rp, R, ng * d.L, Hp, Hp, d.H, d.H, s), "pad R");
  if (b) CK(launch_resize(bp, b, ng * d.L, 1, Hp, 1, d.H, s), "pad b");
  return LSTM_OK;
}

int forward_padded(int cell, const Dims& d, const Dims& p, const float* x, const float* h0, const float* W, const float* R,
                   const float* b, float* y, float* hT, float* reserve, char* ws, hipStream_t s) {
  const RnnPad q = rnn_pad_layout(cell, d, p);
  auto f = [&](size_t off) { return reinterpret_cast<float*>(ws + off); };
  const int LB = d.L * d.B, TB = d.T * d.B;
  int st = pad_rnn_parameters(cell, d, p.H, W, R, b, f(q.W), f(q.R), f(q.b), s);
  if (st != LSTM_OK) return st;
  if (h0) CK(launch_resize(f(q.h0), h0, 1, LB, p.H, LB, d.H, s), "pad h0");
  st = forward_impl(cell, p, x, h0 ? f(q.h0) : nullptr, f(q.W), f(q.R), f(q.b), f(q.y), hT ? f(q.hT) : nullptr, reserve,
                    ws + q.inner, s);
  if (st != LSTM_OK) return st;
  CK(launch_resize(y, f(q.y), 1, TB, d.H, TB, p.H, s), "unpad y");
  if (hT) CK(launch_resize(hT, f(q.hT), 1, LB, d.H, LB, p.H, s), "unpad hT");
  return LSTM_OK;
}

int backward_padded(int cell, const Dims& d, const Dims& p, const float* x, const float* h0, const float* W, const float* R,
                    const float* reserve, const float* dy, const float* dhT, float* dx, float* dh0, float* dW, float* dR,
                    float* db, char* ws, hipStream_t s) {
  const RnnPad q = rnn_pad_layout(cell, d, p);
  auto f = [&](size_t off) { return reinterpret_cast<float*>(ws + off); };
  const int LB = d.L * d.B, TB = d.T * d.B;
  const long ng = gates_of(cell);
  const size_t G = (size_t)ng * d.H, Gp = (size_t)ng * p.H;
  int st = pad_rnn_parameters(cell, d, p.H, W, R, nullptr, f(q.W), f(q.R), nullptr, s);
  if (st != LSTM_OK) return st;
  if (h0) CK(launch_resize(f(q.h0), h0, 1, LB, p.H, LB, d.H, s), "pad h0");
  CK(launch_resize(f(q.dy), dy, 1, TB, p.H, TB, d.H, s), "pad dy");
  if (dhT) CK(launch_resize(f(q.dhT), dhT, 1, LB, p.H, LB, d.H, s), "pad dhT");
  st = backward_impl(cell, p, x, h0 ? f(q.h0) : nullptr, f(q.W), f(q.R), reserve, f(q.dy), dhT ? f(q.dhT) : nullptr, dx,
                     dh0 ? f(q.dh0) : nullptr, f(q.dW), f(q.dR), f(q.db), ws + q.inner, s);
  if (st != LSTM_OK) return st;
  if (dh0) CK(launch_resize(dh0, f(q.dh0), 1, LB, d.H, LB, p.H, s), "unpad dh0");
  CK(launch_resize(dW, f(q.dW), ng, d.H, d.I, p.H, d.I, s), "unpad dW (layer 0)");
  CK(launch_resize(dW + G * d.I, f(q.dW) + Gp * d.I, ng * (d.L - 1), d.H, d.H, p.H, p.H, s), "unpad dW");
  CK(launch_resize(dR, f(q.dR), ng * d.L, d.H, d.H, p.H, p.H, s), "unpad dR");
  CK(launch_resize(db, f(q.db), ng * d.L, 1, d.H, 1, p.H, s), "unpad db");
  return LSTM_OK;
}

}  // namespace
}  // namespace lstm

using namespace lstm;

extern "C" {

size_t rnn_reserve_bytes(int cell, int L, int T, int B, int I, int H) {
  if (gates_of(cell) == 0 || L <= 0 || T <= 0 || B <= 0 || I <= 0 || H <= 0) return 0;
  // (padded or as given, whichever is larger -- padding only grows H -- so that the answer does not depend on the environment)
  return (size_t)L * res_layer_floats(cell, rnn_padded_rule(cell, Dims{L, T, B, I, H})) * sizeof(float);
}

size_t rnn_workspace_bytes(int cell, int L, int T, int B, int I, int H) {
  if (gates_of(cell) == 0 || L <= 0 || T <= 0 || B <= 0 || I <= 0 || H <= 0) return 0;
  const Dims d{L, T, B, I, H}, p = rnn_padded_rule(cell, d);
  const size_t given = ws_total(cell, d);
  return p.H == d.H ? given : std::max(given, rnn_pad_layout(cell, d, p).total);
}

int rnn_forward(int cell, int L, int T, int B, int I, int H, const float* x, const float* h0, const float* W,
                const float* R, const float* b, float* y, float* hT, void* reserve, void* workspace,
                size_t workspace_bytes, void* stream) {
  if (gates_of(cell) == 0 || L <= 0 || T <= 0 || B <= 0 || I <= 0 || H <= 0) return LSTM_INVALID_ARG;
  if (!x || !W || !R || !b || !y || !reserve || !workspace) return LSTM_INVALID_ARG;
  const void* ptrs[] = {x, h0, W, R, b, y, hT, reserve, workspace};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return LSTM_INVALID_ARG;
  const Dims d{L, T, B, I, H}, p = rnn_padded_dims(cell, d);
  if (workspace_bytes < rnn_workspace_bytes(cell, L, T, B, I, H)) return LSTM_BUFFER_TOO_SMALL;
  if (take_watchdog()) return LSTM_INTERNAL;  // an earlier call's persistent kernel gave up waiting: reported once, here
  if (p.H != d.H) {
    return forward_padded(cell, d, p, x, h0, W, R, b, y, hT, reinterpret_cast<float*>(reserve),
                          reinterpret_cast<char*>(workspace), (hipStream_t)stream);
  }
  return forward_impl(cell, d, x, h0, W, R, b, y, hT, reinterpret_cast<float*>(reserve), reinterpret_cast<char*>(workspace),
                      (hipStream_t)stream);
}

int rnn_backward(int cell, int L, int T, int B, int I, int H, const float* x, const float* h0, const float* W,
                 const float* R, const void* reserve, const float* dy, const float* dhT, float* dx, float* dh0, float* dW,
                 float* dR, float* db, void* workspace, size_t workspace_bytes, void* stream) {
  if (gates_of(cell) == 0 || L <= 0 || T <= 0 || B <= 0 || I <= 0 || H <= 0) return LSTM_INVALID_ARG;
  if (!x || !W || !R || !reserve || !dy || !dW || !dR || !db || !workspace) return LSTM_INVALID_ARG;
  const void* ptrs[] = {x, h0, W, R, reserve, dy, dhT, dx, dh0, dW, dR, db, workspace};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return LSTM_INVALID_ARG;
  const Dims d{L, T, B, I, H}, p = rnn_padded_dims(cell, d);
  if (workspace_bytes < rnn_workspace_bytes(cell, L, T, B, I, H)) return LSTM_BUFFER_TOO_SMALL;
  if (take_watchdog()) return LSTM_INTERNAL;  // an earlier call's persistent kernel gave up waiting: reported once, here
  if (p.H != d.H) {
    return backward_padded(cell, d, p, x, h0, W, R, reinterpret_cast<const float*>(reserve), dy, dhT, dx, dh0, dW, dR, db,
                           reinterpret_cast<char*>(workspace), (hipStream_t)stream);
  }
  return backward_impl(cell, d, x, h0, W, R, reinterpret_cast<const float*>(reserve), dy, dhT, dx, dh0, dW, dR, db,
                       reinterpret_cast<char*>(workspace), (hipStream_t)stream);
}

}  // extern "C"
