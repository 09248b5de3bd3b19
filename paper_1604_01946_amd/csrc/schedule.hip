// Host-side schedules: the order in which each execution path enqueues its kernels.
//
// The paths are the rungs of the optimisation ladder of arXiv 1604.01946 (Table 1):
//   naive    -- Section 2.1 / Listing 1: per-gate GEMMs, one kernel per point-wise operation
//   grouped  -- Section 2.1: the four gates stacked into one GEMM per operand
//   fused    -- Section 2.2.2: one fused point-wise kernel per cell
//   step     -- Section 2.3 / Listing 3: input projections of all steps in one GEMM, weights
//               re-laid out once per pass, recurrent GEMM + point-wise fused per step
//   wavefront / persistent -- Section 2.4 and Section 4 (wavefront.hip, persistent.hip)
// The paper's ladder is forward only; the backward schedules mirror it (Section 2.1 on the
// backward pass, Section 2.6 on the weight update).
#include "../../include/lstm.h"
#include "schedule.h"

#include <mutex>
#include <vector>

namespace lstm {

#define CK(expr, what)                                             \
  do {                                                             \
    if (record((expr), what) != hipSuccess) return LSTM_HIP_ERROR; \
  } while (0)

int run_forward_wavefront(const FwdArgs& a);
int run_backward_wavefront(const BwdArgs& a);
int run_forward_persistent(const FwdArgs& a, int cell = 0);
int run_backward_persistent(const BwdArgs& a, int cell = 0, bool* bias_done = nullptr, LayerGradients* lg = nullptr);
bool persistent_supported(const Dims& d, bool backward);

// Per-shape overrides of the automatic choice (lstm_set_path), a few entries, guarded by a mutex.
namespace {
struct PathOverride {
  Dims d;
  bool backward;
  unsigned path;
};
std::mutex g_path_mu;
std::vector<PathOverride> g_path_table;
bool same_shape(const Dims& a, const Dims& b) { return a.L == b.L && a.T == b.T && a.B == b.B && a.I == b.I && a.H == b.H; }
}  // namespace

bool path_takes_shape(const Dims& d, bool backward, unsigned path) {
  switch (path) {
    case LSTM_PATH_NAIVE: case LSTM_PATH_GROUPED: case LSTM_PATH_FUSED: case LSTM_PATH_STEP: case LSTM_PATH_WAVEFRONT: return true;
    case LSTM_PATH_PERSISTENT: return persistent_supported(d, backward);
    default: return false;
  }
}

int set_path_override(const Dims& d, bool backward, unsigned path) {
  // the kernels see the padded hidden size (padded_hidden), so that is the shape a path has to take
  if (path != LSTM_PATH_AUTO && !path_takes_shape(padded_dims(d), backward, path)) return path > LSTM_PATH_PERSISTENT ? LSTM_INVALID_ARG : LSTM_UNSUPPORTED;
  std::lock_guard<std::mutex> lk(g_path_mu);
  for (size_t i = 0; i < g_path_table.size(); ++i)
    if (same_shape(g_path_table[i].d, d) && g_path_table[i].backward == backward) {
      if (path == LSTM_PATH_AUTO) g_path_table.erase(g_path_table.begin() + (long)i);
      else g_path_table[i].path = path;
      return LSTM_OK;
    }
  if (path != LSTM_PATH_AUTO) g_path_table.push_back(PathOverride{d, backward, path});
  return LSTM_OK;
}

namespace {
struct ChunkOverride {
  Dims d;
  int chunks;
};
std::vector<ChunkOverride> g_chunk_table;
}  // namespace

int set_wavefront_chunks(const Dims& user, int chunks) {
  if (chunks < 0) return LSTM_INVALID_ARG;
  const Dims d = padded_dims(user);  // the shape the paths run at
  std::lock_guard<std::mutex> lk(g_path_mu);
  for (size_t i = 0; i < g_chunk_table.size(); ++i)
    if (same_shape(g_chunk_table[i].d, d)) {
      if (chunks == 0) g_chunk_table.erase(g_chunk_table.begin() + (long)i);
      else g_chunk_table[i].chunks = chunks;
      return LSTM_OK;
    }
  if (chunks > 0) g_chunk_table.push_back(ChunkOverride{d, chunks});
  return LSTM_OK;
}

int wavefront_chunks(const Dims& d) {
  std::lock_guard<std::mutex> lk(g_path_mu);
  for (const ChunkOverride& o : g_chunk_table)
    if (same_shape(o.d, d)) return o.chunks;
  return 0;
}

void clear_path_overrides() {
  std::lock_guard<std::mutex> lk(g_path_mu);
  g_path_table.clear();
  g_chunk_table.clear();
}

unsigned resolve_auto_path(const Dims& user, bool backward) {
  {
    std::lock_guard<std::mutex> lk(g_path_mu);
    for (const PathOverride& o : g_path_table)
      if (same_shape(o.d, user) && o.backward == backward) return o.path;
  }
  if (micro_shape(user)) return LSTM_PATH_STEP;  // one launch per pass, steps looped inside (micro.hip)
  const Dims d = padded_dims(user);  // what the kernels will run
  if (persistent_supported(d, backward)) return LSTM_PATH_PERSISTENT;
  const int cus = device_cu_count();
  // Section 3.2 observes that at large minibatches the individual optimisations stop paying.  Here: once the plain
  // [B x 4H] x [H] product of one step gives every CU three 64 x 64 tiles (or one of 128 x 128), the GEMM kernel
  // (grouped gates, fused point-wise kernel) beats the forward step kernel and the stream wavefront by 5-20 %: H = 4096
  // from B = 128 on (there already with two tiles per CU: 113 against 107 TFLOP/s), H = 3072 from 256 (115 against
  // 109), H = 1536 from 512 (115 against 100), H = 1024 from 768 (110 against 93).  Backward the split-K step kernel
  // stays ahead at every size measured (its contraction is four times longer, and it fuses the point-wise work that
  // the GEMM rung runs as a second kernel).
  if (!backward && cus > 0) {
    const long small_tiles = (long)((d.B + 63) / 64) * (4L * d.H / 64);
    if (small_tiles >= 3L * cus || (d.H >= 4096 && small_tiles >= 2L * cus)) return LSTM_PATH_FUSED;
  }
  // Overlapping layers on streams pays when one step kernel leaves CUs idle (Section 2.4: the
  // gain is largest for small layers); a step that already fills the chip runs layer by layer.
  const long wgs = (long)((d.H + 3) / 4) * ((d.B + 63) / 64);
  if (d.L > 1 && (cus == 0 || wgs < 2L * cus)) return LSTM_PATH_WAVEFRONT;
  return LSTM_PATH_STEP;
}

namespace {

inline float* ws_f(char* ws, size_t off) { return reinterpret_cast<float*>(ws + off); }

int copy_final_states(const FwdArgs& a) {
  const Dims& d = a.d;
  const size_t BH = (size_t)d.B * d.H;
  for (int l = 0; l < d.L; ++l) {
    const LayerRes r = layer_res(a.reserve, d, l);
    if (a.hT) CK(launch_ew(EW_COPY, a.hT + l * BH, d.H, r.h + (size_t)(d.T - 1) * BH, d.H, nullptr, 0, d.B, d.H, a.stream), "copy hT");
    if (a.cT) CK(launch_ew(EW_COPY, a.cT + l * BH, d.H, r.c + (size_t)(d.T - 1) * BH, d.H, nullptr, 0, d.B, d.H, a.stream), "copy cT");
  }
  return LSTM_OK;
}

// ------------------------------------------------------------------ forward: step path
int fwd_step(const FwdArgs& a) {
  const Dims& d = a.d;
  const size_t TB = (size_t)d.T * d.B, G = 4 * (size_t)d.H, BH = (size_t)d.B * d.H;
  hipStream_t s = a.stream;
  if (micro_shape(d)) {  // a launch per step would cost more than the step: all of them in one launch
    ProfScope ps(LSTM_PHASE_FWD_RECURRENCE, s);
    CK(launch_micro_forward(a), "forward pass in one workgroup");
    return LSTM_OK;
  }
  float* Rp = ws_f(a.ws, a.w.RT);
  const size_t pf = step_plan(d).pack_floats;
  {
    ProfScope ps(LSTM_PHASE_FWD_PACK, s);
    CK(launch_pack_fwd(a.R, Rp, d.L, d.H, d.B, pf, s), "pack R");
  }
  for (int l = 0; l < d.L; ++l) {
    const int Il = in_dim(d, l);
    const LayerRes r = layer_res(a.reserve, d, l);
    const float* in = l == 0 ? a.x : layer_res(a.reserve, d, l - 1).h;
    const float* Wl = a.W + w_offset(d, l);
    const float* Rl = Rp + (size_t)l * pf;
    float* P = ws_f(a.ws, a.w.P) + (size_t)l * TB * G;
    {
      ProfScope ps(LSTM_PHASE_FWD_INPUT_GEMM, s);
      GemmProblem p{in, Wl, P, (int)TB, (int)G, Il, Il, 1, 1, Il, (long)G, 0};
      CK(launch_gemm_group(&p, 1, s), "input projection GEMM");
    }
    ProfScope ps(LSTM_PHASE_FWD_RECURRENCE, s);
    for (int t = 0; t < d.T; ++t) {
      StepFwdArgs sa;
      sa.Rp = Rl;
      sa.h_prev = t ? r.h + (size_t)(t - 1) * BH : (a.h0 ? a.h0 + l * BH : nullptr);
      sa.c_prev = t ? r.c + (size_t)(t - 1) * BH : (a.c0 ? a.c0 + l * BH : nullptr);
      sa.P = P + (size_t)t * d.B * G;
      sa.bias = a.b + (size_t)l * G;
      sa.h_out = r.h + (size_t)t * BH;
      sa.c_out = r.c + (size_t)t * BH;
      sa.gates_out = r.gates + (size_t)t * d.B * G;
      sa.h_out2 = (l == d.L - 1) ? a.y + (size_t)t * BH : nullptr;
      sa.c_out2 = nullptr;
      sa.B = d.B;
      sa.H = d.H;
      CK(launch_step_fwd(sa, s), "forward step kernel");
    }
  }
  return copy_final_states(a);
}

// ------------------------------------------------------------------ forward: unfused rungs
// level 0: per-gate GEMMs + one kernel per point-wise op; 1: grouped GEMMs; 2: + fused point-wise.
int fwd_unfused(const FwdArgs& a, int level) {
  const Dims& d = a.d;
  const size_t G = 4 * (size_t)d.H, BH = (size_t)d.B * d.H, BG = (size_t)d.B * G;
  const int B = d.B, H = d.H;
  hipStream_t s = a.stream;
  float* S1 = ws_f(a.ws, a.w.scratch);
  float* S2 = S1 + BG;
  float* tmp = S2 + BG;
  float* zero = ws_f(a.ws, a.w.state) + 2 * (size_t)d.L * BH;
  CK(launch_fill_zero(zero, BH * 4, s), "zero block");
  for (int l = 0; l < d.L; ++l) {
    const int Il = in_dim(d, l);
    const LayerRes r = layer_res(a.reserve, d, l);
    const float* in = l == 0 ? a.x : layer_res(a.reserve, d, l - 1).h;
    const float* Wl = a.W + w_offset(d, l);
    const float* Rl = a.R + (size_t)l * G * H;
    const float* bl = a.b + (size_t)l * G;
    for (int t = 0; t < d.T; ++t) {
      const float* xt = in + (size_t)t * B * Il;
      const float* hp = t ? r.h + (size_t)(t - 1) * BH : (a.h0 ? a.h0 + l * BH : zero);
      const float* cp = t ? r.c + (size_t)(t - 1) * BH : (a.c0 ? a.c0 + l * BH : zero);
      float* ht = r.h + (size_t)t * BH;
      float* ct = r.c + (size_t)t * BH;
      float* gt = r.gates + (size_t)t * BG;
      if (level == 0) {
        for (int g = 0; g < 4; ++g) {
          GemmProblem p1{xt, Wl + (size_t)g * H * Il, S1 + g * H, B, H, Il, Il, 1, 1, Il, (long)G, 0};
          CK(launch_gemm_group(&p1, 1, s), "per-gate input GEMM");
          GemmProblem p2{hp, Rl + (size_t)g * H * H, S2 + g * H, B, H, H, H, 1, 1, H, (long)G, 0};
          CK(launch_gemm_group(&p2, 1, s), "per-gate recurrent GEMM");
        }
      } else {
        GemmProblem p1{xt, Wl, S1, B, (int)G, Il, Il, 1, 1, Il, (long)G, 0};
        CK(launch_gemm_group(&p1, 1, s), "grouped input GEMM");
        GemmProblem p2{hp, Rl, S2, B, (int)G, H, H, 1, 1, H, (long)G, 0};
        CK(launch_gemm_group(&p2, 1, s), "grouped recurrent GEMM");
      }
      if (level >= 2) {
        CK(launch_pointwise_fwd(S1, S2, bl, cp, ht, ct, gt, (l == d.L - 1) ? a.y + (size_t)t * BH : nullptr, nullptr, B, H, s),
           "fused point-wise");
        continue;
      }
      if (level == 0) {
        for (int g = 0; g < 4; ++g) CK(launch_ew(EW_ADD, S1 + g * H, G, S1 + g * H, G, S2 + g * H, G, B, H, s), "add");
        for (int g = 0; g < 4; ++g) CK(launch_ew(EW_ADD_BIAS, S1 + g * H, G, S1 + g * H, G, bl + g * H, 0, B, H, s), "bias");
        for (int g = 0; g < 3; ++g) CK(launch_ew(EW_SIGMOID, gt + g * H, G, S1 + g * H, G, nullptr, 0, B, H, s), "sigmoid");
      } else {
        CK(launch_ew(EW_ADD, S1, G, S1, G, S2, G, B, (int)G, s), "add");
        CK(launch_ew(EW_ADD_BIAS, S1, G, S1, G, bl, 0, B, (int)G, s), "bias");
        CK(launch_ew(EW_SIGMOID, gt, G, S1, G, nullptr, 0, B, 3 * H, s), "sigmoid");
      }
      CK(launch_ew(EW_TANH, gt + 3 * H, G, S1 + 3 * H, G, nullptr, 0, B, H, s), "tanh");
      CK(launch_ew(EW_MUL, ct, H, gt + H, G, cp, H, B, H, s), "f*c");
      CK(launch_ew(EW_MUL, tmp, H, gt, G, gt + 3 * H, G, B, H, s), "i*g");
      CK(launch_ew(EW_ADD, ct, H, ct, H, tmp, H, B, H, s), "c");
      CK(launch_ew(EW_TANH, tmp, H, ct, H, nullptr, 0, B, H, s), "tanh c");
      CK(launch_ew(EW_MUL, ht, H, gt + 2 * H, G, tmp, H, B, H, s), "h");
      if (l == d.L - 1) CK(launch_ew(EW_COPY, a.y + (size_t)t * BH, H, ht, H, nullptr, 0, B, H, s), "y");
    }
  }
  return copy_final_states(a);
}

}  // namespace

// ------------------------------------------------------------------ weight update (Section 2.6)
// dW_l = sum_t dA_t^T in_t, dR_l = sum_t dA_t^T h_{t-1}, db_l = sum_t,b dA_t: products over K = T*B
// with no dependencies between them, so all of them go into grouped launches.
int weight_gradients(const BwdArgs& a, const float* dA_all, bool grouped, bool bias_done) {
  return weight_gradients_layers(a, dA_all, 0, a.d.L, a.stream, grouped, bias_done);
}

// Layers l0 .. l1-1, on stream s (which may be another stream than the call's: the caller orders it).
int weight_gradients_layers(const BwdArgs& a, const float* dA_all, int l0, int l1, hipStream_t s, bool grouped,
                            bool bias_done) {
  const Dims& d = a.d;
  const size_t TB = (size_t)d.T * d.B, G = 4 * (size_t)d.H;
  const int H = d.H, B = d.B;
  GemmProblem main_p[kMaxGemmGroup], tail_p[kMaxGemmGroup];
  int nm = 0, nt = 0;
  auto flush = [&](GemmProblem* arr, int& n) -> hipError_t {
    hipError_t e = hipSuccess;
    if (grouped) {
      e = launch_gemm_group(arr, n, s);
    } else {
      for (int i = 0; i < n && e == hipSuccess; ++i) e = launch_gemm_group(arr + i, 1, s);
    }
    n = 0;
    return e;
  };
  if (!bias_done) {
    ProfScope ps(LSTM_PHASE_BIAS_GRAD, s);
    // all layers in one pair of launches: dA [L][T*B][4H] -> db [L][4H]
    CK(launch_colsum_batched(dA_all + (size_t)l0 * TB * G, (int)TB, (int)G, l1 - l0,
                             reinterpret_cast<float*>(a.ws + a.w.dbpart) + (size_t)l0 * 64 * G, a.db + (size_t)l0 * G, s),
       "bias gradient");
  }
  ProfScope ps(LSTM_PHASE_WEIGHT_GRAD, s);
  for (int l = l0; l < l1; ++l) {
    const int Il = in_dim(d, l);
    const float* dA = dA_all + (size_t)l * TB * G;
    const float* in = l == 0 ? a.x : layer_res(a.reserve, d, l - 1).h;
    const LayerRes r = layer_res(a.reserve, d, l);
    float* dWl = a.dW + w_offset(d, l);
    float* dRl = a.dR + (size_t)l * G * H;
    if (nm + 2 > kMaxGemmGroup) CK(flush(main_p, nm), "weight-gradient GEMMs");
    main_p[nm++] = GemmProblem{dA, in, dWl, (int)G, Il, (int)TB, 1, (long)G, Il, 1, Il, 0};
    if (d.T > 1) {
      main_p[nm++] = GemmProblem{dA + (size_t)B * G, r.h, dRl, (int)G, H, (int)(TB - B), 1, (long)G, H, 1, H, 0};
      if (a.h0) {
        if (nt + 1 > kMaxGemmGroup) {
          CK(flush(main_p, nm), "weight-gradient GEMMs");
          CK(flush(tail_p, nt), "weight-gradient GEMMs (initial state term)");
        }
        tail_p[nt++] = GemmProblem{dA, a.h0 + (size_t)l * B * H, dRl, (int)G, H, B, 1, (long)G, H, 1, H, 1};
      }
    } else if (a.h0) {
      main_p[nm++] = GemmProblem{dA, a.h0 + (size_t)l * B * H, dRl, (int)G, H, B, 1, (long)G, H, 1, H, 0};
    } else {
      CK(launch_fill_zero(dRl, G * H * 4, s), "zero dR");
    }
  }
  CK(flush(main_p, nm), "weight-gradient GEMMs");
  CK(flush(tail_p, nt), "weight-gradient GEMMs (initial state term)");
  return LSTM_OK;
}

namespace {

// ------------------------------------------------------------------ backward: step path
int bwd_step(const BwdArgs& a) {
  const Dims& d = a.d;
  const size_t TB = (size_t)d.T * d.B, G = 4 * (size_t)d.H, BH = (size_t)d.B * d.H, BG = (size_t)d.B * G;
  const int H = d.H, B = d.B, T = d.T;
  hipStream_t s = a.stream;
  if (micro_shape(d)) {
    ProfScope ps(LSTM_PHASE_BWD_RECURRENCE, s);
    CK(launch_micro_backward(a), "backward pass in one workgroup");
    return LSTM_OK;
  }
  float* dA_all = ws_f(a.ws, a.w.P);
  float* RT = ws_f(a.ws, a.w.RT);
  const StepPlan sp = step_plan(d);
  const size_t pf = sp.pack_floats;
  float* skpart = ws_f(a.ws, a.w.skpart);
  int* skcnt = reinterpret_cast<int*>(a.ws + a.w.skcnt);
  float* dxb = ws_f(a.ws, a.w.dx);
  float* dcb = ws_f(a.ws, a.w.state);
  // weights re-laid out once per pass: the backward products read R transposed (Section 2.3)
  {
    ProfScope ps(LSTM_PHASE_BWD_PACK, s);
    if (sp.sk) {
      CK(launch_pack_bwd_sk(a.R, RT, d.L, H, B, pf, s), "pack R (transposed, split-K)");
      CK(launch_fill_zero(skcnt, (size_t)d.L * (T + 1) * sp.counter_ints * 4, s), "zero arrival counters");
    } else {
      CK(launch_pack_bwd(a.R, RT, d.L, H, B, pf, s), "pack R (transposed)");
    }
  }
  auto bwd_launch = [&](const StepBwdArgs& sa, int l, int slot) -> hipError_t {
    if (sp.sk)
      return launch_step_bwd_sk(sa, skpart + (size_t)l * sp.part_floats,
                                skcnt + ((size_t)l * (T + 1) + slot) * sp.counter_ints, s);
    return launch_step_bwd(sa, s);
  };
  for (int l = d.L - 1; l >= 0; --l) {
    const int Il = in_dim(d, l);
    const LayerRes r = layer_res(a.reserve, d, l);
    float* dA = dA_all + (size_t)l * TB * G;
    const float* dout = (l == d.L - 1) ? a.dy : dxb + (size_t)(l + 1) * TB * H;
    float* dc = dcb + (size_t)l * BH;
    prof_begin(LSTM_PHASE_BWD_RECURRENCE, s);
    for (int t = T - 1; t >= 0; --t) {
      StepBwdArgs sa;
      sa.RTp = RT + (size_t)l * pf;
      sa.dA_next = (t < T - 1) ? dA + (size_t)(t + 1) * BG : nullptr;
      sa.dh_extra = (t == T - 1 && a.dhT) ? a.dhT + l * BH : nullptr;
      sa.dout = dout + (size_t)t * BH;
      sa.gates = r.gates + (size_t)t * BG;
      sa.c_t = r.c + (size_t)t * BH;
      sa.c_prev = t ? r.c + (size_t)(t - 1) * BH : (a.c0 ? a.c0 + l * BH : nullptr);
      sa.dc_in = (t == T - 1) ? (a.dcT ? a.dcT + l * BH : nullptr) : dc;
      sa.dA = dA + (size_t)t * BG;
      sa.dc_out = (t == 0 && a.dc0) ? a.dc0 + l * BH : dc;
      sa.dh_out = nullptr;
      sa.pointwise = 1;
      sa.B = B;
      sa.H = H;
      CK(bwd_launch(sa, l, t + 1), "backward step kernel");
    }
    if (a.dh0) {
      StepBwdArgs sa{};
      sa.RTp = RT + (size_t)l * pf;
      sa.dA_next = dA;
      sa.dh_out = a.dh0 + l * BH;
      sa.pointwise = 0;
      sa.B = B;
      sa.H = H;
      CK(bwd_launch(sa, l, 0), "backward step kernel (dh0)");
    }
    prof_end(LSTM_PHASE_BWD_RECURRENCE, s);
    // gradient for the layer below (or dx): all T steps in one product
    float* din = l > 0 ? dxb + (size_t)l * TB * H : a.dx;
    if (din) {
      ProfScope ps(LSTM_PHASE_BWD_INPUT_GEMM, s);
      GemmProblem p{dA, a.W + w_offset(d, l), din, (int)TB, Il, (int)G, (long)G, 1, Il, 1, Il, 0};
      CK(launch_gemm_group(&p, 1, s), "input-gradient GEMM");
    }
  }
  return weight_gradients(a, dA_all, true, false);
}

// ------------------------------------------------------------------ backward: unfused rungs
int bwd_unfused(const BwdArgs& a, bool per_gate) {
  const Dims& d = a.d;
  const size_t TB = (size_t)d.T * d.B, G = 4 * (size_t)d.H, BH = (size_t)d.B * d.H, BG = (size_t)d.B * G;
  const int H = d.H, B = d.B, T = d.T;
  hipStream_t s = a.stream;
  float* dA_all = ws_f(a.ws, a.w.P);
  float* dxb = ws_f(a.ws, a.w.dx);
  float* dcb = ws_f(a.ws, a.w.state);
  float* dhb = dcb + (size_t)d.L * BH;
  for (int l = d.L - 1; l >= 0; --l) {
    const int Il = in_dim(d, l);
    const LayerRes r = layer_res(a.reserve, d, l);
    const float* Wl = a.W + w_offset(d, l);
    const float* Rl = a.R + (size_t)l * G * H;
    float* dA = dA_all + (size_t)l * TB * G;
    const float* dout = (l == d.L - 1) ? a.dy : dxb + (size_t)(l + 1) * TB * H;
    float* dc = dcb + (size_t)l * BH;
    float* dh = dhb + (size_t)l * BH;
    float* din = l > 0 ? dxb + (size_t)l * TB * H : a.dx;
    for (int t = T - 1; t >= 0; --t) {
      const float* dh_b = (t == T - 1) ? (a.dhT ? a.dhT + l * BH : nullptr) : dh;
      const float* dc_in = (t == T - 1) ? (a.dcT ? a.dcT + l * BH : nullptr) : dc;
      const float* cp = t ? r.c + (size_t)(t - 1) * BH : (a.c0 ? a.c0 + l * BH : nullptr);
      float* dAt = dA + (size_t)t * BG;
      CK(launch_pointwise_bwd(r.gates + (size_t)t * BG, r.c + (size_t)t * BH, cp, dout + (size_t)t * BH, dh_b, dc_in,
                              dAt, (t == 0 && a.dc0) ? a.dc0 + l * BH : dc, B, H, s),
         "backward point-wise");
      float* dh_dst = (t == 0) ? (a.dh0 ? a.dh0 + l * BH : nullptr) : dh;
      if (per_gate) {
        for (int g = 0; g < 4; ++g) {
          if (dh_dst) {
            GemmProblem p{dAt + g * H, Rl + (size_t)g * H * H, dh_dst, B, H, H, (long)G, 1, H, 1, H, g > 0};
            CK(launch_gemm_group(&p, 1, s), "per-gate recurrent gradient GEMM");
          }
          if (din) {
            GemmProblem p{dAt + g * H, Wl + (size_t)g * H * Il, din + (size_t)t * B * Il, B, Il, H, (long)G, 1, Il, 1, Il, g > 0};
            CK(launch_gemm_group(&p, 1, s), "per-gate input gradient GEMM");
          }
        }
      } else {
        if (dh_dst) {
          GemmProblem p{dAt, Rl, dh_dst, B, H, (int)G, (long)G, 1, H, 1, H, 0};
          CK(launch_gemm_group(&p, 1, s), "recurrent gradient GEMM");
        }
        if (din) {
          GemmProblem p{dAt, Wl, din + (size_t)t * B * Il, B, Il, (int)G, (long)G, 1, Il, 1, Il, 0};
          CK(launch_gemm_group(&p, 1, s), "input gradient GEMM");
        }
      }
    }
  }
  return weight_gradients(a, dA_all, !per_gate, false);
}

}  // namespace

int run_forward(const FwdArgs& a, unsigned path) {
  switch (path) {
    case LSTM_PATH_NAIVE: return fwd_unfused(a, 0);
    case LSTM_PATH_GROUPED: return fwd_unfused(a, 1);
    case LSTM_PATH_FUSED: return fwd_unfused(a, 2);
    case LSTM_PATH_STEP: return fwd_step(a);
    case LSTM_PATH_WAVEFRONT: return run_forward_wavefront(a);
    case LSTM_PATH_PERSISTENT:
      if (!persistent_supported(a.d, false)) return LSTM_UNSUPPORTED;
      return run_forward_persistent(a);
    default: return LSTM_INVALID_ARG;
  }
}

int run_backward(const BwdArgs& a, unsigned path) {
  switch (path) {
    case LSTM_PATH_NAIVE: return bwd_unfused(a, true);
    case LSTM_PATH_GROUPED:
    case LSTM_PATH_FUSED: return bwd_unfused(a, false);
    case LSTM_PATH_STEP: return bwd_step(a);
    case LSTM_PATH_WAVEFRONT: return run_backward_wavefront(a);
    case LSTM_PATH_PERSISTENT:
      if (!persistent_supported(a.d, true)) return LSTM_UNSUPPORTED;
      return run_backward_persistent(a);
    default: return LSTM_INVALID_ARG;
  }
}

}  // namespace lstm
