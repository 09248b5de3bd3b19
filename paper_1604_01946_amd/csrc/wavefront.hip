// Layer wavefront on HIP streams (Section 2.4 and Listing 4 of arXiv 1604.01946) for shapes the
// persistent kernels do not take.
//
// Cell (l, t) depends on (l, t-1) and (l-1, t) only, so layers overlap: layer l works on chunk j
// of the sequence while layer l-1 is already on chunk j+1.  Each layer owns two streams, as in
// the paper: one for its time-batched GEMMs (input projections of a chunk of s steps forward,
// input gradients of a chunk backward) and one for its chain of fused step kernels; events carry
// the (layer, chunk) dependencies, and work is enqueued in diagonal order (fewest edges from the
// first cell first) so that launches whose dependencies are met are never queued behind ones
// that still wait.  The chunk length s trades GEMM efficiency against how long a layer waits for
// the one below (Section 2.3); here the sequence is cut into about 2L chunks.
// All streams have default priority, fork from the caller's stream and join back into it.
#include "../../include/lstm.h"
#include "schedule.h"

#include <mutex>
#include <vector>

namespace lstm {

#define CK(expr, what)                                             \
  do {                                                             \
    if (record((expr), what) != hipSuccess) return LSTM_HIP_ERROR; \
  } while (0)

void release_persistent();
int weight_gradients(const BwdArgs& a, const float* dA_all, bool grouped, bool bias_done);

namespace {

struct Helpers {
  std::vector<hipStream_t> streams;
  std::vector<hipEvent_t> events;
};
std::mutex g_mu;
Helpers g_h[64];

Helpers* helpers() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  return &g_h[dev];
}

hipError_t ensure(Helpers& h, size_t nstreams, size_t nevents) {
  while (h.streams.size() < nstreams) {
    hipStream_t s;
    hipError_t e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);
    if (e != hipSuccess) return e;
    h.streams.push_back(s);
  }
  while (h.events.size() < nevents) {
    hipEvent_t ev;
    hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e != hipSuccess) return e;
    h.events.push_back(ev);
  }
  return hipSuccess;
}

inline int chunk_count(const Dims& d) {
  int n = wavefront_chunks(d);  // lstm_set_wavefront_chunks
  if (n <= 0) {
    n = 2 * d.L;
    if (n < 4) n = 4;
  }
  if (n > d.T) n = d.T;
  if (n > 64) n = 64;  // two events per (layer, chunk)
  return n;
}

inline float* ws_f(char* ws, size_t off) { return reinterpret_cast<float*>(ws + off); }

}  // namespace

void release_helpers() {
  release_persistent();
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& h : g_h) {
    for (auto s : h.streams) (void)hipStreamDestroy(s);
    for (auto e : h.events) (void)hipEventDestroy(e);
    h.streams.clear();
    h.events.clear();
  }
}

int run_forward_wavefront(const FwdArgs& a) {
  const Dims& d = a.d;
  if (d.L == 1) return run_forward(a, LSTM_PATH_STEP);  // nothing to overlap
  const size_t TB = (size_t)d.T * d.B, G = 4 * (size_t)d.H, BH = (size_t)d.B * d.H;
  const int L = d.L, T = d.T, NCH = chunk_count(d), S = (T + NCH - 1) / NCH;
  std::lock_guard<std::mutex> lk(g_mu);
  Helpers* h = helpers();
  if (!h) return LSTM_HIP_ERROR;
  // events: 0 = fork, then per (l, j): gemm done, steps done; then per stream a join event
  const size_t n_ev = 1 + 2 * (size_t)L * NCH + 2 * L;
  CK(ensure(*h, 2 * L, n_ev), "helper streams/events");
  auto gemm_stream = [&](int l) { return h->streams[2 * l]; };
  auto step_stream = [&](int l) { return h->streams[2 * l + 1]; };
  auto ev_gemm = [&](int l, int j) { return h->events[1 + 2 * ((size_t)l * NCH + j)]; };
  auto ev_steps = [&](int l, int j) { return h->events[2 + 2 * ((size_t)l * NCH + j)]; };

  float* Rp = ws_f(a.ws, a.w.RT);
  const size_t pf = step_plan(d).pack_floats;
  {
    ProfScope ps(LSTM_PHASE_FWD_PACK, a.stream);
    CK(launch_pack_fwd(a.R, Rp, L, d.H, d.B, pf, a.stream), "pack R");
  }
  CK(hipEventRecord(h->events[0], a.stream), "fork");
  for (int i = 0; i < 2 * L; ++i) CK(hipStreamWaitEvent(h->streams[i], h->events[0], 0), "fork wait");
  prof_begin(LSTM_PHASE_FWD_RECURRENCE, a.stream);

  for (int dg = 0; dg < L + NCH - 1; ++dg) {
    for (int l = 0; l < L; ++l) {
      const int j = dg - l;
      if (j < 0 || j >= NCH) continue;
      const int t0 = j * S, t1 = (t0 + S < T) ? t0 + S : T;
      if (t0 >= t1) continue;
      const int Il = in_dim(d, l);
      const LayerRes r = layer_res(a.reserve, d, l);
      const float* in = l == 0 ? a.x : layer_res(a.reserve, d, l - 1).h;
      float* P = ws_f(a.ws, a.w.P) + (size_t)l * TB * G;
      // time-batched input projection of this chunk
      if (l > 0) CK(hipStreamWaitEvent(gemm_stream(l), ev_steps(l - 1, j), 0), "wait lower layer");
      GemmProblem p{in + (size_t)t0 * d.B * Il, a.W + w_offset(d, l), P + (size_t)t0 * d.B * G,
                    (t1 - t0) * d.B, (int)G, Il, Il, 1, 1, Il, (long)G, 0};
      CK(launch_gemm_group(&p, 1, gemm_stream(l)), "input projection GEMM");
      CK(hipEventRecord(ev_gemm(l, j), gemm_stream(l)), "record gemm");
      // the chunk's recurrent chain
      CK(hipStreamWaitEvent(step_stream(l), ev_gemm(l, j), 0), "wait gemm");
      for (int t = t0; t < t1; ++t) {
        StepFwdArgs sa;
        sa.Rp = Rp + (size_t)l * pf;
        sa.h_prev = t ? r.h + (size_t)(t - 1) * BH : (a.h0 ? a.h0 + l * BH : nullptr);
        sa.c_prev = t ? r.c + (size_t)(t - 1) * BH : (a.c0 ? a.c0 + l * BH : nullptr);
        sa.P = P + (size_t)t * d.B * G;
        sa.bias = a.b + (size_t)l * G;
        sa.h_out = r.h + (size_t)t * BH;
        sa.c_out = r.c + (size_t)t * BH;
        sa.gates_out = r.gates + (size_t)t * d.B * G;
        sa.h_out2 = (l == L - 1) ? a.y + (size_t)t * BH : nullptr;
        sa.c_out2 = nullptr;
        if (t == T - 1) {
          // final states straight from the last step (y for the top layer is written by a copy below)
          if (l == L - 1) {
            sa.c_out2 = a.cT ? a.cT + l * BH : nullptr;
          } else {
            sa.h_out2 = a.hT ? a.hT + l * BH : nullptr;
            sa.c_out2 = a.cT ? a.cT + l * BH : nullptr;
          }
        }
        sa.B = d.B;
        sa.H = d.H;
        CK(launch_step_fwd(sa, step_stream(l)), "forward step kernel");
      }
      CK(hipEventRecord(ev_steps(l, j), step_stream(l)), "record steps");
    }
  }
  if (a.hT)
    CK(launch_ew(EW_COPY, a.hT + (size_t)(L - 1) * BH, d.H, a.y + (size_t)(T - 1) * BH, d.H, nullptr, 0, d.B, d.H,
                 step_stream(L - 1)),
       "copy hT of the top layer");
  // join
  for (int i = 0; i < 2 * L; ++i) {
    hipEvent_t ev = h->events[1 + 2 * (size_t)L * NCH + i];
    CK(hipEventRecord(ev, h->streams[i]), "join record");
    CK(hipStreamWaitEvent(a.stream, ev, 0), "join wait");
  }
  prof_end(LSTM_PHASE_FWD_RECURRENCE, a.stream);
  return LSTM_OK;
}

int run_backward_wavefront(const BwdArgs& a) {
  const Dims& d = a.d;
  if (d.L == 1) return run_backward(a, LSTM_PATH_STEP);
  const size_t TB = (size_t)d.T * d.B, G = 4 * (size_t)d.H, BH = (size_t)d.B * d.H, BG = (size_t)d.B * G;
  const int L = d.L, T = d.T, H = d.H, B = d.B, NCH = chunk_count(d), S = (T + NCH - 1) / NCH;
  float* dA_all = ws_f(a.ws, a.w.P);
  float* RT = ws_f(a.ws, a.w.RT);
  float* dxb = ws_f(a.ws, a.w.dx);
  float* dcb = ws_f(a.ws, a.w.state);
  const StepPlan sp = step_plan(d);
  const size_t pf = sp.pack_floats;
  float* skpart = ws_f(a.ws, a.w.skpart);
  int* skcnt = reinterpret_cast<int*>(a.ws + a.w.skcnt);
  {
    ProfScope ps(LSTM_PHASE_BWD_PACK, a.stream);
    if (sp.sk) {
      CK(launch_pack_bwd_sk(a.R, RT, L, H, B, pf, a.stream), "pack R (transposed, split-K)");
      CK(launch_fill_zero(skcnt, (size_t)L * (T + 1) * sp.counter_ints * 4, a.stream), "zero arrival counters");
    } else {
      CK(launch_pack_bwd(a.R, RT, L, H, B, pf, a.stream), "pack R (transposed)");
    }
  }
  auto bwd_launch = [&](const StepBwdArgs& sa, int l, int slot, hipStream_t st) -> hipError_t {
    if (sp.sk)
      return launch_step_bwd_sk(sa, skpart + (size_t)l * sp.part_floats,
                                skcnt + ((size_t)l * (T + 1) + slot) * sp.counter_ints, st);
    return launch_step_bwd(sa, st);
  };
  {
    std::lock_guard<std::mutex> lk(g_mu);
    Helpers* h = helpers();
    if (!h) return LSTM_HIP_ERROR;
    const size_t n_ev = 1 + 2 * (size_t)L * NCH + 2 * L;
    CK(ensure(*h, 2 * L, n_ev), "helper streams/events");
    auto gemm_stream = [&](int l) { return h->streams[2 * l]; };
    auto step_stream = [&](int l) { return h->streams[2 * l + 1]; };
    auto ev_gemm = [&](int l, int j) { return h->events[1 + 2 * ((size_t)l * NCH + j)]; };
    auto ev_steps = [&](int l, int j) { return h->events[2 + 2 * ((size_t)l * NCH + j)]; };

    CK(hipEventRecord(h->events[0], a.stream), "fork");
    for (int i = 0; i < 2 * L; ++i) CK(hipStreamWaitEvent(h->streams[i], h->events[0], 0), "fork wait");
    prof_begin(LSTM_PHASE_BWD_RECURRENCE, a.stream);

    // diagonal order, mirrored: top layer first, last chunk first
    for (int dg = 0; dg < L + NCH - 1; ++dg) {
      for (int lr = 0; lr < L; ++lr) {
        const int jr = dg - lr;
        if (jr < 0 || jr >= NCH) continue;
        const int l = L - 1 - lr, j = NCH - 1 - jr;
        const int t0 = j * S, t1 = (t0 + S < T) ? t0 + S : T;
        if (t0 >= t1) continue;
        const int Il = in_dim(d, l);
        const LayerRes r = layer_res(a.reserve, d, l);
        float* dA = dA_all + (size_t)l * TB * G;
        const float* dout = (l == L - 1) ? a.dy : dxb + (size_t)(l + 1) * TB * H;
        float* dc = dcb + (size_t)l * BH;
        if (l < L - 1) CK(hipStreamWaitEvent(step_stream(l), ev_gemm(l + 1, j), 0), "wait upper layer");
        for (int t = t1 - 1; t >= t0; --t) {
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
          CK(bwd_launch(sa, l, t + 1, step_stream(l)), "backward step kernel");
        }
        if (t0 == 0 && a.dh0) {
          StepBwdArgs sa{};
          sa.RTp = RT + (size_t)l * pf;
          sa.dA_next = dA;
          sa.dh_out = a.dh0 + l * BH;
          sa.pointwise = 0;
          sa.B = B;
          sa.H = H;
          CK(bwd_launch(sa, l, 0, step_stream(l)), "backward step kernel (dh0)");
        }
        CK(hipEventRecord(ev_steps(l, j), step_stream(l)), "record steps");
        // the chunk's input gradient: dout of the layer below, or dx
        float* din = l > 0 ? dxb + (size_t)l * TB * H : a.dx;
        CK(hipStreamWaitEvent(gemm_stream(l), ev_steps(l, j), 0), "wait steps");
        if (din) {
          GemmProblem p{dA + (size_t)t0 * BG, a.W + w_offset(d, l), din + (size_t)t0 * B * Il,
                        (t1 - t0) * B, Il, (int)G, (long)G, 1, Il, 1, Il, 0};
          CK(launch_gemm_group(&p, 1, gemm_stream(l)), "input-gradient GEMM");
        }
        CK(hipEventRecord(ev_gemm(l, j), gemm_stream(l)), "record gemm");
      }
    }
    for (int i = 0; i < 2 * L; ++i) {
      hipEvent_t ev = h->events[1 + 2 * (size_t)L * NCH + i];
      CK(hipEventRecord(ev, h->streams[i]), "join record");
      CK(hipStreamWaitEvent(a.stream, ev, 0), "join wait");
    }
    prof_end(LSTM_PHASE_BWD_RECURRENCE, a.stream);
  }
  return weight_gradients(a, dA_all, true, false);
}

}  // namespace lstm
