// Host-side plan structures shared by the API and the per-path schedules.
#pragma once
#include "internal.h"

namespace lstm {

struct Dims {
  int L, T, B, I, H;
};

// Byte offsets of the regions carved out of the caller's workspace.
struct WsLayout {
  size_t P;        // [L][T*B][4H]  forward: input projections; backward: gate gradients dA
  size_t dx;       // [L][T*B][H]   backward: gradient handed from layer l to layer l-1
  size_t RT;       // [L][step_pack_floats(H)]  recurrent matrices packed for the step kernels
  size_t state;    // [4][L][B][H]  carried cell/hidden gradients, zero block
  size_t dbpart;   // [L][64][4H]   bias-gradient partial sums
  size_t scratch;  // [8][B][4H]    per-cell temporaries of the unfused paths
  size_t xchg;     // persistent path: k-major exchange buffers
  size_t flags;    // persistent path: step counters and the watchdog word
  size_t skpart;   // [L][splitk_partial_floats]  split-K partial sums
  size_t skcnt;    // [L][T+1][splitk_counter_ints] split-K arrival counters
  size_t resv;     // stand-in for `reserve` when the caller runs inference
  size_t total;
};

struct FwdArgs {
  Dims d;
  const float *x, *h0, *c0, *W, *R, *b;
  float *y, *hT, *cT;
  float* reserve;
  char* ws;
  WsLayout w;
  hipStream_t stream;
  bool inference = false;  // the caller passed no reserve: `reserve` is a stand-in inside the workspace, nobody reads it
};

struct BwdArgs {
  Dims d;
  const float *x, *h0, *c0, *W, *R;
  const float* reserve;
  const float *dy, *dhT, *dcT;
  float *dx, *dh0, *dc0, *dW, *dR, *db;
  char* ws;
  WsLayout w;
  hipStream_t stream;
};

// Hidden size the kernels run a shape at.  Hidden units with zero weights, bias and initial state stay at h = c = 0
// for every step and receive zero gradients, so a network padded that way computes exactly the given one; the
// persistent kernels exist for H = 128, 256 and 512, and any other hidden size below 512 runs faster (several times,
// with more than one layer) padded to the next of them than on the per-step paths.  LSTM_NO_PAD=1 in the environment disables it.
// micro.hip: a whole pass in one workgroup, for the smallest networks (part of the step path)
bool micro_shape(const Dims& d);
hipError_t launch_micro_forward(const FwdArgs& a);
hipError_t launch_micro_backward(const BwdArgs& a);
int padded_hidden(const Dims& d);
int padded_hidden_rule(const Dims& d);  // the same without looking at LSTM_NO_PAD (size queries cover both settings)
inline Dims padded_dims(const Dims& d) { return Dims{d.L, d.T, d.B, d.I, padded_hidden(d)}; }
// dst [outer][rd][cd] <- src [outer][rs][cs]: the common corner is copied, the rest of dst is zero (pads and crops).
hipError_t launch_resize(float* dst, const float* src, long outer, int rd, int cd, int rs, int cs, hipStream_t s);

size_t reserve_bytes(const Dims& d);
WsLayout ws_layout(const Dims& d, bool wide_rows = false);
unsigned resolve_auto_path(const Dims& d, bool backward);
int set_path_override(const Dims& d, bool backward, unsigned path);  // LSTM_PATH_AUTO removes the entry
int set_wavefront_chunks(const Dims& d, int chunks);                 // 0 removes the entry
int wavefront_chunks(const Dims& d);                                 // 0: no entry (d as the kernels see it)
void clear_path_overrides();
// Weight gradients of one layer on a given stream, supplied by the caller of the persistent backward pass for the
// cells whose gradient products it forms itself; *used is set when the pass has called it for every layer.
struct LayerGradients {
  int (*fn)(void* ctx, int layer, hipStream_t s);
  void* ctx;
  bool used;
};

int weight_gradients_layers(const BwdArgs& a, const float* dA_all, int l0, int l1, hipStream_t s, bool grouped,
                            bool bias_done);
int run_forward(const FwdArgs& a, unsigned path);
int run_backward(const BwdArgs& a, unsigned path);
void release_helpers();
hipError_t setup_persistent();  // creates, for the current device, what the persistent path otherwise creates on first use
bool take_watchdog();  // true once after a bounded wait of a persistent kernel expired (clears the word)
void set_trace(void* buf, size_t bytes, int block);
hipError_t record(hipError_t e, const char* what);

// Phase timing hooks (no-ops unless lstm_profile_enable(1)).
void prof_begin(int phase, hipStream_t s);
void prof_end(int phase, hipStream_t s);
struct ProfScope {
  int phase;
  hipStream_t s;
  ProfScope(int p, hipStream_t st) : phase(p), s(st) { prof_begin(p, st); }
  ~ProfScope() { prof_end(phase, s); }
};

// Recurrent weights packed once per pass for the step kernels, and one step launch; both pick the
// split-K kernels when the hidden size calls for them.
struct StepPlan {
  bool sk;               // backward steps use the split-K kernel
  size_t pack_floats;    // per layer (room for either packed layout)
  size_t part_floats;    // per layer
  size_t counter_ints;   // per (layer, step)
};
inline StepPlan step_plan(const Dims& d) {
  StepPlan p;
  p.sk = splitk_supported(d.H);
  const size_t a = step_pack_floats(d.H), b = p.sk ? splitk_pack_floats(d.H) : 0;
  p.pack_floats = a > b ? a : b;
  p.part_floats = splitk_partial_floats(d.H, d.B);
  p.counter_ints = splitk_counter_ints(d.H, d.B);
  return p;
}

inline int in_dim(const Dims& d, int l) { return l == 0 ? d.I : d.H; }
inline size_t w_offset(const Dims& d, int l) {
  return l == 0 ? 0 : (size_t)4 * d.H * d.I + (size_t)(l - 1) * 4 * d.H * d.H;
}

// Per-layer views of the reserve buffer: gates [T][B][4H] (activated i,f,o,c'), c and h [T][B][H].
struct LayerRes {
  float* gates;
  float* c;
  float* h;
};
inline LayerRes layer_res(const float* reserve, const Dims& d, int l) {
  const size_t TB = (size_t)d.T * d.B, H = d.H;
  float* base = const_cast<float*>(reserve) + (size_t)l * TB * 6 * H;
  return LayerRes{base, base + TB * 4 * H, base + TB * 5 * H};
}

}  // namespace lstm
