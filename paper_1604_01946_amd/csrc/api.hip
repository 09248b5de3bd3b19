// C ABI of the LSTM library: argument validation, workspace carving and the host-side
// schedules of every execution path (see include/lstm.h for the contract).
#include "../../include/lstm.h"
#include "internal.h"
#include "schedule.h"
#include "knobs.h"
#include <algorithm>
#include <mutex>

#include <stdlib.h>
#include <string.h>
#include <stdio.h>
#include <string>
#include <vector>

using namespace lstm;

namespace lstm {
thread_local std::string g_last_error;

hipError_t record(hipError_t e, const char* what) {
  if (e != hipSuccess) {
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();
  }
  return e;
}

namespace {
std::mutex g_knob_mu;
Knobs g_knobs;
bool g_knobs_read = false;

bool env_is(const char* name, char c) {
  const char* e = getenv(name);
  return e && *e == c;
}
int env_int(const char* name, long lo, long hi, int unset) {
  const char* e = getenv(name);
  if (!e || !*e) return unset;
  const long v = atol(e);
  return (v >= lo && v <= hi) ? (int)v : unset;
}
}  // namespace

const Knobs& knobs() {
  std::lock_guard<std::mutex> lk(g_knob_mu);
  if (!g_knobs_read) {
    Knobs k;
    k.no_pad = env_is("LSTM_NO_PAD", '1');
    k.gemm_staged = env_is("LSTM_GEMM_STAGED", '1');
    k.gemm_split = !env_is("LSTM_GEMM_SPLIT", '0');
    k.tiny = !env_is("LSTM_TINY", '0');
    k.gemm_swap = !env_is("LSTM_GEMM_SWAP", '0');
    k.large_pp = !env_is("LSTM_LARGE_PP", '0');
    k.large_ksplit = !env_is("LSTM_LARGE_KSPLIT", '0');
    k.rnn_pp = !env_is("RNN_PINGPONG", '0');
    k.micro = env_is("LSTM_MICRO", '0') ? 0 : (env_is("LSTM_MICRO", '2') ? 2 : 1);
    k.spin_limit = env_int("LSTM_SPIN_LIMIT", 1, (1L << 30) - 1, 1 << 21);
    const char* ff = getenv("LSTM_FULL_FENCES");
    k.full_fences = ff && *ff && *ff != '0';
    k.coop_launch = env_is("LSTM_COOP_LAUNCH", '1');
    k.plain_launch = env_is("LSTM_PLAIN_LAUNCH", '1');
    k.two_chains = env_is("LSTM_CHAINS", '2');
    k.fwd_narrow = env_int("LSTM_FWD_NARROW", 0, 1, -1);
    k.bwd_narrow = env_int("LSTM_BWD_NARROW", 0, 1, -1);
    k.no_large_persistent = env_is("LSTM_NO_LARGE_PERSISTENT", '1');
    k.no_wgrad_overlap = env_is("LSTM_NO_WGRAD_OVERLAP", '1');
    k.fwd_batched_input = env_is("LSTM_FWD_BATCHED_INPUT", '1');
    k.rnn_no_persistent = env_is("RNN_NO_PERSISTENT", '1');
    k.step_mt = env_int("LSTM_STEP_MT", 1, 4, 0);
    k.splitk_min_h = env_int("LSTM_SPLITK_MIN_H", 1, 1 << 20, 0);
    k.pingpong = env_int("LSTM_PINGPONG", 0, 1, -1);
    g_knobs = k;
    g_knobs_read = true;
  }
  return g_knobs;
}

void reset_knobs() {
  std::lock_guard<std::mutex> lk(g_knob_mu);
  g_knobs_read = false;
}

namespace {
struct ProfInterval {
  int phase;
  hipEvent_t start, stop;
  bool open;
  double flops;  // algorithmic FLOPs of the matrix products launched inside the interval
};
bool g_prof_on = false;
std::vector<ProfInterval> g_prof;
const char* g_prof_kernel[LSTM_PHASE_COUNT] = {};
}  // namespace

void prof_flops(double flops, const char* kernel) {
  if (!g_prof_on) return;
  for (size_t i = g_prof.size(); i-- > 0;) {
    if (g_prof[i].open) {
      g_prof[i].flops += flops;
      if (kernel && g_prof[i].phase >= 0 && g_prof[i].phase < LSTM_PHASE_COUNT) g_prof_kernel[g_prof[i].phase] = kernel;
      return;
    }
  }
}

void prof_begin(int phase, hipStream_t s) {
  if (!g_prof_on) return;
  ProfInterval iv{phase, nullptr, nullptr, true, 0.0};
  if (hipEventCreate(&iv.start) != hipSuccess || hipEventCreate(&iv.stop) != hipSuccess) return;
  (void)hipEventRecord(iv.start, s);
  g_prof.push_back(iv);
}
void prof_end(int phase, hipStream_t s) {
  if (!g_prof_on) return;
  for (size_t i = g_prof.size(); i-- > 0;) {
    if (g_prof[i].phase == phase && g_prof[i].open) {
      (void)hipEventRecord(g_prof[i].stop, s);
      g_prof[i].open = false;
      return;
    }
  }
}
}  // namespace lstm

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool dims_ok(int L, int T, int B, int I, int H) { return L > 0 && T > 0 && B > 0 && I > 0 && H > 0; }

}  // namespace

namespace lstm {

size_t reserve_bytes(const Dims& d) { return (size_t)d.L * d.T * d.B * 6 * d.H * sizeof(float); }

// wide_rows: the exchange slots hold 64 batch rows also for batches of 32 rows and fewer (the GRU runs those on the
// wide persistent kernels).
WsLayout ws_layout(const Dims& d, bool wide_rows) {
  WsLayout w;
  const size_t TB = (size_t)d.T * d.B, G = 4 * (size_t)d.H, H = d.H, L = d.L;
  const size_t Bp = (d.B > 32 || wide_rows) ? align_up((size_t)d.B, 64) : (d.B <= 16 ? 16 : 32);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  w.P = take(L * TB * G * 4);
  w.dx = take(L * TB * H * 4);
  w.RT = take(L * step_plan(d).pack_floats * 4);
  w.state = take(4 * L * d.B * H * 4);
  w.dbpart = take(L * 64 * G * 4);
  w.scratch = take(8 * (size_t)d.B * G * 4);
  // persistent paths: exchange buffers (large-H backward: gate gradients and partial sums of one layer,
  // 5 MB per step at H = 2048)
  size_t xchg = L * ((size_t)d.T + 1) * G * Bp * 4;
  if (d.H == 2048 || d.H == 1024) {  // up to four slices of 32 batch rows side by side (one at H = 2048)
    const size_t nbk = d.H / 128, sl = std::min<size_t>(((size_t)d.B + 31) / 32, d.H == 2048 ? 1 : 4);
    // (one or two slices at H = 1024 cut their tiles' K in four or two: as many partial sums as four slices)
    const size_t psl = (d.H == 1024 && sl <= 2) ? 4 : sl;
    const size_t need = d.T * (sl * nbk * 4 * 128 * 32 + psl * nbk * nbk * 128 * 32) * 4;
    if (need > xchg) xchg = need;
    const size_t fwd = sl * ((size_t)d.T + 1) * d.H * 32 * 4;
    if (fwd > xchg) xchg = fwd;
  }
  w.xchg = take(xchg);
  w.flags = take((4 * (L > 16 ? L : 16) * ((size_t)d.T + 2) * 256 + 64 + 16 * 32 * ((size_t)d.T + 2)) * 4);  // step counters, one KB each
  w.skpart = take(splitk_supported(d.H) ? L * splitk_partial_floats(d.H, d.B) * 4 : 0);
  w.skcnt = take(splitk_supported(d.H) ? L * ((size_t)d.T + 1) * splitk_counter_ints(d.H, d.B) * 4 : 0);
  w.resv = take(reserve_bytes(d));
  w.total = off;
  return w;
}

}  // namespace lstm

namespace {
// dst [outer][rd][cd] <- src [outer][rs][cs]: the common corner is copied, the rest of dst is zero.
__global__ void resize_kernel(float* __restrict__ dst, const float* __restrict__ src, long outer, int rd, int cd, int rs,
                              int cs) {
  const long n = outer * rd * cd;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    const int c = (int)(i % cd);
    const long t = i / cd;
    const int r = (int)(t % rd);
    const long o = t / rd;
    dst[i] = (r < rs && c < cs) ? src[(o * rs + r) * cs + c] : 0.f;
  }
}
}  // namespace

namespace lstm {

hipError_t launch_resize(float* dst, const float* src, long outer, int rd, int cd, int rs, int cs, hipStream_t s) {
  const long n = outer * rd * cd;
  if (n <= 0) return hipSuccess;
  const unsigned blocks = (unsigned)std::min<long>((n + 255) / 256, 4096);
  hipLaunchKernelGGL(resize_kernel, dim3(blocks), dim3(256), 0, s, dst, src, outer, rd, cd, rs, cs);
  return hipGetLastError();
}

int padded_hidden(const Dims& d) { return (knobs().no_pad || micro_shape(d)) ? d.H : padded_hidden_rule(d); }

int padded_hidden_rule(const Dims& d) {
  // 512 < H < 1024: the one-layer persistent kernels of H = 1024 against the step kernels at the given size (which
  // have no weights on chip).  Padded, the rate in terms of the given network is about 105 (H/1024)^2 TFLOP/s at 64 rows
  // and more, and better than that of the given size wherever the latter is short of rows or of arithmetic: with up
  // to 64 rows everywhere (L = 4, B = 64: H = 544 17.5 ms as given, 12.8 padded), with up to 128 rows from H = 608 on,
  // up to 256 from 640, up to 768 (the limit of those kernels) from 832.
  if (d.H > 512 && d.H < 1024 && d.B <= 768) {
    const int hmin = d.B <= 64 ? 513 : (d.B <= 128 ? 608 : (d.B <= 256 ? 640 : 832));
    if (d.H >= hmin) return 1024;
  }
  // 1024 < H < 2048 with few rows: the one-layer kernels of H = 2048 (L = 4, T = 100: 21.6 ms at 32 rows, 43.2 at 64, plus
  // about 1 ms for the copies) against the step kernels at the given size (B = 32: H = 1536 24.5 ms, H = 1792 28.1;
  // B = 64: H = 1536 43.0, H = 1792 48.7)
  if (d.H > 1024 && d.H < 2048 && ((d.B <= 32 && d.H >= 1472) || (d.B <= 64 && d.H >= 1664))) return 2048;
  if (d.H >= 512 || d.B > 16384) return d.H;  // B: the limit of the persistent kernels
  // a few steps of one layer: the copies and the weights' way onto the chip cost more than they save (T = 8: 0.14 ms
  // padded against 0.12 as given at 16 rows, but 0.16 against 0.20 at 64 rows; T = 16: 0.19 / 0.20 and 0.21 / 0.34)
  if (d.L == 1 && (d.T < 8 || (d.T < 16 && d.B < 48))) return d.H;
  const int p = d.H <= 128 ? 128 : (d.H <= 256 ? 256 : 512);
  // Above 512 rows the per-step kernels and the GEMM rung have enough to do at the given size, and padding to 512
  // pays only while it adds little arithmetic (L = 4, B = 1024: H = 448 75 TFLOP/s padded against 62 as given,
  // H = 384 55 against 55, H = 320 39 against 43; B = 2048: H = 384 56 against 72); padding to 128 or 256 pays at
  // every batch size (H = 200, B = 2048: 47 against 38; H = 100: 26 against 18).
  if (d.B > 512 && p == 512 && d.H < 416) return d.H;
  return p;
}

}  // namespace lstm

namespace {

#define CK(expr, what)                                             \
  do {                                                             \
    if (record((expr), what) != hipSuccess) return LSTM_HIP_ERROR; \
  } while (0)

inline hipError_t resize(float* dst, const float* src, long outer, int rd, int cd, int rs, int cs, hipStream_t s) {
  return launch_resize(dst, src, outer, rd, cd, rs, cs, s);
}

// Workspace of a padded call: the padded copies of every operand with a hidden axis, then the workspace of the
// padded problem.  Offsets in bytes.
struct PadLayout {
  size_t W, R, b, h0, c0, y, hT, cT, dy, dhT, dcT, dh0, dc0, dW, dR, db, inner, total;
  WsLayout w;  // of the padded problem, relative to `inner`
};

PadLayout pad_layout(const Dims& d, const Dims& p) {
  PadLayout q;
  size_t off = 0;
  auto take = [&](size_t floats) {
    size_t o = off;
    off = align_up(off + floats * sizeof(float), 256);
    return o;
  };
  const size_t G = 4 * (size_t)p.H, nW = G * d.I + (size_t)(d.L - 1) * G * p.H, nR = (size_t)d.L * G * p.H;
  const size_t nS = (size_t)d.L * d.B * p.H, nY = (size_t)d.T * d.B * p.H;
  q.W = take(nW); q.R = take(nR); q.b = take(d.L * G);
  q.h0 = take(nS); q.c0 = take(nS); q.y = take(nY); q.hT = take(nS); q.cT = take(nS);
  q.dy = take(nY); q.dhT = take(nS); q.dcT = take(nS); q.dh0 = take(nS); q.dc0 = take(nS);
  q.dW = take(nW); q.dR = take(nR); q.db = take(d.L * G);
  q.inner = off;
  q.w = ws_layout(p);
  q.total = off + q.w.total;
  return q;
}

// Recurrent and input matrices and the bias with every gate block grown from H to Hp rows (and, where the columns
// run over hidden units, from H to Hp columns).
int pad_parameters(const Dims& d, int Hp, const float* W, const float* R, const float* b, float* Wp, float* Rp, float* bp,
                   hipStream_t s) {
  const size_t G = 4 * (size_t)d.H, Gp = 4 * (size_t)Hp;
  CK(resize(Wp, W, 4, Hp, d.I, d.H, d.I, s), "pad W (layer 0)");
  CK(resize(Wp + Gp * d.I, W + G * d.I, 4L * (d.L - 1), Hp, Hp, d.H, d.H, s), "pad W");
  CK(resize(Rp, R, 4L * d.L, Hp, Hp, d.H, d.H, s), "pad R");
  if (b) CK(resize(bp, b, 4L * d.L, 1, Hp, 1, d.H, s), "pad b");
  return LSTM_OK;
}

int forward_padded(const Dims& d, const Dims& p, const float* x, const float* h0, const float* c0, const float* W,
                   const float* R, const float* b, float* y, float* hT, float* cT, void* reserve, char* ws,
                   hipStream_t s, unsigned flags, bool no_new_resources) {
  const PadLayout q = pad_layout(d, p);
  auto f = [&](size_t off) { return reinterpret_cast<float*>(ws + off); };
  const long LB = (long)d.L * d.B, TB = (long)d.T * d.B;
  {
    ProfScope ps(LSTM_PHASE_FWD_PACK, s);
    const int st = pad_parameters(d, p.H, W, R, b, f(q.W), f(q.R), f(q.b), s);
    if (st != LSTM_OK) return st;
    if (h0) CK(resize(f(q.h0), h0, 1, (int)LB, p.H, (int)LB, d.H, s), "pad h0");
    if (c0) CK(resize(f(q.c0), c0, 1, (int)LB, p.H, (int)LB, d.H, s), "pad c0");
  }
  char* inner = ws + q.inner;
  FwdArgs a{p, x, h0 ? f(q.h0) : nullptr, c0 ? f(q.c0) : nullptr, f(q.W), f(q.R), f(q.b), f(q.y), hT ? f(q.hT) : nullptr,
            cT ? f(q.cT) : nullptr, reserve ? (float*)reserve : (float*)(inner + q.w.resv), inner, q.w, s};
  a.inference = reserve == nullptr;
  unsigned path = flags & LSTM_PATH_MASK;
  if (path == LSTM_PATH_AUTO) path = resolve_auto_path(d, false);
  if (no_new_resources && path == LSTM_PATH_WAVEFRONT) path = LSTM_PATH_STEP;
  const int st = run_forward(a, path);
  if (st != LSTM_OK) return st;
  ProfScope ps(LSTM_PHASE_FWD_PACK, s);
  CK(resize(y, f(q.y), 1, (int)TB, d.H, (int)TB, p.H, s), "unpad y");
  if (hT) CK(resize(hT, f(q.hT), 1, (int)LB, d.H, (int)LB, p.H, s), "unpad hT");
  if (cT) CK(resize(cT, f(q.cT), 1, (int)LB, d.H, (int)LB, p.H, s), "unpad cT");
  return LSTM_OK;
}

int backward_padded(const Dims& d, const Dims& p, const float* x, const float* h0, const float* c0, const float* W,
                    const float* R, const void* reserve, const float* dy, const float* dhT, const float* dcT, float* dx,
                    float* dh0, float* dc0, float* dW, float* dR, float* db, char* ws, hipStream_t s, unsigned flags) {
  const PadLayout q = pad_layout(d, p);
  auto f = [&](size_t off) { return reinterpret_cast<float*>(ws + off); };
  const long LB = (long)d.L * d.B, TB = (long)d.T * d.B;
  const size_t G = 4 * (size_t)d.H, Gp = 4 * (size_t)p.H;
  {
    ProfScope ps(LSTM_PHASE_BWD_PACK, s);
    const int st = pad_parameters(d, p.H, W, R, nullptr, f(q.W), f(q.R), nullptr, s);
    if (st != LSTM_OK) return st;
    if (h0) CK(resize(f(q.h0), h0, 1, (int)LB, p.H, (int)LB, d.H, s), "pad h0");
    if (c0) CK(resize(f(q.c0), c0, 1, (int)LB, p.H, (int)LB, d.H, s), "pad c0");
    CK(resize(f(q.dy), dy, 1, (int)TB, p.H, (int)TB, d.H, s), "pad dy");
    if (dhT) CK(resize(f(q.dhT), dhT, 1, (int)LB, p.H, (int)LB, d.H, s), "pad dhT");
    if (dcT) CK(resize(f(q.dcT), dcT, 1, (int)LB, p.H, (int)LB, d.H, s), "pad dcT");
  }
  char* inner = ws + q.inner;
  BwdArgs a{p, x, h0 ? f(q.h0) : nullptr, c0 ? f(q.c0) : nullptr, f(q.W), f(q.R), (const float*)reserve, f(q.dy),
            dhT ? f(q.dhT) : nullptr, dcT ? f(q.dcT) : nullptr, dx, dh0 ? f(q.dh0) : nullptr, dc0 ? f(q.dc0) : nullptr,
            f(q.dW), f(q.dR), f(q.db), inner, q.w, s};
  unsigned path = flags & LSTM_PATH_MASK;
  if (path == LSTM_PATH_AUTO) path = resolve_auto_path(d, true);
  const int st = run_backward(a, path);
  if (st != LSTM_OK) return st;
  ProfScope ps(LSTM_PHASE_BWD_PACK, s);
  if (dh0) CK(resize(dh0, f(q.dh0), 1, (int)LB, d.H, (int)LB, p.H, s), "unpad dh0");
  if (dc0) CK(resize(dc0, f(q.dc0), 1, (int)LB, d.H, (int)LB, p.H, s), "unpad dc0");
  CK(resize(dW, f(q.dW), 4, d.H, d.I, p.H, d.I, s), "unpad dW (layer 0)");
  CK(resize(dW + G * d.I, f(q.dW) + Gp * d.I, 4L * (d.L - 1), d.H, d.H, p.H, p.H, s), "unpad dW");
  CK(resize(dR, f(q.dR), 4L * d.L, d.H, d.H, p.H, p.H, s), "unpad dR");
  CK(resize(db, f(q.db), 4L * d.L, 1, d.H, 1, p.H, s), "unpad db");
  return LSTM_OK;
}

}  // namespace

// ---------------------------------------------------------------- scratch of lstm_forward_noalloc
// One array per GPU, held from the moment the library is loaded until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress: the device address is resolved once per device, with that device
// current, and every later use goes through the resolved pointer.
constexpr size_t kScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
std::mutex g_scratch_mu;
void* g_scratch_ptr[64] = {};
bool g_init_done[64] = {};   // set-up of the persistent path done on this device (undone by lstm_shutdown)

int scratch_of_current_device(void** out) {
  int dev = -1;
  if (record(hipGetDevice(&dev), "hipGetDevice") != hipSuccess) return LSTM_HIP_ERROR;
  if (dev < 0 || dev >= 64) {
    g_last_error = "lstm_forward_noalloc: device index out of range";
    return LSTM_HIP_ERROR;
  }
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (record(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)") != hipSuccess || !p) return LSTM_HIP_ERROR;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LSTM_OK;
}

bool lstm_init_needed() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return true;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  return g_scratch_ptr[dev] == nullptr || !g_init_done[dev];
}

int forward_call(int L, int T, int B, int I, int H, const float* x, const float* h0, const float* c0, const float* W,
                 const float* R, const float* b, float* y, float* hT, float* cT, void* reserve, void* workspace,
                 size_t workspace_bytes, void* stream, unsigned flags, bool no_new_resources);
}  // namespace

extern "C" {

// Both size queries answer for the padded and for the as-given run, whichever needs more, so that the answer does
// not depend on LSTM_NO_PAD: a buffer sized under one setting is large enough under the other.
size_t lstm_reserve_bytes(int L, int T, int B, int I, int H) {
  if (!dims_ok(L, T, B, I, H)) return 0;
  const Dims d{L, T, B, I, H};
  return reserve_bytes(Dims{L, T, B, I, padded_hidden_rule(d)});  // never below the as-given size: padding only grows H
}

size_t lstm_workspace_bytes(int L, int T, int B, int I, int H) {
  if (!dims_ok(L, T, B, I, H)) return 0;
  const Dims d{L, T, B, I, H}, p{L, T, B, I, padded_hidden_rule(d)};
  const size_t given = ws_layout(d).total;
  return p.H == d.H ? given : std::max(given, pad_layout(d, p).total);
}

const char* lstm_status_string(int status) {
  switch (status) {
    case LSTM_OK: return "ok";
    case LSTM_INVALID_ARG: return "invalid argument (non-positive dimension, NULL or misaligned pointer, bad flags)";
    case LSTM_BUFFER_TOO_SMALL: return "workspace smaller than lstm_workspace_bytes()";
    case LSTM_HIP_ERROR: return "HIP runtime error (see lstm_last_error())";
    case LSTM_INTERNAL: return "internal error: a kernel's bounded wait expired";
    case LSTM_UNSUPPORTED: return "the forced path does not support this shape on this device";
    default: return "unknown status";
  }
}

const char* lstm_last_error(void) { return g_last_error.c_str(); }

void lstm_shutdown(void) {
  {
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    for (bool& v : g_init_done) v = false;   // the watchdog word and the chain events are released below
  }
  release_helpers();
  clear_path_overrides();
  reset_knobs();
}

void lstm_debug_set_trace(void* device_buf, size_t bytes, int block) { set_trace(device_buf, bytes, block); }

void lstm_profile_enable(int on) { g_prof_on = on != 0; }

const char* lstm_profile_kernel(int phase) {
  return (phase >= 0 && phase < LSTM_PHASE_COUNT && g_prof_kernel[phase]) ? g_prof_kernel[phase] : "";
}

int lstm_profile_read(float* ms, int* count, double* flops) {
  if (!ms || !count) return LSTM_INVALID_ARG;
  for (int i = 0; i < LSTM_PHASE_COUNT; ++i) {
    ms[i] = 0.f;
    count[i] = 0;
    if (flops) flops[i] = 0.0;
  }
  int status = LSTM_OK;
  for (auto& iv : g_prof) {
    float t = 0.f;
    if (!iv.open && hipEventSynchronize(iv.stop) == hipSuccess && hipEventElapsedTime(&t, iv.start, iv.stop) == hipSuccess) {
      if (iv.phase >= 0 && iv.phase < LSTM_PHASE_COUNT) {
        ms[iv.phase] += t;
        count[iv.phase] += 1;
        if (flops) flops[iv.phase] += iv.flops;
      }
    } else {
      (void)hipGetLastError();
      status = LSTM_HIP_ERROR;
    }
    (void)hipEventDestroy(iv.start);
    (void)hipEventDestroy(iv.stop);
  }
  g_prof.clear();
  return status;
}

const char* lstm_phase_name(int phase) {
  static const char* names[LSTM_PHASE_COUNT] = {"fwd_pack",       "fwd_input_gemm", "fwd_recurrence", "bwd_pack",
                                                "bwd_recurrence", "bwd_input_gemm", "weight_grad",    "bias_grad"};
  return (phase >= 0 && phase < LSTM_PHASE_COUNT) ? names[phase] : "unknown";
}

unsigned lstm_auto_path(int L, int T, int B, int I, int H, int backward) {
  if (!dims_ok(L, T, B, I, H)) return LSTM_PATH_AUTO;
  return resolve_auto_path(Dims{L, T, B, I, H}, backward != 0);
}

int lstm_set_path(int L, int T, int B, int I, int H, int backward, unsigned path) {
  if (!dims_ok(L, T, B, I, H)) return LSTM_INVALID_ARG;
  return set_path_override(Dims{L, T, B, I, H}, backward != 0, path);
}

int lstm_set_wavefront_chunks(int L, int T, int B, int I, int H, int chunks) {
  if (!dims_ok(L, T, B, I, H)) return LSTM_INVALID_ARG;
  return set_wavefront_chunks(Dims{L, T, B, I, H}, chunks);
}

int lstm_gemm_f32(int M, int N, int K, const float* A, long sAm, long sAk, const float* B, long sBk, long sBn,
                  float* C, long ldc, int accumulate, void* stream) {
  if (M <= 0 || N <= 0 || K <= 0 || !A || !B || !C || ldc < N) return LSTM_INVALID_ARG;
  if ((sAm != 1 && sAk != 1) || (sBk != 1 && sBn != 1)) return LSTM_INVALID_ARG;
  GemmProblem p{A, B, C, M, N, K, sAm, sAk, sBk, sBn, ldc, accumulate};
  if (record(launch_gemm_group(&p, 1, (hipStream_t)stream), "gemm launch") != hipSuccess) return LSTM_HIP_ERROR;
  return LSTM_OK;
}

int lstm_gemm_f32_ws(int M, int N, int K, const float* A, long sAm, long sAk, const float* B, long sBk, long sBn,
                     float* C, long ldc, int accumulate, void* scratch, size_t scratch_bytes, void* stream) {
  if (M <= 0 || N <= 0 || K <= 0 || !A || !B || !C || ldc < N) return LSTM_INVALID_ARG;
  if ((sAm != 1 && sAk != 1) || (sBk != 1 && sBn != 1)) return LSTM_INVALID_ARG;
  if (scratch && (reinterpret_cast<uintptr_t>(scratch) & 15u) != 0) return LSTM_INVALID_ARG;
  GemmProblem p{A, B, C, M, N, K, sAm, sAk, sBk, sBn, ldc, accumulate};
  if (record(launch_gemm_split(p, (float*)scratch, scratch ? scratch_bytes : 0, (hipStream_t)stream), "gemm launch") != hipSuccess)
    return LSTM_HIP_ERROR;
  return LSTM_OK;
}

int lstm_init(void) {
  g_last_error.clear();
  void* p = nullptr;
  if (scratch_of_current_device(&p) != LSTM_OK) return LSTM_HIP_ERROR;
  if (record(setup_persistent(), "lstm_init: watchdog word / launch-chain event") != hipSuccess) return LSTM_HIP_ERROR;
  int dev = -1;
  if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64) {
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    g_init_done[dev] = true;
  }
  return LSTM_OK;
}

int lstm_forward_noalloc(int L, int T, int B, int I, int H, const float* x, const float* h0, const float* c0,
                         const float* W, const float* R, const float* b, float* y, float* hT, float* cT, void* reserve,
                         void* stream, unsigned flags) {
  g_last_error.clear();
  if (!dims_ok(L, T, B, I, H)) return LSTM_INVALID_ARG;
  if ((flags & LSTM_PATH_MASK) == LSTM_PATH_WAVEFRONT) return LSTM_UNSUPPORTED;  // that path creates helper streams sized by the shape
  const size_t need = lstm_workspace_bytes(L, T, B, I, H);
  if (need > kScratchBytes) {
    g_last_error = "lstm_forward_noalloc: this shape needs " + std::to_string(need) + " bytes of scratch, the static array holds " +
                   std::to_string(kScratchBytes);
    return LSTM_BUFFER_TOO_SMALL;
  }
  void* ws = nullptr;
  const int st = lstm_init_needed() ? lstm_init() : LSTM_OK;
  if (st != LSTM_OK) return st;
  if (scratch_of_current_device(&ws) != LSTM_OK) return LSTM_HIP_ERROR;
  return forward_call(L, T, B, I, H, x, h0, c0, W, R, b, y, hT, cT, reserve, ws, kScratchBytes, stream, flags, true);
}

int lstm_forward(int L, int T, int B, int I, int H, const float* x, const float* h0, const float* c0, const float* W,
                 const float* R, const float* b, float* y, float* hT, float* cT, void* reserve, void* workspace,
                 size_t workspace_bytes, void* stream, unsigned flags) {
  return forward_call(L, T, B, I, H, x, h0, c0, W, R, b, y, hT, cT, reserve, workspace, workspace_bytes, stream, flags, false);
}

}  // extern "C"

namespace {
// no_new_resources: the caller may create nothing (lstm_forward_noalloc); the stream wavefront, whose helper streams
// and events are created to the size of the shape, is then replaced by the step path.
int forward_call(int L, int T, int B, int I, int H, const float* x, const float* h0, const float* c0, const float* W,
                 const float* R, const float* b, float* y, float* hT, float* cT, void* reserve, void* workspace,
                 size_t workspace_bytes, void* stream, unsigned flags, bool no_new_resources) {
  g_last_error.clear();
  if (!dims_ok(L, T, B, I, H)) return LSTM_INVALID_ARG;
  if (!x || !W || !R || !b || !y || !workspace) return LSTM_INVALID_ARG;
  const void* ptrs[] = {x, h0, c0, W, R, b, y, hT, cT, reserve, workspace};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return LSTM_INVALID_ARG;
  if ((flags & ~LSTM_PATH_MASK) != 0 || (flags & LSTM_PATH_MASK) > LSTM_PATH_PERSISTENT) return LSTM_INVALID_ARG;
  const Dims d{L, T, B, I, H}, p = padded_dims(d);
  if (workspace_bytes < lstm_workspace_bytes(L, T, B, I, H)) return LSTM_BUFFER_TOO_SMALL;
  if (take_watchdog()) return LSTM_INTERNAL;  // an earlier call's persistent kernel gave up waiting: reported once, here
  if (p.H != d.H) {
    return forward_padded(d, p, x, h0, c0, W, R, b, y, hT, cT, reserve, (char*)workspace, (hipStream_t)stream, flags,
                          no_new_resources);
  }
  const WsLayout w = ws_layout(d);

  FwdArgs a{d, x, h0, c0, W, R, b, y, hT, cT,
            reserve ? (float*)reserve : (float*)((char*)workspace + w.resv), (char*)workspace, w, (hipStream_t)stream};
  a.inference = reserve == nullptr;
  unsigned path = flags & LSTM_PATH_MASK;
  if (path == LSTM_PATH_AUTO) path = resolve_auto_path(d, false);
  if (no_new_resources && path == LSTM_PATH_WAVEFRONT) path = LSTM_PATH_STEP;
  return run_forward(a, path);
}
}  // namespace

extern "C" {

int lstm_backward(int L, int T, int B, int I, int H, const float* x, const float* h0, const float* c0,
                  const float* W, const float* R, const void* reserve, const float* dy, const float* dhT,
                  const float* dcT, float* dx, float* dh0, float* dc0, float* dW, float* dR, float* db,
                  void* workspace, size_t workspace_bytes, void* stream, unsigned flags) {
  g_last_error.clear();
  if (!dims_ok(L, T, B, I, H)) return LSTM_INVALID_ARG;
  if (!x || !W || !R || !reserve || !dy || !dW || !dR || !db || !workspace) return LSTM_INVALID_ARG;
  const void* ptrs[] = {x, h0, c0, W, R, reserve, dy, dhT, dcT, dx, dh0, dc0, dW, dR, db, workspace};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return LSTM_INVALID_ARG;
  if ((flags & ~LSTM_PATH_MASK) != 0 || (flags & LSTM_PATH_MASK) > LSTM_PATH_PERSISTENT) return LSTM_INVALID_ARG;
  const Dims d{L, T, B, I, H}, p = padded_dims(d);
  if (workspace_bytes < lstm_workspace_bytes(L, T, B, I, H)) return LSTM_BUFFER_TOO_SMALL;
  if (take_watchdog()) return LSTM_INTERNAL;  // an earlier call's persistent kernel gave up waiting: reported once, here
  if (p.H != d.H) {
    return backward_padded(d, p, x, h0, c0, W, R, reserve, dy, dhT, dcT, dx, dh0, dc0, dW, dR, db, (char*)workspace,
                           (hipStream_t)stream, flags);
  }
  const WsLayout w = ws_layout(d);

  BwdArgs a{d, x, h0, c0, W, R, (const float*)reserve, dy, dhT, dcT, dx, dh0, dc0, dW, dR, db,
            (char*)workspace, w, (hipStream_t)stream};
  unsigned path = flags & LSTM_PATH_MASK;
  if (path == LSTM_PATH_AUTO) path = resolve_auto_path(d, true);
  return run_backward(a, path);
}

}  // extern "C"
