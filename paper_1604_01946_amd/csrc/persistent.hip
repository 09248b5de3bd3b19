// Persistent recurrence: the whole T-step, L-layer recurrence in ONE
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
// This file is the host side: device properties, the watchdog word, how persistent kernels are launched so that
// they are resident, which shapes run on which kernel family, groups of layers for stacks deeper than the chip
// holds, batch slices.  The kernels are in persistent_narrow / _wide / _pp / _large.hip (see persistent.h).
#include "../../include/lstm.h"
#include "persistent.h"
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

}  // namespace

// Raises a kernel's dynamic LDS limit once per process (`done` is the caller's flag for that kernel); callers on
// several host threads are serialised.
hipError_t allow_dynamic_lds(const void* fn, size_t smem, bool& done) {
  std::lock_guard<std::mutex> lk(g_launch_mu);
  if (done) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e == hipSuccess) done = true;
  return e;
}

hipError_t launch_resident(const void* fn, int grid, void** params, unsigned smem, hipStream_t s, int threads) {
  if (knobs().coop_launch) return hipLaunchCooperativeKernel(fn, dim3(grid), dim3(threads), params, smem, s);
  int dev = 0;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (knobs().plain_launch || hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16 ||
      hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
    (void)hipGetLastError();
    return hipLaunchKernel(fn, dim3(grid), dim3(threads), params, smem, s);  // (a stream under capture is ordered by its graph)
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
  st = hipLaunchKernel(fn, dim3(grid), dim3(threads), params, smem, s);
  if (st != hipSuccess) return st;
  g_last_launch_recorded[dev] = true;
  return hipEventRecord(g_last_launch[dev], s);
}

namespace {

BatchPlan batch_plan(int B) {
  const bool two = knobs().two_chains;
  if (B <= 16) return {1, 1};
  if (B <= 32) return two ? BatchPlan{1, 2} : BatchPlan{2, 1};
  return two ? BatchPlan{2, 2} : BatchPlan{4, 1};
}



// The wide-batch forward kernel (32x32x2 MFMA, two batch tiles of 32).
// Height of the batch slices (16 or 32 rows) that run side by side on the narrow kernels, or 0 where the batch is
// taken whole (B <= 16, or no room) or by the wide kernels.  While all slices fit the chip in one launch the narrow
// kernels are the faster ones: a step's matrix work per workgroup shrinks with the slice and more CUs share it (one or
// two layers at H = 512, up to four at H = 256; L = 1, H = 512, B = 64, T = 100: forward recurrence 0.40 ms on four
// slices of 16 rows, 0.53 on two of 32, 0.74 on the wide kernel; backward 0.65 against 1.14).  `env` names the
// setting that pins the choice (LSTM_FWD_NARROW / LSTM_BWD_NARROW): 1 = one slice on the narrow kernel (B <= 64), 0 = never slices.
// Backward, from H = 256 on, slices of 32 rows lose to the kernel with two alternating chains per slice of 64 rows
// (whole iterations, T = 100: L = 2, H = 512, B = 64 2.46 -> 2.28 ms; L = 4, H = 256, B = 64 1.46 -> 1.37; L = 2, H = 256,
// B = 128 1.55 -> 1.44), while slices of 16 rows stay ahead of it (L = 1, H = 512, B = 64 1.40 against 2.02 ms).
int narrow_slice_rows(const Dims& d, int cell, int pinned, bool backward) {
  if (cell != 0) return 0;  // the narrow kernels are LSTM kernels
  if (pinned >= 0 || knobs().two_chains) return 0;
  DeviceInfo di;
  if (!device_info(di)) return 0;
  for (int rows = 16; rows <= 32; rows *= 2) {
    if (backward && rows == 32 && d.H >= 256) break;
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


// A single sequence: the kernels of persistent_tiny.hip (one wave per two hidden units, 32 workgroups per layer, all
// of them resident).
bool tiny_path(const Dims& d, int cell) {
  if (cell != 0 || d.B != 1 || !knobs().tiny) return false;
  if (!(d.H == 128 || d.H == 256 || d.H == 512)) return false;
  DeviceInfo di;
  return device_info(di) && 32L * d.L <= di.cus;  // 32 workgroups per layer, one per CU
}

// The wide-batch backward kernel: two batch halves, 16 hidden units per workgroup.
bool bwd_wide(const Dims& d) {
  if (d.B > 64) return true;
  if (knobs().bwd_narrow == 1) return false;
  return d.B > 32;
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
// measured faster than the GEMM rung forward with the step kernels backward up to here (L = 1 / L = 4: 108 / 104 against
// 106 / 102 TFLOP/s at B = 768; 108 / 103 against 116 / 110 at B = 1024).
constexpr int kLargeMaxBatch1024 = 768;
// At H = 2048 one slice of 32 rows fills the chip: larger batches run slice after slice, at a constant 5.55 ms per slice
// and 100 steps (116-119 TFLOP/s for forward, backward and weight gradients together).  The step kernels and GEMM
// rungs, which stream R once per step for the whole batch, gain with the batch: 96 TFLOP/s at 192 rows, 110 at 256,
// 107 at 384, 121 at 512.
constexpr int kLargeMaxBatch2048 = 448;

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
  // Slices of 64 rows, one after the other once the chip is full: the rate does not depend on their number (L = 4,
  // H = 512: 110 TFLOP/s at 2048 rows), and the GEMM rungs never catch up (84-90 TFLOP/s at 4096 and 8192 rows; H = 256:
  // 85 against 64-71; H = 128: 45 against 33-37).  The limit only bounds the number of launches of one call.
  if (d.B > 16384) return false;
  DeviceInfo di;
  if (!device_info(di) || !di.coop) return false;
  return d.H / 8 <= di.cus;  // deeper stacks than the chip holds run as groups of layers (run_forward_persistent)
}

namespace {



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
  const bool lpp = (cell == 0 || knobs().rnn_pp) && d.H == 2048 && knobs().large_pp;  // the LSTM at H = 2048: two alternating chains of 16 rows per slice
  for (int l = 0; l < d.L; ++l) {
    const int Il = in_dim(d, l);
    const float* in = l == 0 ? a.x : a.reserve + (size_t)(l - 1) * rstride + res_h_offset(cell, TB, d.H);
    const float* Wl = a.W + (l == 0 ? 0 : G * d.I + (size_t)(l - 1) * G * d.H);
    {
      ProfScope ps(LSTM_PHASE_FWD_INPUT_GEMM, s);
      GemmProblem p{in, Wl, P, (int)TB, (int)G, Il, Il, 1, 1, Il, (long)G, 0};
      // (the exchange area is idle between two recurrences: it takes the partial tiles)
      CK(launch_gemm_split(p, hx, a.w.flags - a.w.xchg, s), "input projection GEMM");
    }
   for (int s0 = 0; s0 < slices; s0 += cap) {
    const int nsl = slices - s0 < cap ? slices - s0 : cap;
    {
      ProfScope ps(LSTM_PHASE_FWD_PACK, s);
      const size_t counter_ints = lpp ? fwdLpp_flag_ints() : (size_t)16 * kFlagStride;
      CK(launch_fill_zero(flags, (size_t)nsl * (d.T + 1) * counter_ints * 4, s), "zero step counters");
      if (lpp) CK(launch_pack_stateLpp(a.h0 ? a.h0 + (size_t)l * BH : nullptr, hx, d.T, d.B, d.H, 32 * s0, nsl, s), "pack h0");
      else CK(launch_pack_stateL(a.h0 ? a.h0 + (size_t)l * BH : nullptr, hx, d.T, d.B, d.H, 32 * s0, nsl, s), "pack h0");
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
    k.trace = (g_trace_bytes >= (size_t)d.T * 64 * (lpp ? 2 : 1)) ? g_trace_buf : nullptr;
    k.trace_block = g_trace_block;
    ProfScope ps(LSTM_PHASE_FWD_RECURRENCE, s);
    prof_flops(2.0 * G * d.H * std::min(32 * nsl, d.B - 32 * s0) * d.T, lpp ? "pers_fwdLpp_kernel" : "pers_fwdL_kernel");
    if (lpp) CK(launch_fwdLpp(cell, d.H, k, s), "persistent forward launch (large H, alternating chains)");
    else CK(launch_fwdL_any(d.H, cell, k, s), "persistent forward launch (large H)");
   }
  }
  return LSTM_OK;
}


}  // namespace

int weight_gradients(const BwdArgs& a, const float* dA_all, bool grouped, bool bias_done);

namespace {

// Backward pass of the large-H shapes: per layer (top down) one persistent launch for the recurrence, then
// the batched product that hands the gradient to the layer below; weight gradients at the end.

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
  // A single slice at H = 1024 would occupy 64 CUs: the tiles' K is cut in four, 256 workgroups (LSTM_LARGE_KSPLIT=0:
  // not); two slices of a single layer cut it in two (with more layers the idle CUs are used by the weight gradients
  // of the layer above, which is worth more: L = 4, B = 64).
  const int ks = (d.H != 1024 || !knobs().large_ksplit) ? 1 : (slices == 1 ? (d.L > 1 ? 2 : 4) : ((slices == 2 && d.L == 1) ? 2 : 1));
  // A launch that occupies at most half of the CUs (H = 1024 with one or two slices) leaves room for the weight
  // gradients of the layer above, which are complete once that layer's recurrence is: they run on a side stream
  // while this layer's recurrence runs (Section 2.6 wants them after the propagation of *their* layer, not of all
  // layers).  The side stream starts them behind the counter reset that precedes the persistent launch, so that the
  // launch gets its CUs first and the products fill the rest.  LSTM_NO_WGRAD_OVERLAP=1 keeps one stream.
  bool overlap = (cell == 0 || lg) && d.L > 1 && 2 * maxsl * NBK * NBK * ks <= di.cus && slices <= cap;
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
      k.T = d.T; k.B = d.B; k.b0 = 32 * s0; k.nsl = nsl; k.ks = ks; k.spin_limit = spin_limit(); k.full_fences = full_fences();
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
      CK(launch_gemm_split(p, reinterpret_cast<float*>(a.ws + a.w.xchg), a.w.flags - a.w.xchg, s), "input-gradient GEMM");
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
  if (d.B > 16384) return false;  // (the cells' own limits are lower: rnn_cells.hip)
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
  const int slice_rows_narrow = narrow_slice_rows(d, cell, knobs().fwd_narrow, false);
  const bool narrow_slices = slice_rows_narrow > 0;
  const BatchPlan bp = narrow_slices ? BatchPlan{slice_rows_narrow / 16, 1} : batch_plan(d.B);
  const int BP = 16 * bp.NT;
  const bool wide = cell != 0 || (!narrow_slices && fwd_wide(d));
  float* hx = reinterpret_cast<float*>(a.ws + a.w.xchg);
  int* flags = reinterpret_cast<int*>(a.ws + a.w.flags);
  float* P0 = reinterpret_cast<float*>(a.ws + a.w.P);
  if (tiny_path(d, cell)) {
    {
      ProfScope ps(LSTM_PHASE_FWD_INPUT_GEMM, s);
      GemmProblem p{a.x, a.W, P0, (int)TB, (int)G, d.I, d.I, 1, 1, d.I, (long)G, 0};
      CK(launch_gemm_group(&p, 1, s), "input projection GEMM (layer 0)");
    }
    PersFwdArgs k{};
    k.W = a.W; k.R = a.R; k.bias = a.b; k.P0 = P0; k.c0 = a.c0; k.h0 = a.h0; k.hx = hx; k.watchdog = g_watch_dev;
    k.res = a.reserve; k.y = a.y; k.hT = a.hT; k.cT = a.cT;
    k.L = d.L; k.T = d.T; k.B = d.B; k.I = d.I; k.H = d.H; k.spin_limit = spin_limit();
    k.trace = (g_trace_bytes >= (size_t)d.T * 64) ? g_trace_buf : nullptr;
    k.trace_block = g_trace_block;
    ProfScope ps(LSTM_PHASE_FWD_RECURRENCE, s);
    prof_flops(2.0 * G * d.T * d.H * (2 * d.L - 1), "pers_fwd_tiny_kernel");
    CK(launch_fwd_tiny(d.H, k, s), "persistent forward launch (single sequence)");
    return LSTM_OK;
  }
  // Wide kernel with I == H: layer 0 multiplies by W_0 inside the kernel like the layers above it (its workgroups
  // are otherwise idle half of every step), reading x from a copy in exchange layout that takes the place of the
  // projection in the workspace.  LSTM_FWD_BATCHED_INPUT=1 keeps the batched product of Section 2.3 instead.
  // (Section 2.3 notes that batching the input products pays at some sizes and not at others; here the batched
  // product only wins where nothing would be idle otherwise: one layer, one slice -- by about 4 %.)
  // (the kernels with two alternating chains also take I < H: x zero-padded to H columns in that copy)
  const bool pp_ok = (cell == 0 || knobs().rnn_pp) && knobs().pingpong != 0;
  bool x_in_kernel = wide && (d.I == d.H || (pp_ok && d.I < d.H)) && !(d.L == 1 && d.B <= 64);
  if (x_in_kernel) {
    if (knobs().fwd_batched_input) x_in_kernel = false;
    const size_t rows = (size_t)(d.B + 63) / 64 * 64;  // the copy of x: T+1 slots of H x 64 per slice
    if (((size_t)d.T + 1) * rows * d.H > (size_t)d.L * TB * 4 * d.H) x_in_kernel = false;
  }
  // LSTM with every layer multiplying its input in the kernel: the two half-slices of 32 rows take turns inside the
  // waves (pers_fwd_pp_kernel); LSTM_PINGPONG=0 keeps the one-chain kernel
  const bool pp = x_in_kernel && pp_ok;
  if (!x_in_kernel) {
    ProfScope ps(LSTM_PHASE_FWD_INPUT_GEMM, s);
    GemmProblem p{a.x, a.W, P0, (int)TB, (int)G, d.I, d.I, 1, 1, d.I, (long)G, 0};
    CK(launch_gemm_group(&p, 1, s), "input projection GEMM (layer 0)");
  }
  PersFwdArgs k;
  k.xin = x_in_kernel ? P0 : nullptr;
  k.keep = a.inference ? 0 : 1;
  k.dummy = reinterpret_cast<float*>(a.ws + a.w.scratch);
  k.W = a.W; k.R = a.R; k.bias = a.b; k.P0 = P0; k.c0 = a.c0; k.h0 = a.h0; k.hx = hx; k.flags = flags; k.watchdog = g_watch_dev;
  k.res = a.reserve; k.y = a.y; k.hT = a.hT; k.cT = a.cT;
  k.L = d.L; k.T = d.T; k.B = d.B; k.I = d.I; k.H = d.H; k.has_h0 = a.h0 != nullptr; k.spin_limit = spin_limit();
  k.full_fences = full_fences();
  k.trace = (g_trace_bytes >= (size_t)d.T * 64 * (pp ? 2 : 1)) ? g_trace_buf : nullptr;
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
      const size_t counter_ints = pp ? (size_t)2 * (d.H / 16) * kFlagStride : (size_t)bp.NC * kFlagInts;
      CK(launch_fill_zero(flags, (size_t)nsl * d.L * (d.T + 1) * counter_ints * 4, s), "zero step counters");
      if (pp) {
        CK(launch_pack_state_pp(a.h0, hx, d.L, d.T, d.B, d.H, k.b0, nsl, s), "pack h0");
        if (x_in_kernel) CK(launch_pack_x_pp(a.x, P0, d.T, d.B, d.I, d.H, k.b0, nsl, s), "pack x");
      } else if (wide) {
        CK(launch_pack_state32(a.h0, hx, d.L, d.T, d.B, d.H, k.b0, nsl, s), "pack h0");
        if (x_in_kernel) {
          CK(launch_pack_x32(a.x, P0, flags, d.L, d.T, d.B, d.H, k.b0, nsl, d.H / 8, s), "pack x");
        }
      } else if (a.h0) {
        CK(launch_pack_state(a.h0, hx, d.L, d.T, d.B, d.H, BP, bp.NC, k.b0, nsl, s), "pack h0");
      }
    }
    ProfScope ps(LSTM_PHASE_FWD_RECURRENCE, s);
    {  // recurrent products of every layer, input products of the layers above the first, and layer 0's when x is multiplied in the kernel
      const double rows = std::min(slice_rows * nsl, d.B - k.b0), per = 2.0 * G * rows * d.T;
      prof_flops(per * d.H * (2 * d.L - 1) + (x_in_kernel ? per * d.I : 0.0),
                 pp ? "pers_fwd_pp_kernel" : (wide ? "pers_fwd32_kernel" : "pers_fwd_kernel"));
    }
    hipError_t e = hipErrorInvalidValue;
    if (pp) e = launch_fwd_pp(cell, d.H, grid * nsl, k, s);
    else if (wide) e = launch_fwd_wide(cell, d.H, grid * nsl, k, s);
    else e = launch_fwd_narrow(d.H, bp, grid * nsl, k, s);
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
  const int slice_rows_narrow = narrow_slice_rows(d, cell, knobs().bwd_narrow, true);
  const bool narrow_slices = slice_rows_narrow > 0;
  const BatchPlan bp = narrow_slices ? BatchPlan{slice_rows_narrow / 16, 1} : batch_plan(d.B);
  const bool wide = cell != 0 || (!narrow_slices && bwd_wide(d));
  int* flags = reinterpret_cast<int*>(a.ws + a.w.flags);
  float* dA = reinterpret_cast<float*>(a.ws + a.w.P);
  if (tiny_path(d, cell)) {
    PersBwdArgs k{};
    k.W = a.W; k.R = a.R; k.res = a.reserve; k.c0 = a.c0; k.dy = a.dy; k.dhT = a.dhT; k.dcT = a.dcT;
    k.dA = dA; k.dAx = reinterpret_cast<float*>(a.ws + a.w.xchg); k.dxbuf = reinterpret_cast<float*>(a.ws + a.w.dx);
    k.dh0 = a.dh0; k.dc0 = a.dc0; k.watchdog = g_watch_dev;
    k.dx0 = (a.dx && d.I == d.H) ? a.dx : nullptr;
    k.db = a.db;  // every element written by the one lane that owns the unit
    k.L = d.L; k.T = d.T; k.B = d.B; k.I = d.I; k.H = d.H; k.spin_limit = spin_limit();
    k.trace = (g_trace_bytes >= (size_t)d.T * 64) ? g_trace_buf : nullptr;
    k.trace_block = g_trace_block;
    {
      ProfScope ps(LSTM_PHASE_BWD_RECURRENCE, s);
      const double per = 2.0 * G * d.T;
      prof_flops(per * d.H * (2 * d.L - 1) + (k.dx0 ? per * d.I : 0.0), "pers_bwd_tiny_kernel");
      CK(launch_bwd_tiny(d.H, k, s), "persistent backward launch (single sequence)");
    }
    if (a.dx && !k.dx0) {  // layer 0's input gradient: all T steps in one product
      ProfScope ps(LSTM_PHASE_BWD_INPUT_GEMM, s);
      GemmProblem p{dA, a.W, a.dx, (int)TB, d.I, (int)GW, (long)G, 1, d.I, 1, d.I, 0};
      CK(launch_gemm_group(&p, 1, s), "input-gradient GEMM (layer 0)");
    }
    if (bias_done) *bias_done = a.db != nullptr;
    if (!with_weight_gradients) return LSTM_OK;
    return weight_gradients(a, dA, true, a.db != nullptr);
  }
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
  // two alternating chains per workgroup (LSTM, slices of 64 rows): counters of H/16 lines per (layer, step, quarter)
  const bool pp = wide && (cell == 0 || knobs().rnn_pp) && knobs().pingpong != 0;
  k.dummy = reinterpret_cast<float*>(a.ws + a.w.scratch);
  k.trace = (g_trace_bytes >= (size_t)d.T * 64 * (pp ? 2 : 1)) ? g_trace_buf : nullptr;
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
      const size_t per_slot = pp ? (size_t)4 * (d.H / 16) * kFlagStride : (size_t)2 * kFlagInts;  // ints per (slice, layer, step)
      CK(launch_fill_zero(flags, (size_t)nsl * d.L * (d.T + 2) * per_slot * 4, s), "zero step counters");
    }
    ProfScope ps(LSTM_PHASE_BWD_RECURRENCE, s);
    {  // dh products of every layer, dx products of the layers above the first, and layer 0's when the kernel writes dx itself
      const double rows = std::min(slice_rows * nsl, d.B - k.b0), per = 2.0 * GW * rows * d.T;
      prof_flops(per * d.H * (2 * d.L - 1) + (k.dx0 ? per * d.I : 0.0), pp ? "pers_bwd_pp_kernel" : (wide ? "pers_bwd32_kernel" : "pers_bwd_kernel"));
    }
    hipError_t e = hipErrorInvalidValue;
    if (pp) e = launch_bwd_pp(cell, d.H, k, 2 * nsl, s);
    else if (wide) e = launch_bwd_wide(cell, d.H, k, 2 * nsl, s);
    else e = launch_bwd_narrow(d.H, bp, grid * nsl, k, s);
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
