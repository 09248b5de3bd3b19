// Persistent recurrence kernels: what the kernel translation units and the host-side dispatch share -- the kernel
// argument blocks, the layout constants of the step counters, and the launch functions of every kernel family.
// (Section 4 of arXiv 1604.01946 names the idea: the recurrent weights are reused by every step and could stay in a
// lower level of the memory hierarchy for the whole sequence, at the price of a capacity limit and of workgroups that
// are all resident and wait on each other.)
//   persistent_dev.h      device helpers: bounded waits, signals, write-through stores
//   persistent_narrow.hip pers_fwd_kernel / pers_bwd_kernel: tiles of 16 batch rows (B <= 32, slices of 16 / 32 rows)
//   persistent_wide.hip   pers_fwd32_kernel / pers_bwd32_kernel: slices of 64 rows, 32x32x2 tiles, templated on the cell
//   persistent_pp.hip     pers_fwd_pp_kernel: two half-slices of 32 rows alternating on the matrix cores
//   persistent_bpp.hip    pers_bwd_pp_kernel: two quarter-slices of 16 rows alternating on the matrix cores
//   persistent_tiny.hip   pers_fwd_tiny_kernel / pers_bwd_tiny_kernel: B = 1, the exchanged values are their own flags
//   persistent_large.hip  pers_fwdL_kernel / pers_bwdL_kernel: one layer per launch, H = 1024 / 2048
//   persistent_large_pp.hip  pers_fwdLpp_kernel: the LSTM forward kernel of H = 2048 with two alternating chains per slice
//   persistent.hip        host side: residency, launches, which shapes run where, layer groups, batch slices
#pragma once
#include "schedule.h"

namespace lstm {

// A step counter is split into kFlagSub words, each on a cache line of its own (kFlagStride ints
// apart).  Agent-scope atomics from many workgroups on one line are served one after the other by the
// memory side, about 25 ns each (6.4 us for 256 arrivals on one line, measured), so arrivals are spread
// over the lines by slice index and a waiter reads all of them with one load (lane i reads word i).
constexpr int kFlagStride = 32;
constexpr int kFlagSub = 8;
constexpr int kFlagInts = kFlagSub * kFlagStride;  // ints per counter

struct PersFwdArgs {
  const float* W;     // flat input matrices; layers >= 1 are read
  const float* R;     // [L][4H][H]
  const float* bias;  // [L][4H]
  const float* P0;    // [T][B][4H] input projection of layer 0 (batched GEMM before the launch), unless xin is set
  const float* xin;   // wide kernel, I == H: x in exchange layout, [nsl][T+1][H*64] with slot t+1 = x_t; layer 0 then
                      // multiplies by W_0 itself, step by step, like the layers above it
  const float* c0;    // [L][B][H] or null
  const float* h0;    // [L][B][H] or null: read by the GRU variant of the wide kernel (its cell update needs h_{t-1})
  float* hx;          // [L][T+1][NC][H][BP] exchange, slot t+1 = h_t, slot 0 = h0
  int* flags;         // [L][T+1][NC], slot t+1 counts the slices of layer l that finished step t
  int* watchdog;
  float* res;         // reserve base
  float* y;
  float* hT;
  float* cT;
  int L, T, B, I, H;
  int b0;             // wide kernel: first batch row of this launch (a multiple of 64)
  int nsl;            // wide kernel: batch slices of 64 rows that run side by side in this launch (grid = nsl * L * H/8)
  int has_h0;
  int spin_limit;
  int full_fences;
  long long* trace;
  int trace_block;
  int keep;           // wide kernel: 0 = inference call (no reserve wanted): only y, hT, cT are written
  float* dummy;       // pers_fwd_pp_kernel: 128 bytes of scratch that take the stores nobody wants
};

// ------------------------------------------------------------------ backward
// Workgroup (l, s) owns hidden units u0..u0+7 of layer l.  Per step t (descending) and batch chain:
//   point-wise   dh_t = dout_t + dh_rec,  gate gradients dA_t (4 x 8 x BP values), dc carry;
//                dA_t goes to the standard [T][B][4H] array (weight-gradient GEMMs) and, k-major
//                ([4H][BP]), to the exchange buffer;
//   GEMM         [dh_rec_{t-1} ; dx_{l,t}] (16 rows) = [R_l[:, units] | W_l[:, units]]^T * dA_t, K = 4H:
//                rows 0-7 stay in registers for the next point-wise step, rows 8-15 are the gradient
//                for the same units of layer l-1 at step t (its dout) and go to dxbuf; for layer 0 they
//                are the gradient of the network input and go to the caller's dx when I == H (the
//                tile rows would otherwise multiply zeros), else a batched GEMM follows the launch.
// Section 2.1's remark on the backward pass (four gate gradients map to one output through the
// stacked matrices) is the K = 4H contraction; wave w takes the K range of gate w.
// Counters: slot t+1 of layer l = "point-wise of step t published" (which, by program order, also
// covers dx of step t+1); slot 0 = "dx of step 0 published".
struct PersBwdArgs {
  const float* W;      // flat input matrices (layer 0's only when dx0 is set)
  const float* R;      // [L][4H][H]
  const float* res;    // reserve written by the forward pass
  const float* c0;     // [L][B][H] or null
  const float* dy;     // [T][B][H]
  const float* dhT;    // [L][B][H] or null
  const float* dcT;    // [L][B][H] or null
  float* dA;           // [L][T][B][4H] gate gradients (standard layout)
  float* dAx;          // [L][T][NC][4H][BP] exchange
  float* dxbuf;        // [L][T][B][H] gradient for the layer below (slice l written by layer l, l >= 1)
  float* dx0;          // [T][B][I] gradient of the network input, written by layer 0 when I == H; else null
  float* dh0;          // [L][B][H] or null
  float* dc0;          // [L][B][H] or null
  float* db;           // [L][4H] bias gradient, zeroed before the launch (wide kernel only), or null
  int* flags;          // [L][T+1][NC]
  int* watchdog;
  int L, T, B, I, H;
  int b0;              // first batch row of this launch (a multiple of the slice height)
  int spin_limit;
  int full_fences;
  long long* trace;
  int trace_block;
  const float* h0;     // [L][B][H] or null: read by the GRU variant of the wide kernel
  float* dummy;        // pers_bwd_pp_kernel: 128 bytes of scratch that take the stores nobody wants
};

// Exchange layout of a slot (H x 32 floats): for k = wave*H/4 + 8*k8 + 2*m + kk and batch row n,
// element (wave*H/32 + k8)*256 + ((kk*32 + n)*4 + m) -- the 8 units of slice s are one contiguous KB.
struct PersFwdLArgs {
  const float* R;     // [4H][H] of this layer
  const float* bias;  // [4H]
  const float* P;     // [T][B][4H] input projection of this layer
  const float* c0;    // [B][H] or null
  float* hx;          // [T+1][H*32] exchange, slot t+1 = h_t, slot 0 = h0 (or zeros)
  int* flags;         // [T+1][16][kFlagStride]: slot t+1 counts the slices that published h_t, spread over 16 lines
  int* watchdog;
  float* res;         // reserve of this layer
  float* y;           // [T][B][H] or null (top layer only)
  float* hT;          // [B][H] or null
  float* cT;          // [B][H] or null
  int T, B;
  int b0;             // first batch row of this launch (a multiple of 32)
  int nsl;            // batch slices of 32 rows side by side in this launch (grid = nsl * H/8), each with its own
                      // exchange slots and counters
  int spin_limit;
  int full_fences;
  long long* trace;
  int trace_block;
};

struct PersBwdLArgs {
  const float* R;      // [4H][H] of this layer
  const float* res;    // reserve of this layer
  const float* c0;     // [B][H] or null
  const float* dout;   // [T][B][H]: dy (top layer) or the gradient handed down by the layer above
  const float* dhT;    // [B][H] or null
  const float* dcT;    // [B][H] or null
  float* dA;           // [T][B][4H] gate gradients (standard layout)
  float* X;            // [nsl][T][NBK][4*UB*32] exchange
  float* Pp;           // [nsl][T][NBK][NBK * ks][UB*32] partial sums
  float* dh0;          // [B][H] or null
  float* dc0;          // [B][H] or null
  float* db;           // [4H] or null (must be null when the batch has more than one slice: column sums follow instead)
  int* flagsA;         // [nsl][T][NBK] counters: gate gradients of (step, unit block) published
  int* flagsP;         // [nsl][T][NBK] counters: partial sums of (step, output block) published
  int* watchdog;
  int T, B;
  int b0;              // first batch row of this launch (a multiple of 32)
  int nsl;             // batch slices side by side in this launch (grid = nsl * NBK * NBK * ks)
  int ks;              // parts that a tile's K is cut into, each on a workgroup of its own: 1, or 4 (H = 1024, one slice)
  int spin_limit;
  int full_fences;
  long long* trace;
  int trace_block;
};

// Batch tiles per chain and number of chains.  One chain is the default: on MI355X two chains
// measured slower at B = 64 (the step is bound by MFMA issue forward and by L2->CU bandwidth
// backward, and half-width 8-byte exchange loads are less efficient); LSTM_CHAINS=2 selects two.
struct BatchPlan {
  int NT, NC;
};

// ---- launches (each in the translation unit of its kernels) ---------------------------------------------------
// All workgroups of a persistent kernel must be resident at once: launch_resident (persistent.hip) is the one way
// they are launched; allow_dynamic_lds raises a kernel's dynamic LDS limit once (`done` is the caller's flag).
hipError_t launch_resident(const void* fn, int grid, void** params, unsigned smem, hipStream_t s, int threads = 256);
hipError_t allow_dynamic_lds(const void* fn, size_t smem, bool& done);

hipError_t launch_fwd_narrow(int H, BatchPlan bp, int grid, const PersFwdArgs& a, hipStream_t s);
hipError_t launch_bwd_narrow(int H, BatchPlan bp, int grid, const PersBwdArgs& a, hipStream_t s);
hipError_t launch_pack_state(const float* h0, float* hx, int L, int T, int B, int H, int BP, int NC, int b0, int nsl, hipStream_t s);

hipError_t launch_fwd_wide(int cell, int H, int grid, const PersFwdArgs& a, hipStream_t s);
hipError_t launch_bwd_wide(int cell, int H, const PersBwdArgs& a, int nbh, hipStream_t s);
hipError_t launch_pack_state32(const float* h0, float* hx, int L, int T, int B, int H, int b0, int nsl, hipStream_t s);
hipError_t launch_pack_x32(const float* x, float* xin, int* flags, int L, int T, int B, int H, int b0, int nsl, int ready, hipStream_t s);

// two half-slices of 32 rows alternating on the matrix cores (512 threads per workgroup; exchange slots and counters
// per chain, see persistent_pp.hip)
hipError_t launch_fwd_pp(int cell, int H, int grid, const PersFwdArgs& a, hipStream_t s);  // cell 0: LSTM, 1: GRU
hipError_t launch_pack_state_pp(const float* h0, float* hx, int L, int T, int B, int H, int b0, int nsl, hipStream_t s);
hipError_t launch_pack_x_pp(const float* x, float* xin, int T, int B, int I, int H, int b0, int nsl, hipStream_t s);

// backward counterpart: two chains of 16 rows per workgroup (batch half), 16x16x4 tiles; counters of H/16 lines per
// (layer, step, half, chain), see persistent_bpp.hip
hipError_t launch_bwd_pp(int cell, int H, const PersBwdArgs& a, int nbh, hipStream_t s);  // cell 0: LSTM, 1: GRU

// a single sequence (B = 1): one wave per two hidden units, the exchanged values are their own flags
// (persistent_tiny.hip); hx [L][T+1][H], dAx [L][T][4H], dxbuf [L][T][H]
hipError_t launch_fwd_tiny(int H, const PersFwdArgs& a, hipStream_t s);
hipError_t launch_bwd_tiny(int H, const PersBwdArgs& a, hipStream_t s);

hipError_t launch_fwdL_any(int H, int cell, const PersFwdLArgs& k, hipStream_t s);
hipError_t launch_bwdL_any(int H, int cell, const PersBwdLArgs& k, hipStream_t s);
hipError_t launch_pack_stateL(const float* h0, float* hx, int T, int B, int H, int b0, int nsl, hipStream_t s);
// persistent_large_pp.hip: the LSTM forward kernel of the same shapes with two alternating chains of 16 rows per slice
hipError_t launch_fwdLpp(int cell, int H, const PersFwdLArgs& k, hipStream_t s);  // cell: 0 LSTM, 1 GRU, 2 ReLU, 3 tanh
hipError_t launch_pack_stateLpp(const float* h0, float* hx, int T, int B, int H, int b0, int nsl, hipStream_t s);
size_t fwdLpp_flag_ints();  // counter ints per (slice, step)

}  // namespace lstm
