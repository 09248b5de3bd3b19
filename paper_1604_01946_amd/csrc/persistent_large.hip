// Persistent recurrence for large hidden sizes (H = 1024 / 2048): pers_fwdL_kernel and pers_bwdL_kernel, one layer
// per launch with the layer's recurrent matrix spread over all CUs (registers + LDS).
#include "../../include/lstm.h"
#include "persistent_dev.h"

namespace lstm {
namespace {

// ------------------------------------------------------------------ one layer, large hidden size
// Section 4 of arXiv 1604.01946 puts the limit of the persistent approach at the capacity of the
// on-chip memory.  On MI355X the 256 CUs together hold 128 MB of registers and 40 MB of LDS, so a
// whole [4H x H] recurrent matrix of H = 2048 (64 MiB) fits: every workgroup keeps the 32 rows of
// 8 hidden units (4 gates x 8 units x H floats = 256 KB) for all T steps, half of it in VGPRs and half
// in LDS, exactly the split of pers_bwd32_kernel.  One launch runs one layer (all CUs are needed for
// it, so the layers cannot overlap); the layer's input projection is a batched GEMM before it, as for
// layer 0 above.  Per step a workgroup multiplies its [32 x H] slice by h_{t-1} ([H x 32 batch rows],
// read from the exchange slot), K split over the four waves, and finalises 8 units x 32 batch rows.

// CELL as in pers_fwd32_kernel (0 LSTM, 1 GRU, 2 / 3 single gate with ReLU / tanh).  Only recurrent weights live here
// (the input projection P is a batched product), so the GRU's four row groups are r, z, an empty one and R_n, and P's
// third block (W_n x) is added in the epilogue; the single gate uses the first group alone.
template <int HH, int CELL>
__global__ __launch_bounds__(256) void pers_fwdL_kernel(const PersFwdLArgs a) {
  constexpr int H = HH, NG = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1), G = NG * H, NS = H / 8;  // G: rows of R, bias, P
  constexpr int NB8 = H / 32;                // 8-k groups per wave
  constexpr int KPW = H / 8;                 // k-pairs per wave
  constexpr int RP = KPW < 128 ? KPW : 128;  // k-pairs whose weights live in registers
  constexpr int LP = KPW - RP;               // k-pairs whose weights live in LDS
  constexpr int DEPTH = NB8 < 16 ? NB8 : 16;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* const part = smem;         // [4 waves][16 regs][64 lanes]
  float* const xs = smem + 4096;    // [256]: this step's h slice in exchange order
  float* const ro = smem + 4352;    // [6 arrays][32 batch rows][8 units]
  float* const wl = smem + 6144;    // [4 waves][LP][64 lanes]

  const int sl = blockIdx.x / NS, s = blockIdx.x % NS, u0 = 8 * s;
  const int T = a.T, B = a.B, b0 = a.b0 + 32 * sl;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kk = lane >> 5, n = lane & 31;
  const size_t TB = (size_t)T * B;
  // the waves read the slot in orders rotated against each other, in steps of four groups: the address of a request is
  // then a scalar base + the lane's fixed offset + an immediate (vector address arithmetic costs a wave that runs matrix
  // instructions back to back its full issue time, scalar arithmetic nothing)
  const int rot = 4 * (((int)(blockIdx.x >> 3) * (NB8 / 32 > 0 ? NB8 / 32 : 1) + 2 * __builtin_amdgcn_readfirstlane(wave)) & (NB8 / 4 - 1));
  float* const hx = a.hx + (size_t)sl * (T + 1) * H * 32;
  int* const flags = a.flags + (size_t)sl * (T + 1) * 16 * kFlagStride;

  // ---- weights: A operand row rho = lane%32 = (gate rho/8, unit rho%8); register / LDS entry i covers
  //      k = wave*H/4 + 8*((i/4 + rot) mod NB8) + 2*(i%4) + kk
  float wreg[RP];
  {
    const int grp = n >> 3;
    const int gate = CELL >= 2 ? 0 : ((CELL == 1 && grp == 3) ? 2 : grp);
    const bool live = CELL == 0 || (CELL == 1 ? grp != 2 : grp == 0);
    const float* src = a.R + ((size_t)gate * H + u0 + (n & 7)) * H + (size_t)wave * (H / 4) + kk;
#pragma unroll
    for (int i = 0; i < KPW; ++i) {
      const int k8 = ((i >> 2) + rot) & (NB8 - 1), m = i & 3;
      const float v = live ? src[8 * k8 + 2 * m] : 0.f;
      if (i < RP)
        wreg[i < RP ? i : 0] = v;
      else  // the four k-pairs of a group side by side: one 16-byte LDS read per group
        wl[(((size_t)wave * (LP / 4) + ((i - RP) >> 2)) * 64 + lane) * 4 + (i & 3)] = v;
    }
  }

  // ---- the cell this thread finalises: unit u0 + 4*kk + wave, batch row n (D register 4*gate + wave)
  const int uj = 4 * kk + wave;
  const int bb = b0 + n;  // batch row in the tensors
  const bool valid = bb < B;
  float c_state = (CELL <= 1 && valid && a.c0) ? a.c0[(size_t)bb * H + u0 + uj] : 0.f;  // c_{t-1} (LSTM), h_{t-1} (GRU: a.c0 = h0)
  float c_bias[4], pin[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    c_bias[g] = g < NG ? a.bias[g * H + u0 + uj] : 0.f;
    pin[g] = (valid && g < NG) ? a.P[(size_t)bb * G + g * H + u0 + uj] : 0.f;
  }
  float* const res_gates = CELL == 0 ? a.res : a.res + TB * H;  // the four saved arrays [T][B][4H] (LSTM, GRU)
  float* const res_c = a.res + TB * 4 * H;                       // LSTM only
  float* const res_h = CELL == 0 ? a.res + TB * 5 * H : a.res;
  auto slot = [&](int st) { return hx + (size_t)st * H * 32; };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2
  __syncthreads();                                    // LDS weights are in place

  int rv = rot;
  for (int t = 0; t < T; ++t) {
    tr.mark(t, 0);
    hide(rv);  // keeps the rotated offsets next to their loads
    // (the first look at the counter is held back: a poll that comes too early is in the way of the arrivals it waits
    // for.  L = 4, H = 1024, B = 32, T = 50: 1.31 ms without a pause, 1.23 with 512 cycles, 1.25 with 1024, 1.32 with 2048)
    __builtin_amdgcn_s_sleep(8);
    if (t > 0) w.template wait_split<16>(flags + (size_t)16 * kFlagStride * t, NS / 16);  // slot 0 was written before the launch
    tr.mark(t, 2);
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float pnx[4];
    {
      const char* const src = reinterpret_cast<const char*>(slot(t) + (size_t)__builtin_amdgcn_readfirstlane(wave) * NB8 * 256);
      floatx4 bv[NB8];
      floatx4 al[NB8];
      unsigned lo = lane * 16;  // met anew by the optimiser here and after every branch, so that it stays a 32-bit offset
      asm volatile("" : "+v"(lo));
      auto ldb = [&](int g) {
        const char* const sb = src + (size_t)(4 * (((g >> 2) + (rv >> 2)) & (NB8 / 4 - 1))) * 1024;
        bv[g] = *reinterpret_cast<const floatx4*>(sb + lo + (g & 3) * 1024);
      };
      auto ldw = [&](int g) {
        if (g * 4 >= RP) al[g] = *reinterpret_cast<const floatx4*>(wl + (((size_t)wave * (LP / 4) + (g - RP / 4)) * 64 + lane) * 4);
      };
#pragma unroll
      for (int g = 0; g < DEPTH; ++g) ldb(g);
      ldw(0);
      if (NB8 > 1) ldw(1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < NB8; ++g) {
        if (g + DEPTH < NB8) ldb(g + DEPTH);
        if (g + 2 < NB8) ldw(g + 2);
        if (g == NB8 - DEPTH) {  // next step's input projection, behind the last exchange load of this step
#pragma unroll
          for (int q = 0; q < 4; ++q)
            pnx[q] = (valid && t + 1 < T && q < NG) ? a.P[((size_t)(t + 1) * B + bb) * G + q * H + u0 + uj] : 0.f;
          lo = lane * 16;
          asm volatile("" : "+v"(lo));
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const int pr = g * 4 + m;
          const float av = (pr < RP) ? wreg[pr < RP ? pr : 0] : al[g][m];
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[g][m], acc, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) part[(wave * 16 + r) * 64 + lane] = acc[r];
    tr.mark(t, 3);
    __syncthreads();
    tr.mark(t, 4);
    float sg[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int r = 4 * g + wave;
      sg[g] = (part[(0 * 16 + r) * 64 + lane] + part[(1 * 16 + r) * 64 + lane]) +
              (part[(2 * 16 + r) * 64 + lane] + part[(3 * 16 + r) * 64 + lane]) + pin[g] + c_bias[g];
    }
    float gi, gf, go, gg, cv, hv;
    if (CELL == 0) {
      gi = sigmoidf_dev(sg[0]); gf = sigmoidf_dev(sg[1]); go = sigmoidf_dev(sg[2]); gg = tanhf_dev(sg[3]);
      cv = gf * c_state + gi * gg;
      hv = go * tanhf_dev(cv);
      c_state = cv;
    } else if (CELL == 1) {  // sg: r, z pre-activations; W_n x + b_n (from P: this group has no weights here); R_n h
      gi = sigmoidf_dev(sg[0]); gf = sigmoidf_dev(sg[1]);
      go = tanhf_dev(sg[2] + gi * sg[3]);
      gg = sg[3];
      hv = (1.f - gf) * go + gf * c_state;
      cv = 0.f;
      c_state = hv;
    } else {
      gi = gf = go = gg = cv = 0.f;
      hv = CELL == 3 ? tanhf_dev(sg[0]) : fmaxf(sg[0], 0.f);
    }
    xs[((uj & 1) * 32 + n) * 4 + (uj >> 1)] = valid ? hv : 0.f;
    __syncthreads();
    if (threadIdx.x < 64)
      xstore4(slot(t + 1) + (size_t)s * 256 + 4 * threadIdx.x, *reinterpret_cast<const floatx4*>(xs + 4 * threadIdx.x));
    tr.mark(t, 5);
    signal(flags + ((size_t)16 * (t + 1) + (s & 15)) * kFlagStride, a.full_fences);  // publish h_t (the barrier also protects `part` and `xs`)
    tr.mark(t, 6);
    // reserve and outputs: staged through LDS so that every store instruction writes 16-byte runs
    ro[(0 * 32 + n) * 8 + uj] = gi;
    ro[(1 * 32 + n) * 8 + uj] = gf;
    ro[(2 * 32 + n) * 8 + uj] = go;
    ro[(3 * 32 + n) * 8 + uj] = gg;
    ro[(4 * 32 + n) * 8 + uj] = cv;
    ro[(5 * 32 + n) * 8 + uj] = hv;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = threadIdx.x + 256 * i;  // (array 0..5, batch row, half of the 8 units)
      const int arr = idx >> 6, l2 = (idx >> 1) & 31, hf = idx & 1;
      const int b2 = b0 + l2;
      if (idx < 384 && b2 < B) {
        const floatx4 v = *reinterpret_cast<const floatx4*>(ro + (arr * 32 + l2) * 8 + 4 * hf);
        const size_t e = ((size_t)t * B + b2) * H + u0 + 4 * hf;
        if (arr < 4) {
          if (CELL <= 1) *reinterpret_cast<floatx4*>(res_gates + ((size_t)t * B + b2) * 4 * H + (size_t)arr * H + u0 + 4 * hf) = v;
        } else if (arr == 4) {
          if (CELL == 0) {
            *reinterpret_cast<floatx4*>(res_c + e) = v;
            if (t == T - 1 && a.cT) *reinterpret_cast<floatx4*>(a.cT + (size_t)b2 * H + u0 + 4 * hf) = v;
          }
        } else {
          *reinterpret_cast<floatx4*>(res_h + e) = v;
          if (a.y) *reinterpret_cast<floatx4*>(a.y + e) = v;
          if (t == T - 1 && a.hT) *reinterpret_cast<floatx4*>(a.hT + (size_t)b2 * H + u0 + 4 * hf) = v;
        }
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) pin[g] = pnx[g];
  }
}

// h0 [B][H] of one layer (zeros if null) -> exchange slot 0 of every slice in the layout of pers_fwdL_kernel, all 32 batch columns.
__global__ void pack_stateL_kernel(const float* __restrict__ h0, float* __restrict__ hx, int T, int B, int H, int b0,
                                   int nsl) {
  const long cnt = (long)nsl * 32 * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < cnt; e += (long)gridDim.x * blockDim.x) {
    const int k = (int)(e % H), lb = (int)((e / H) % 32), sl = (int)(e / ((long)H * 32));
    const int bb = b0 + 32 * sl + lb;
    const int wv = k / (H / 4), kr = k % (H / 4), k8 = kr >> 3, m = (kr >> 1) & 3, kk = kr & 1;
    hx[(size_t)sl * (T + 1) * H * 32 + ((size_t)wv * (H / 32) + k8) * 256 + (kk * 32 + lb) * 4 + m] =
        (h0 && bb < B) ? h0[(size_t)bb * H + k] : 0.f;
  }
}

// ------------------------------------------------------------------ one layer, large hidden size, backward
// dh_{t-1} = R^T dA_t has K = 4H, four times the forward product: slicing it by output units would make
// every workgroup read all of dA_t (1 MB per step at H = 2048).  The [4H x H] matrix is therefore cut in
// two dimensions, NBK x NBK tiles of [4*UB gate rows x UB output units] (UB = 128: tiles of 256 KB, half
// in VGPRs, half in LDS; 256 tiles at H = 2048, 64 at H = 1024).  Workgroup (i, j) multiplies the gate
// gradients of unit block i into a partial sum for the output units of block j; the NBK partial sums of a
// block are then added -- always in the order of i, so the result does not depend on arrival order -- by
// the same NBK workgroups, each taking UB/NBK of the block's 128 units (8 at H = 2048, 16 at H = 1024: one
// or two cells per thread), which also run the point-wise stage of the next step for those units and
// publish their gate gradients to the NBK workgroups (j, .) that consume unit block j.
// Per step: 64 KB of dA read and 16 KB of partial sums written per workgroup, two synchronisation
// hops of NBK arrivals each.  The gradient for the layer below is a batched GEMM after the launch.
// The batch runs in slices of 32 rows, each with its own workgroups, exchange buffers and counters; at
// H = 1024 four slices fit side by side on 256 CUs.
// Exchange layouts: dA_t of a unit block: [k8][(kk*32 + n)*4 + m] for k = 8*k8 + 2*m + kk, batch row n,
// where k8 = 4*(unit/8 within the block) + gate and k%8 = unit%8; partial sums: [unit in block][32].

// CELL as in pers_bwd32_kernel: the four K groups of a unit octet are the gradients with respect to the four gate
// pre-activations (LSTM); to the r and z pre-activations, W_n x + b_n and R_n h (GRU: the third has no weights here,
// dh_{t-1} also receives dh_t o z_t); to the one pre-activation (single gate).  For the other cells `res` is that
// cell's reserve, c0 carries h0, dcT / dc0 are unused, R and db have 3H or H rows.
// KS > 1 (a single slice at H = 1024, where NBK x NBK workgroups would leave three quarters of the CUs idle): the tile's
// K = 4*UB is cut into KS parts, each on a workgroup of its own (ks, i, j); a block's partial sums are then NBK * KS, and
// the workgroups with ks = 0 finalise as before while the others go straight on to wait for the next step's gradients.
template <int HH, int CELL, int KS>
__global__ __launch_bounds__(256) void pers_bwdL_kernel(const PersBwdLArgs a) {
  constexpr int H = HH, G = 4 * H, UB = 128, NBK = H / UB;
  constexpr int NG = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1);  // gate blocks of R and db
  constexpr int UF = UB / NBK;               // units a workgroup finalises: 8 or 16
  constexpr int CPT = UF / 8;                // cells per thread in the point-wise stage
  constexpr int NG8 = 4 * UB / 8 / KS;       // 8-k groups of this workgroup's part of the tile's K = 4*UB
  constexpr int KP = 4 * UB / 2 / KS;        // k-pairs; every wave runs all of them for its 32 output units
  constexpr int RP = KS > 1 ? KP : (UF == 16 ? 136 : 128);  // k-pairs with weights in registers (more where the staging arrays are larger)
  constexpr int LP = KP - RP;                // k-pairs with weights in LDS
  constexpr int DEPTH = NG8 < 16 ? NG8 : 16;
  constexpr int NPART = NBK * KS;            // partial sums of an output block
  constexpr int kPauseA = 16, kPauseP = 32;  // pauses before the first look at a counter, in units of 64 cycles
  static_assert(NBK % kFlagSub == 0, "arrivals must spread evenly over the counter lines");
  static_assert(UF == 8 || UF == 16, "one or two cells per thread");
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* const stage = smem;              // [UB][32] partial sums of this step; also the bias-gradient reduction
  float* const xsA = smem + 4096;         // [UF/8 octets][4 gates][256] gate gradients of the finalised units, exchange order
  float* const ro = xsA + 1024 * CPT;     // [4 gates][32 batch rows][UF units] the same in standard order
  float* const wl = ro + 128 * UF;        // [4 waves][LP][64 lanes]; 152 KB in all

  const int sl = blockIdx.x / (NBK * NBK * KS), bid = blockIdx.x % (NBK * NBK), ks = (blockIdx.x / (NBK * NBK)) % KS;
  const int i = bid / NBK, j = bid % NBK;
  const bool fin = ks == 0;      // this workgroup finalises (adds the partial sums, point-wise stage, publication)
  const int g0 = ks * NG8;       // first 8-k group of this workgroup's part
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kk = lane >> 5, n = lane & 31;
  const size_t TB = (size_t)T * B;
  const int rot = (4 * j + 16 * __builtin_amdgcn_readfirstlane(wave)) & (NG8 - 1);

  // ---- weights: A operand row n = output unit UB*j + 32*wave + n; entry p covers
  //      k = 8*k8 + 2*(p%4) + kk with k8 = (p/4 + rot) mod NG8: gate k8%4, unit UB*i + 8*(k8/4) + k%8
  float wreg[RP];
  {
    const float* col = a.R + UB * j + 32 * wave + n;
#pragma unroll
    for (int p = 0; p < KP; ++p) {
      const int k8 = g0 + (((p >> 2) + rot) & (NG8 - 1)), m = p & 3;
      const int unit = UB * i + 8 * (k8 >> 2) + 2 * m + kk;
      const int grp = k8 & 3;
      const int gate = CELL >= 2 ? 0 : ((CELL == 1 && grp == 3) ? 2 : grp);
      const bool live = CELL == 0 || (CELL == 1 ? grp != 2 : grp == 0);
      const float v = live ? col[((size_t)gate * H + unit) * H] : 0.f;
      if (p < RP)
        wreg[p < RP ? p : 0] = v;
      else  // the four k-pairs of a group side by side: one 16-byte LDS read per group
        wl[(((size_t)wave * (LP / 4) + ((p - RP) >> 2)) * 64 + lane) * 4 + (p & 3)] = v;
    }
  }

  // ---- the cells this thread finalises: units UB*j + UF*i + 8*c + 2*wave + kk (c < CPT), batch row b0 + n
  const int j8 = 2 * wave + kk;
  const int bb = a.b0 + 32 * sl + n;
  const bool valid = bb < B;
  int cu[CPT];
  float dc[CPT], dh_rec[CPT], dbsum[CPT][4];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    cu[c] = UB * j + UF * i + 8 * c + j8;
    dc[c] = (CELL == 0 && valid && a.dcT) ? a.dcT[(size_t)bb * H + cu[c]] : 0.f;  // GRU: the direct term dh_t o z_t
    dh_rec[c] = (valid && a.dhT) ? a.dhT[(size_t)bb * H + cu[c]] : 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g) dbsum[c][g] = 0.f;
  }
  const float* const res_gates = CELL == 0 ? a.res : a.res + TB * H;  // the four saved arrays [T][B][4H] (LSTM, GRU)
  const float* const res_c = CELL == 0 ? a.res + TB * 4 * H : a.res;   // c (LSTM) or h: the state array the step reads
  float* const Xs = a.X + (size_t)sl * T * NBK * (4 * UB * 32);
  float* const Ps = a.Pp + (size_t)sl * T * NBK * NPART * (UB * 32);
  int* const fA = a.flagsA + (size_t)sl * T * NBK * kFlagInts;
  int* const fP = a.flagsP + (size_t)sl * T * NBK * kFlagInts;
  auto slotX = [&](int t, int blk) { return Xs + ((size_t)t * NBK + blk) * (4 * UB * 32); };
  auto slotP = [&](int t, int jb, int ib) { return Ps + (((size_t)t * NBK + jb) * NPART + ib) * (UB * 32); };
  auto flagA = [&](int t, int blk) { return fA + ((size_t)t * NBK + blk) * kFlagInts; };
  auto flagP = [&](int t, int blk) { return fP + ((size_t)t * NBK + blk) * kFlagInts; };

  // reserve values and upstream gradient of the step the point-wise stage handles next: fetched ahead,
  // under the MFMAs, so that no miss to HBM sits in front of a counter poll (loads return in order)
  float fg[CPT][4], fct[CPT], fcp[CPT], fdo[CPT];
  auto fetch_step = [&](int t) {
    if (valid) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const size_t e = ((size_t)t * B + bb) * H + cu[c];
        const size_t g0 = ((size_t)t * B + bb) * G + cu[c];
        if (CELL <= 1) {
#pragma unroll
          for (int g = 0; g < 4; ++g) fg[c][g] = res_gates[g0 + (size_t)g * H];
        }
        if (CELL != 1) fct[c] = res_c[e];  // c_t (LSTM), h_t (single gate)
        if (CELL <= 1) fcp[c] = t > 0 ? res_c[e - (size_t)B * H] : (a.c0 ? a.c0[(size_t)bb * H + cu[c]] : 0.f);
        fdo[c] = a.dout[e];
      }
    }
  };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2

  // point-wise stage of step t for the UF units of this workgroup, and publication of their gate gradients
  auto pointwise_publish = [&](int t) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      float dA4[4] = {0.f, 0.f, 0.f, 0.f};
      if (valid) {
        const float dh = fdo[c] + dh_rec[c];
        if (CELL == 0) {
          const float tc = tanhf_dev(fct[c]);
          const float dcv = dc[c] + dh * fg[c][2] * (1.f - tc * tc);
          dA4[0] = dcv * fg[c][3] * fg[c][0] * (1.f - fg[c][0]);
          dA4[1] = dcv * fcp[c] * fg[c][1] * (1.f - fg[c][1]);
          dA4[2] = dh * tc * fg[c][2] * (1.f - fg[c][2]);
          dA4[3] = dcv * fg[c][0] * (1.f - fg[c][3] * fg[c][3]);
          dc[c] = dcv * fg[c][1];
        } else if (CELL == 1) {  // fg: r, z, n, R_n h; fcp: h_{t-1}
          const float dn = dh * (1.f - fg[c][1]) * (1.f - fg[c][2] * fg[c][2]);
          dA4[0] = dn * fg[c][3] * fg[c][0] * (1.f - fg[c][0]);
          dA4[1] = dh * (fcp[c] - fg[c][2]) * fg[c][1] * (1.f - fg[c][1]);
          dA4[2] = dn;
          dA4[3] = dn * fg[c][0];
          dc[c] = dh * fg[c][1];
        } else {  // fct: h_t
          dA4[0] = CELL == 3 ? dh * (1.f - fct[c] * fct[c]) : (fct[c] > 0.f ? dh : 0.f);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) dbsum[c][g] += dA4[g];
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        xsA[(c * 4 + g) * 256 + (kk * 32 + n) * 4 + wave] = dA4[g];  // k%8 = j8 = 2*wave + kk: m = wave
        ro[(g * 32 + n) * UF + 8 * c + j8] = dA4[g];
      }
    }
    __syncthreads();
    // the unit octets of this workgroup are k8 blocks 4*(UF/8*i + c) + gate of the block's slot: contiguous
#pragma unroll
    for (int c = 0; c < CPT; ++c)
      xstore4(slotX(t, j) + (size_t)(4 * (CPT * i + c)) * 256 + 4 * threadIdx.x,
              *reinterpret_cast<const floatx4*>(xsA + c * 1024 + 4 * threadIdx.x));
    signal(flagA(t, j) + (i & (kFlagSub - 1)) * kFlagStride, a.full_fences);
    // standard layout for the weight-gradient products: (gate, batch row, four of the UF units) per store
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
      const int idx = threadIdx.x + 256 * q;
      const int g = idx / (8 * UF), l2 = (idx / (UF / 4)) & 31, hf = idx % (UF / 4);
      const int b2 = a.b0 + 32 * sl + l2;
      if (b2 < B)
        *reinterpret_cast<floatx4*>(a.dA + ((size_t)t * B + b2) * G + (size_t)g * H + UB * j + UF * i + 4 * hf) =
            *reinterpret_cast<const floatx4*>(ro + (g * 32 + l2) * UF + 4 * hf);
    }
  };

  __syncthreads();  // LDS weights are in place
  if (fin) {
    fetch_step(T - 1);
    pointwise_publish(T - 1);
  }

  int rv = rot;
  for (int t = T - 1; t >= 0; --t) {
    tr.mark(t, 0);
    hide(rv);
    __builtin_amdgcn_s_sleep(kPauseA);
    w.wait(flagA(t, i), NBK);
    tr.mark(t, 1);
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    {
      const char* const src = reinterpret_cast<const char*>(slotX(t, i));
      floatx4 bv[NG8];
      floatx4 al[NG8];
      unsigned lo = lane * 16;  // met anew by the optimiser here and after every branch, so that it stays a 32-bit offset
      asm volatile("" : "+v"(lo));
      // (rot is a multiple of four groups: scalar base + lane offset + immediate)
      auto ldb = [&](int g) {
        const char* const sb = src + (size_t)(g0 + 4 * (((g >> 2) + (rv >> 2)) & (NG8 / 4 - 1))) * 1024;
        bv[g] = *reinterpret_cast<const floatx4*>(sb + lo + (g & 3) * 1024);
      };
      auto ldw = [&](int g) {
        if (g * 4 >= RP) al[g] = *reinterpret_cast<const floatx4*>(wl + (((size_t)wave * (LP / 4) + (g - RP / 4)) * 64 + lane) * 4);
      };
#pragma unroll
      for (int g = 0; g < DEPTH; ++g) ldb(g);
      ldw(0);
      ldw(1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < NG8; ++g) {
        if (g + DEPTH < NG8) ldb(g + DEPTH);
        if (g + 2 < NG8) ldw(g + 2);
        if (g == NG8 - DEPTH && t > 0 && fin) fetch_step(t - 1);  // behind the last exchange load of this step
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const int pr = g * 4 + m;
          const float av = (pr < RP) ? wreg[pr < RP ? pr : 0] : al[g][m];
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[g][m], acc, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // partial sums -> LDS (rows of the D layout) -> one coalesced, write-through 16 KB block
#pragma unroll
    for (int r = 0; r < 16; ++r) stage[(32 * wave + 8 * (r >> 2) + 4 * kk + (r & 3)) * 32 + n] = acc[r];
    tr.mark(t, 2);
    __syncthreads();
    {
      float* const dst = slotP(t, j, i * KS + ks);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int idx = threadIdx.x + 256 * q;
        xstore4(dst + 4 * idx, *reinterpret_cast<const floatx4*>(stage + 4 * idx));
      }
    }
    signal(flagP(t, j) + ((i * KS + ks) & (kFlagSub - 1)) * kFlagStride, a.full_fences);
    tr.mark(t, 3);
    if (!fin) continue;
    // A poll that comes too early is in the way of the arrivals it waits for (every wave of every workgroup polls):
    // the first look at a counter is held back until the arrivals are about due.  cfg4 backward recurrence (ms) by
    // pause before the poll for the dA slot / for the partial sums, in units of 64 cycles: none 2.84, 8 / 8 2.80,
    // 16 / 16 2.74, 16 / 32 2.67, 16 / 24 2.70, 12 / 32 2.71, 20 / 32 2.69, 16 / 40 2.71, 24 / 48 2.73, 32 / 64 2.83.
    __builtin_amdgcn_s_sleep(kPauseP);
    w.wait(flagP(t, j), NPART);
    tr.mark(t, 4);
#pragma unroll
    for (int c = 0; c < CPT; ++c) {  // dh_rec of this thread's cells: the NBK partial sums in fixed order
      float pv[NPART];
#pragma unroll
      for (int ib = 0; ib < NPART; ++ib) pv[ib] = slotP(t, j, ib)[(UF * i + 8 * c + j8) * 32 + n];
      float sum = 0.f;
#pragma unroll
      for (int ib = 0; ib < NPART; ++ib) sum += pv[ib];
      dh_rec[c] = CELL == 1 ? sum + dc[c] : sum;
    }
    tr.mark(t, 5);
    if (t > 0) pointwise_publish(t - 1);
    tr.mark(t, 6);
  }
  if (valid && fin) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      if (a.dh0) a.dh0[(size_t)bb * H + cu[c]] = dh_rec[c];
      if (CELL == 0 && a.dc0) a.dc0[(size_t)bb * H + cu[c]] = dc[c];
    }
  }
  if (a.db && fin) {  // single slice: this workgroup owns its units for every batch row, plain sums, no atomics
    __syncthreads();
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
      for (int g = 0; g < 4; ++g) stage[(g * UF + 8 * c + j8) * 32 + n] = dbsum[c][g];
    __syncthreads();
    if (threadIdx.x < NG * UF) {
      float sum = 0.f;
#pragma unroll
      for (int q = 0; q < 32; ++q) sum += stage[threadIdx.x * 32 + ((q + threadIdx.x) & 31)];
      a.db[(size_t)(threadIdx.x / UF) * H + UB * j + UF * i + (threadIdx.x % UF)] = sum;
    }
  }
}

template <int HH, int CELL>
hipError_t launch_fwdL(const PersFwdLArgs& a, hipStream_t s) {
  constexpr int KPW = HH / 8, LP = KPW > 128 ? KPW - 128 : 0;
  const size_t smem = (6144 + (size_t)4 * LP * 64) * sizeof(float);
  const void* fn = (const void*)pers_fwdL_kernel<HH, CELL>;
  static bool attr_set = false;
  if (hipError_t e = allow_dynamic_lds(fn, smem, attr_set); e != hipSuccess) return e;
  void* params[] = {const_cast<PersFwdLArgs*>(&a)};
  return launch_resident(fn, a.nsl * (HH / 8), params, (unsigned)smem, s);
}

template <int HH, int CELL, int KS = 1>
hipError_t launch_bwdL(const PersBwdLArgs& a, hipStream_t s) {
  constexpr int NBK = HH / 128, UF = 128 / NBK, LP = KS > 1 ? 0 : 256 - (UF == 16 ? 136 : 128);
  const size_t smem = (4096 + 128 * (size_t)UF + 128 * (size_t)UF + (size_t)4 * LP * 64) * sizeof(float);
  const void* fn = (const void*)pers_bwdL_kernel<HH, CELL, KS>;
  static bool attr_set = false;
  if (hipError_t e = allow_dynamic_lds(fn, smem, attr_set); e != hipSuccess) return e;
  void* params[] = {const_cast<PersBwdLArgs*>(&a)};
  return launch_resident(fn, a.nsl * NBK * NBK * KS, params, (unsigned)smem, s);
}

}  // namespace

// Dispatch over (hidden size, cell) of the one-layer kernels.
hipError_t launch_fwdL_any(int H, int cell, const PersFwdLArgs& k, hipStream_t s) {
  if (H == 2048) {
    return cell == 0 ? launch_fwdL<2048, 0>(k, s) : (cell == 1 ? launch_fwdL<2048, 1>(k, s)
                     : (cell == 2 ? launch_fwdL<2048, 2>(k, s) : launch_fwdL<2048, 3>(k, s)));
  }
  return cell == 0 ? launch_fwdL<1024, 0>(k, s) : (cell == 1 ? launch_fwdL<1024, 1>(k, s)
                   : (cell == 2 ? launch_fwdL<1024, 2>(k, s) : launch_fwdL<1024, 3>(k, s)));
}

hipError_t launch_bwdL_any(int H, int cell, const PersBwdLArgs& k, hipStream_t s) {
  if (H == 2048) {
    return cell == 0 ? launch_bwdL<2048, 0>(k, s) : (cell == 1 ? launch_bwdL<2048, 1>(k, s)
                     : (cell == 2 ? launch_bwdL<2048, 2>(k, s) : launch_bwdL<2048, 3>(k, s)));
  }
  if (k.ks == 4) {
    return cell == 0 ? launch_bwdL<1024, 0, 4>(k, s) : (cell == 1 ? launch_bwdL<1024, 1, 4>(k, s)
                     : (cell == 2 ? launch_bwdL<1024, 2, 4>(k, s) : launch_bwdL<1024, 3, 4>(k, s)));
  }
  if (k.ks == 2) {
    return cell == 0 ? launch_bwdL<1024, 0, 2>(k, s) : (cell == 1 ? launch_bwdL<1024, 1, 2>(k, s)
                     : (cell == 2 ? launch_bwdL<1024, 2, 2>(k, s) : launch_bwdL<1024, 3, 2>(k, s)));
  }
  return cell == 0 ? launch_bwdL<1024, 0>(k, s) : (cell == 1 ? launch_bwdL<1024, 1>(k, s)
                   : (cell == 2 ? launch_bwdL<1024, 2>(k, s) : launch_bwdL<1024, 3>(k, s)));
}

hipError_t launch_pack_stateL(const float* h0, float* hx, int T, int B, int H, int b0, int nsl, hipStream_t s) {
  hipLaunchKernelGGL(pack_stateL_kernel, dim3((unsigned)((32L * nsl * H + 255) / 256)), dim3(256), 0, s, h0, hx, T, B, H, b0, nsl);
  return hipGetLastError();
}

}  // namespace lstm
