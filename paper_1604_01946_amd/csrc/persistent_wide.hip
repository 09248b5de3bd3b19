// Persistent recurrence, slices of 64 batch rows on 32x32x2 tiles: pers_fwd32_kernel and pers_bwd32_kernel, templated
// on the cell (LSTM, GRU, single gate), with the kernels that put h0 and x into their exchange layout.
#include "../../include/lstm.h"
#include "persistent_dev.h"

namespace lstm {
namespace {

// ------------------------------------------------------------------ forward, wide-batch variant
// Same decomposition as pers_fwd_kernel (8 hidden units x all batch rows per workgroup) for
// 32 < B <= 64, on v_mfma_f32_32x32x2_f32: with one wave per SIMD the 16x16x4 shape issues at about
// three quarters of the fp32 matrix rate, the 32x32 shape at nearly all of it.  M = 32 weight rows
// ordered gate-major (row = 8*gate + unit) so that, in the D layout, a lane holds all four gates of
// four units; N = two tiles of 32 batch rows (tile j, column n = batch 2n + j).
// Exchange layout of one (layer, step) slot: for k = 4*k4 + 2*m + kk and batch b = 2n + j, element
// ((k4*2 + kk)*32 + n)*4 + 2*m + j -- lane (kk, n) fetches two k-pairs of both tiles with one
// 16-byte load, 1 KB per wave and instruction.
// CELL = 1 runs a GRU on the same machinery (convention of rnn.h: gates r, z, n; the reset gate multiplies the
// recurrent product): the four row groups of a workgroup's tile are then r, z, the input half of n (W_n x, no
// recurrent weights) and the recurrent half of n (R_n h, no input weights) -- a quarter of the MFMA work
// multiplies zeros, everything else is unchanged.  Its reserve is h [T][B][H] followed by r, z, n, R_n h as [T][B][4H].
// CELL = 2 / 3: single-gate RNN with ReLU / tanh: only the first row group carries weights (three quarters of the
// MFMA work multiply zeros -- these small cells are bound by the synchronisation of a step, not by the products);
// the reserve is h [T][B][H].
template <int HH, int CELL>
__global__ __launch_bounds__(256) void pers_fwd32_kernel(const PersFwdArgs a) {
  constexpr int H = HH, NG = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1), G = NG * H, NS = H / 8;  // G: rows of W, R, b and of the projection P0
  constexpr int NK4 = H / 16;  // 4-k groups per wave and operand half
  __shared__ float part[4][32][64];
  __shared__ __attribute__((aligned(16))) float xs[512];  // this step's h slice in exchange order
  __shared__ __attribute__((aligned(16))) float ro[6 * 64 * 8];  // gates, c, h of the slice: [array][batch][unit]

  // The recurrences of different batch rows are independent: slices of 64 rows run side by side as
  // separate groups of workgroups with their own exchange slots and counters.
  int l, s;
  map_block(a.L, NS * a.nsl, l, s);
  const int sl = s / NS;
  s -= sl * NS;
  const int b0 = a.b0 + 64 * sl;
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kk = lane >> 5, n = lane & 31;
  const int u0 = 8 * s;
  const size_t TB = (size_t)T * B;
  const int rot = ((int)(blockIdx.x >> 3) + __builtin_amdgcn_readfirstlane(wave)) & (NK4 - 1);

  // ---- weights -> registers: A operand row rho = lane%32 = (gate rho/8, unit rho%8), k = wave*H/4 + 4*k4 + 2*m + kk
  float wR[NK4][2], wW[NK4][2];
  {
    const float* Rl = a.R + (size_t)l * G * H;
    const float* Wl = l > 0 ? a.W + (size_t)G * a.I + (size_t)(l - 1) * G * H : a.W;  // layer 0: [G][I], read if I == H
    const int grp = n >> 3;
    // matrix row behind tile row group grp: the gate itself (LSTM); r, z, n (input half), n (recurrent half) for the GRU
    const int gate = CELL >= 2 ? 0 : ((CELL == 1 && grp == 3) ? 2 : grp);
    const bool useR = CELL == 0 || (CELL == 1 ? grp != 2 : grp == 0);
    const bool useW = (CELL == 0 || (CELL == 1 ? grp != 3 : grp == 0)) && (l > 0 || a.xin);
    const size_t row = ((size_t)gate * H + u0 + (n & 7)) * H;
#pragma unroll
    for (int i = 0; i < NK4; ++i) {
      const int k4 = (i + rot) & (NK4 - 1);
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        const int k = wave * (H / 4) + 4 * k4 + 2 * m + kk;
        wR[i][m] = useR ? Rl[row + k] : 0.f;
        wW[i][m] = useW ? Wl[row + k] : 0.f;
      }
    }
  }

  // ---- the two cells this lane finalises: wave w takes batch tile j = w%2 and unit pair up = w/2;
  //      D register r of a lane is row 8*(r/4) + 4*kk + r%4 = (gate r/4, unit 4*kk + r%4)
  const int tj = wave & 1, up = wave >> 1;
  const int lb = 2 * n + tj;   // batch row inside this launch's 64
  const int bb = b0 + lb;      // batch row in the tensors
  const bool valid = bb < B;
  int c_unit[2];
  float c_state[2], c_bias[2][4];  // c_state: c_{t-1} (LSTM), h_{t-1} (GRU)
#pragma unroll
  for (int ci = 0; ci < 2; ++ci) {
    c_unit[ci] = u0 + 4 * kk + 2 * up + ci;
    const float* const s0 = CELL == 0 ? a.c0 : (CELL == 1 ? a.h0 : nullptr);
    c_state[ci] = (valid && s0) ? s0[((size_t)l * B + bb) * H + c_unit[ci]] : 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g) c_bias[ci][g] = g < NG ? a.bias[(size_t)l * G + g * H + c_unit[ci]] : 0.f;
  }

  float* const res_l = a.res + (size_t)l * TB * (CELL == 0 ? 6 : (CELL == 1 ? 5 : 1)) * H;
  float* const res_gates = CELL == 0 ? res_l : res_l + TB * H;  // the four saved arrays, [T][B][4H]
  float* const res_c = res_l + TB * 4 * H;                       // LSTM only
  float* const res_h = CELL == 0 ? res_l + TB * 5 * H : res_l;
  float* const hx = a.hx + (size_t)sl * a.L * (T + 1) * H * 64;
  int* const flags = a.flags + (size_t)sl * a.L * (T + 1) * kFlagInts;
  auto slot = [&](int layer, int st) { return hx + ((size_t)layer * (T + 1) + st) * H * 64; };
  auto flag = [&](int layer, int st) { return flags + ((size_t)layer * (T + 1) + st) * kFlagInts; };
  const size_t boff = (size_t)wave * NK4 * 256 + lane * 4;  // this lane's offset inside a slot

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2

  // One 16-byte load of a lane feeds four MFMAs (two k-pairs x two batch tiles).  `rv` is `rot`
  // made opaque once per step (see hide()), so that the rotated offsets are computed next to their
  // loads with a few scalar instructions.
  int rv = rot;
  auto ldx = [&](const float* src, int i) {
    return *reinterpret_cast<const floatx4*>(src + (size_t)((i + rv) & (NK4 - 1)) * 256);
  };

  // ---- everything after the MFMAs of step t: K-split reduction, gates, publish h_t, reserve
  auto finish_step = [&](const floatx16 (&acc)[2], const float (&pin)[2][4], const int t) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) part[wave][j * 16 + r][lane] = acc[j][r];
    tr.mark(t, 3);
    __syncthreads();
    tr.mark(t, 4);
    float o_gate[2][4], o_c[2], o_h[2];
#pragma unroll
    for (int ci = 0; ci < 2; ++ci) {
      float sg[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int row = tj * 16 + 4 * g + 2 * up + ci;
        sg[g] = (part[0][row][lane] + part[1][row][lane]) + (part[2][row][lane] + part[3][row][lane]) +
                pin[ci][g] + c_bias[ci][g];
      }
      if (CELL == 0) {
        o_gate[ci][0] = sigmoidf_dev(sg[0]);
        o_gate[ci][1] = sigmoidf_dev(sg[1]);
        o_gate[ci][2] = sigmoidf_dev(sg[2]);
        o_gate[ci][3] = tanhf_dev(sg[3]);
        o_c[ci] = o_gate[ci][1] * c_state[ci] + o_gate[ci][0] * o_gate[ci][3];
        o_h[ci] = o_gate[ci][2] * tanhf_dev(o_c[ci]);
        c_state[ci] = o_c[ci];
      } else if (CELL >= 2) {
#pragma unroll
        for (int g = 0; g < 4; ++g) o_gate[ci][g] = 0.f;
        o_h[ci] = CELL == 3 ? tanhf_dev(sg[0]) : fmaxf(sg[0], 0.f);
        o_c[ci] = 0.f;
      } else {  // sg: r and z pre-activations, W_n x + b_n, R_n h
        o_gate[ci][0] = sigmoidf_dev(sg[0]);
        o_gate[ci][1] = sigmoidf_dev(sg[1]);
        o_gate[ci][2] = tanhf_dev(sg[2] + o_gate[ci][0] * sg[3]);
        o_gate[ci][3] = sg[3];
        o_h[ci] = (1.f - o_gate[ci][1]) * o_gate[ci][2] + o_gate[ci][1] * c_state[ci];
        o_c[ci] = 0.f;
        c_state[ci] = o_h[ci];
      }
      // unit offset ul = 4*kk + 2*up + ci: k4 block ul/4 = kk, m = up, parity ci; batch (n, tj)
      xs[kk * 256 + (ci * 32 + n) * 4 + 2 * up + tj] = valid ? o_h[ci] : 0.f;
    }
    __syncthreads();
    if (threadIdx.x < 128)  // the slice's 8 units are two contiguous 1 KB blocks of the exchange slot
      xstore4(slot(l, t + 1) + (size_t)(u0 / 4) * 256 + 4 * threadIdx.x, *reinterpret_cast<const floatx4*>(xs + 4 * threadIdx.x));
    tr.mark(t, 5);
    signal(flag(l, t + 1) + (s & (kFlagSub - 1)) * kFlagStride, a.full_fences);  // publish h_t (the barrier also protects `part` and `xs`)
    tr.mark(t, 6);
    // The reserve and the outputs are not read before the kernel ends, so they are written after the
    // signal -- staged through LDS so that each store instruction writes 16-byte runs (scattered
    // 4-byte stores keep the address unit busy for longer than the whole epilogue).  An inference call
    // has nothing to write for the lower layers except the final states.
    if (!(a.keep || l == a.L - 1 || t == T - 1)) return;
#pragma unroll
    for (int ci = 0; ci < 2; ++ci) {
      const int ul = 4 * kk + 2 * up + ci;
#pragma unroll
      for (int g = 0; g < 4; ++g) ro[(g * 64 + lb) * 8 + ul] = o_gate[ci][g];
      ro[(4 * 64 + lb) * 8 + ul] = o_c[ci];
      ro[(5 * 64 + lb) * 8 + ul] = o_h[ci];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int idx = threadIdx.x + 256 * i;  // (array 0..5, batch row, half of the 8 units)
      const int arr = idx >> 7, l2 = (idx >> 1) & 63, hf = idx & 1;
      const int b2 = b0 + l2;
      if (b2 < B) {
        const floatx4 v = *reinterpret_cast<const floatx4*>(ro + (arr * 64 + l2) * 8 + 4 * hf);
        const size_t e = ((size_t)t * B + b2) * H + u0 + 4 * hf;
        if (arr < 4) {
          if (CELL <= 1 && a.keep) *reinterpret_cast<floatx4*>(res_gates + ((size_t)t * B + b2) * 4 * H + (size_t)arr * H + u0 + 4 * hf) = v;
        } else if (arr == 4) {
          if (CELL == 0) {
            if (a.keep) *reinterpret_cast<floatx4*>(res_c + e) = v;
            if (t == T - 1 && a.cT) *reinterpret_cast<floatx4*>(a.cT + ((size_t)l * B + b2) * H + u0 + 4 * hf) = v;
          }
        } else {
          if (a.keep) *reinterpret_cast<floatx4*>(res_h + e) = v;
          if (l == a.L - 1) *reinterpret_cast<floatx4*>(a.y + e) = v;
          if (t == T - 1 && a.hT) *reinterpret_cast<floatx4*>(a.hT + ((size_t)l * B + b2) * H + u0 + 4 * hf) = v;
        }
      }
    }
  };

  if (l == 0 && !a.xin) {
    // ---- layer 0: the input half is the batched projection P_0 (added in the epilogue); its values
    //      for the next step are fetched one step ahead, behind the exchange loads, so that a miss to
    //      HBM never sits in front of a counter poll (loads return in order).
    float pin[2][4];
#pragma unroll
    for (int ci = 0; ci < 2; ++ci)
#pragma unroll
      for (int g = 0; g < 4; ++g) pin[ci][g] = (valid && g < NG) ? a.P0[(size_t)bb * G + g * H + c_unit[ci]] : 0.f;
    for (int t = 0; t < T; ++t) {
      tr.mark(t, 0);
      hide(rv);
      floatx16 acc[2];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
      if (t > 0) w.wait(flag(0, t), NS);  // slot 0 (h0 or zeros) was written before the launch
      tr.mark(t, 2);
      const float* src = slot(0, t) + boff;
      floatx4 br[NK4];
#pragma unroll
      for (int i = 0; i < NK4; ++i) br[i] = ldx(src, i);
      float pnx[2][4];
#pragma unroll
      for (int ci = 0; ci < 2; ++ci)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          pnx[ci][g] = (valid && t + 1 < T && g < NG) ? a.P0[((size_t)(t + 1) * B + bb) * G + g * H + c_unit[ci]] : 0.f;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NK4; ++i)
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wR[i][m], br[i][2 * m + j], acc[j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      finish_step(acc, pin, t);
#pragma unroll
      for (int ci = 0; ci < 2; ++ci)
#pragma unroll
        for (int g = 0; g < 4; ++g) pin[ci][g] = pnx[ci][g];
    }
    return;
  }

  // ---- layers >= 1.  Order of one step, in k-groups of 4:
  //   1. input MFMAs on the first half of h_{l-1,t}, already in registers; the second half is fetched
  //      between them.  This part also covers the time the own layer's h_{t-1} needs to become visible.
  //   2. wait for h_{l,t-1}; input MFMAs on the second half, the recurrent operand fetched between them.
  //   3. recurrent MFMAs; between the first of them the first half of h_{l-1,t+1} is fetched if the
  //      layer below (which normally runs ahead) has published it.  If it has not, the same loads
  //      re-read the current step's slot -- valid memory, values unused -- so that the step is one
  //      straight line of code, and the operand is fetched after a wait at the end of the step.
  // Loads are issued between MFMAs rather than in bulk (a bulk of 32 16-byte loads per wave holds the
  // wave in the address unit for about a microsecond while the matrix cores idle); the scheduling
  // barriers pin that order.  Only half an operand is carried from step to step, which keeps the
  // kernel inside the register file.
  // The layer below is, for layer 0 with I == H, the input sequence itself: x in exchange layout, all
  // of it there before the launch, with one counter that reads "published" for every step.
  constexpr int HK = NK4 / 2;
  const float zero_pin[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  const float* const in_base = l > 0 ? slot(l - 1, 0) : a.xin + (size_t)sl * (T + 1) * H * 64;
  int* const in_flag_base = l > 0 ? flag(l - 1, 0) : a.flags + (size_t)a.nsl * a.L * (T + 1) * kFlagInts;
  const int in_flag_step = l > 0 ? kFlagInts : 0;
  auto in_slot = [&](int st) { return in_base + (size_t)st * H * 64; };
  auto in_flag = [&](int st) { return in_flag_base + (size_t)st * in_flag_step; };
  floatx4 bl[HK];
  w.wait(in_flag(1), NS);
  {
    const float* src = in_slot(1) + boff;
#pragma unroll
    for (int i = 0; i < HK; ++i) bl[i] = ldx(src, i);
    drain_vmem();
  }
  for (int t = 0; t < T; ++t) {
    tr.mark(t, 0);
    hide(rv);
    floatx16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    auto mma4 = [&](const float (&wgt)[2], const floatx4& bv) {
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wgt[m], bv[2 * m + j], acc[j], 0, 0, 0);
    };
    // both counters are read now; the answers arrive under the MFMAs of part 1
    // (slots that do not exist at the ends of the sequence are replaced by ones that do; their values are not used)
    int seen_rec = Waiter::peek_all(flag(l, t > 0 ? t : 1));
    int seen_in = Waiter::peek_all(in_flag(t + 1 < T ? t + 2 : t + 1));
    floatx4 bh[HK], br[NK4];
    {
      const float* src = in_slot(t + 1) + boff;
      tr.mark(t, 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < HK; ++i) {
        bh[i] = ldx(src, HK + i);
        mma4(wW[i], bl[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    Waiter::land(seen_rec);
    w.wait(flag(l, t), NS, t > 0 ? seen_rec : NS);  // h_{l,t-1}; slot 0 (h0 or zeros) was written before the launch
    tr.mark(t, 2);
    {
      const float* src = slot(l, t) + boff;
#pragma unroll
      for (int i = 0; i < HK; ++i) {
        br[2 * i] = ldx(src, 2 * i);
        br[2 * i + 1] = ldx(src, 2 * i + 1);
        mma4(wW[HK + i], bh[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    const bool more = t + 1 < T;
    Waiter::land(seen_in);
    const bool pre = more && __all(seen_in >= NS / kFlagSub) && !w.dead;
    {
      const float* nsrc = in_slot(pre ? t + 2 : t + 1) + boff;
#pragma unroll
      for (int i = 0; i < NK4; ++i) {
        if (i < HK) bl[i] = ldx(nsrc, i);
        mma4(wR[i], br[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    finish_step(acc, zero_pin, t);
    if (more && !pre) {  // the layer below was late: wait for it now, after this step is published
      w.wait(in_flag(t + 2), NS);
      const float* src = in_slot(t + 2) + boff;
#pragma unroll
      for (int i = 0; i < HK; ++i) bl[i] = ldx(src, i);
      drain_vmem();
    }
  }
}

// h0 [L][B][H] (zeros if null) -> exchange slot 0 of every layer in the layout of pers_fwd32_kernel.
__global__ void pack_state32_kernel(const float* __restrict__ h0, float* __restrict__ hx, int L, int T, int B, int H, int b0,
                                    int nsl) {
  const long cnt = (long)nsl * L * 64 * H;  // all 64 batch columns of every slot: rows past the batch hold zeros
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < cnt; e += (long)gridDim.x * blockDim.x) {
    const int k = (int)(e % H), lb = (int)((e / H) % 64), l = (int)((e / ((long)H * 64)) % L);
    const int sl = (int)(e / ((long)H * 64 * L));
    const int k4 = k >> 2, m = (k >> 1) & 1, kk = k & 1, n = lb >> 1, j = lb & 1;
    const int bb = b0 + 64 * sl + lb;
    hx[(((size_t)sl * L + l) * (T + 1)) * H * 64 + ((size_t)(k4 * 2 + kk) * 32 + n) * 4 + 2 * m + j] =
        (h0 && bb < B) ? h0[((size_t)l * B + bb) * H + k] : 0.f;
  }
}

// x [T][B][H] (I == H) -> exchange layout of pers_fwd32_kernel, slots 1..T of xin [nsl][T+1][H*64], rows past the
// batch zero; also sets the counter that stands for "every step of the input is published" (nsl*L*(T+1) counters
// into `flags`).  Block (kb, t, sl) moves the 64 batch rows x 64 inputs [64*kb, 64*kb+64) of one step through LDS:
// whole rows in, one contiguous 16 KB piece of the slot out.
__global__ __launch_bounds__(256) void pack_x32_kernel(const float* __restrict__ x, float* __restrict__ xin, int* flags,
                                                       int L, int T, int B, int H, int b0, int nsl, int ready) {
  __shared__ float tile[64][65];
  const int kb = blockIdx.x, t = blockIdx.y, sl = blockIdx.z;
  if (kb == 0 && t == 0 && sl == 0 && threadIdx.x < kFlagSub)
    flags[(size_t)nsl * L * (T + 1) * kFlagInts + threadIdx.x * kFlagStride] = ready;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int e = threadIdx.x + 256 * i, lb = e >> 6, kc = e & 63;
    const int bb = b0 + 64 * sl + lb;
    tile[lb][kc] = bb < B ? x[((size_t)t * B + bb) * H + 64 * kb + kc] : 0.f;
  }
  __syncthreads();
  float* const dst = xin + ((size_t)sl * (T + 1) + t + 1) * H * 64 + (size_t)kb * 4096;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int o = threadIdx.x + 256 * i;  // 16-byte piece: ((k4*2 + kk)*32 + n), holding (m, j) = (0,0) (0,1) (1,0) (1,1)
    const int n = o & 31, kk = (o >> 5) & 1, k4 = o >> 6;
    floatx4 v;
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = tile[2 * n + (q & 1)][4 * k4 + 2 * (q >> 1) + kk];
    *reinterpret_cast<floatx4*>(dst + 4 * o) = v;
  }
}

// ------------------------------------------------------------------ backward, wide-batch variant
// For 32 < B <= 64 the kernel above is bound by L2->CU bandwidth: every workgroup reads the whole
// dA_t (4H x 64 values per step).  This variant halves that traffic by giving a workgroup 16 hidden
// units of ONE half of the batch: M = 32 rows (16 dh_rec + 16 dx), N = 32 batch rows, which is one
// v_mfma_f32_32x32x2_f32 tile (the fp32 MFMA shape that issues at full rate with one wave per
// SIMD).  Its weight slice is [32 x 4H] = 256 KB at H = 512: the first 128 k-pairs of every wave
// stay in VGPRs, the rest sit in LDS (152 KB of the CU's 160 KB are used).  The two batch halves
// never exchange data, so they are placed on different XCDs.
// Exchange layout of one (layer, step, half) slot: for k = 8*k8 + 2*m + kk and batch row n,
// element ((k8*2 + kk)*32 + n)*4 + m -- lane (kk, n) of a wave fetches the four k-pairs of an
// 8-k group with one 16-byte load, 1 KB per wave and instruction.
// CELL = 1: GRU (see pers_fwd32_kernel).  The four K groups are then the gradients with respect to the r and z
// pre-activations, to W_n x + b_n, and to R_n h; the recurrent rows of the tile have no weights in the third group,
// the input rows none in the fourth, and dh_{t-1} also receives dh_t o z_t directly.  The arrays c0 / dcT / dc0 of
// the arguments are not used; `res` is the GRU reserve, W / R / db have 3H rows.
// CELL = 2 / 3: single-gate RNN (ReLU / tanh): only the first K group is non-zero; `res` holds h alone.
template <int HH, int CELL>
__global__ __launch_bounds__(256) void pers_bwd32_kernel(const PersBwdArgs a, const int NBH) {
  constexpr int H = HH, G = 4 * H, NS2 = H / 16;  // G: width of the gate-gradient arrays (four groups for both cells)
  constexpr int NG = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1), GW = NG * H;  // rows of W, R, db
  constexpr int NB8 = H / 8;                 // 8-k groups per wave (wave w covers the rows of gate w)
  constexpr int KPW = H / 2;                 // k-pairs per wave
  constexpr int RP = KPW < 128 ? KPW : 128;  // k-pairs whose weights live in registers
  constexpr int LP = KPW - RP;               // k-pairs whose weights live in LDS
  constexpr int DEPTH = NB8 < 16 ? NB8 : 16;  // 8-k groups whose exchange loads are in flight ahead of the MFMAs
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* const part = smem;         // [4 waves][16 regs][64 lanes]
  float* const xs = smem + 4096;    // [8 blocks of 8 k][256]: this step's dA slice in exchange order
  float* const wl = smem + 6144;    // [4 waves][LP][64 lanes]

  // blockIdx -> (layer, batch half, slice): one (layer, half) group per 8/(L*NBH) XCDs when that divides
  int l, bh, s2;
  {
    const int bid = blockIdx.x, groups = a.L * NBH;
    if (groups <= 8 && 8 % groups == 0 && NS2 % (8 / groups) == 0 && (gridDim.x % 8) == 0) {
      const int per = 8 / groups, xcd = bid & 7, grp = xcd / per;
      l = grp / NBH;
      bh = grp % NBH;
      s2 = (bid >> 3) * per + (xcd % per);
    } else {
      l = bid / (NS2 * NBH);
      bh = (bid / NS2) % NBH;
      s2 = bid % NS2;
    }
  }
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kk = lane >> 5, n = lane & 31;
  const int u0 = 16 * s2;
  const size_t TB = (size_t)T * B;
  const int rot = ((int)(blockIdx.x >> 3) * (NB8 / 32 > 0 ? NB8 / 32 : 1) + 2 * __builtin_amdgcn_readfirstlane(wave)) & (NB8 - 1);

  // ---- weights: A operand row rho = lane%32 (< 16: column u0+rho of R_l, >= 16: column u0+rho-16 of W_l)
  float wreg[RP];
  {
    const float* Rl = a.R + (size_t)l * GW * H;
    const float* Wl = a.W + (size_t)GW * a.I + (size_t)(l > 0 ? l - 1 : 0) * GW * H;
    const float* src = (n < 16) ? Rl + u0 + n : (l > 0 ? Wl : a.W) + u0 + (n - 16);  // layer 0: its own [GW][I], I == H
    // matrix row block behind K group `wave`: the gate itself (LSTM); GRU: r, z, then n for the input rows only,
    // then n for the recurrent rows only
    const int gate = CELL >= 2 ? 0 : ((CELL == 1 && wave == 3) ? 2 : wave);
    const bool live = ((n < 16) || (l > 0) || a.dx0) &&
                      (CELL == 0 || (CELL == 1 ? (n < 16 ? wave != 2 : wave != 3) : wave == 0));
#pragma unroll
    for (int i = 0; i < KPW; ++i) {
      const int k8 = ((i >> 2) + rot) & (NB8 - 1), m = i & 3;
      const float v = live ? src[(size_t)(gate * H + 8 * k8 + 2 * m + kk) * H] : 0.f;
      if (i < RP)
        wreg[i < RP ? i : 0] = v;
      else
        wl[((size_t)wave * LP + (i - RP)) * 64 + lane] = v;
    }
  }

  // ---- roles: waves 0,1 run the point-wise stage on units u0 + 8*wave + 4*kk + {0..3};
  //      waves 2,3 publish dx of units u0 + 8*(wave-2) + 4*kk + {0..3}; batch row bh*32 + n
  const int bb = a.b0 + bh * 32 + n;  // batch row in the tensors; the exchange slots hold this launch's 64 rows
  const bool pwv = wave < 2 && bb < B;
  const bool dxl = wave >= 2 && bb < B && (l > 0 || a.dx0);
  const int unit0 = u0 + 8 * (wave & 1) + 4 * kk;
  float dc[4], dh_rec[4];  // dc: carried cell gradient (LSTM); the direct term dh_t o z_t (GRU)
  float dbsum[4][4];  // this lane's share of the bias gradient: sum over t of dA_t, per (gate, unit)
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const size_t se = ((size_t)l * B + bb) * H + unit0 + r;
    dc[r] = (CELL == 0 && pwv && a.dcT) ? a.dcT[se] : 0.f;
    dh_rec[r] = (pwv && a.dhT) ? a.dhT[se] : 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g) dbsum[g][r] = 0.f;
  }

  const float* const res_l = a.res + (size_t)l * TB * (CELL == 0 ? 6 : (CELL == 1 ? 5 : 1)) * H;
  const float* const res_gates = CELL == 0 ? res_l : res_l + TB * H;  // the four saved arrays, [T][B][4H] (LSTM, GRU)
  const float* const res_c = CELL == 0 ? res_l + TB * 4 * H : res_l;   // c (LSTM) or h: the state array the step reads
  const float* const s0 = CELL == 0 ? a.c0 : a.h0;
  float* const dA_l = a.dA + (size_t)l * TB * G;
  const bool has_up = l < a.L - 1;
  const float* const dout_base = has_up ? a.dxbuf + (size_t)(l + 1) * TB * H : a.dy;
  float* const dx_out = l > 0 ? a.dxbuf + (size_t)l * TB * H : a.dx0;
  auto slot = [&](int t) { return a.dAx + (((size_t)l * T + t) * NBH + bh) * G * 32; };
  auto flag = [&](int layer, int sl) { return a.flags + (((size_t)layer * (T + 1) + sl) * NBH + bh) * kFlagInts; };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2
  __syncthreads();                                    // LDS weights are in place

  // Reserve values (and, for the top layer, dy) of the step the point-wise stage handles next.  They do
  // not depend on any counter, so they are fetched one step ahead, under the MFMAs of the previous
  // step: loads return in order, and a miss to HBM in front of the counter polls would otherwise
  // stall every poll behind it.
  floatx4 gi, gf, go, gg, ct, cp, dpre;
  auto fetch_step = [&](int t) {
    if (pwv) {
      const size_t e = ((size_t)t * B + bb) * H + unit0;
      const size_t g0 = ((size_t)t * B + bb) * G + unit0;
      if (CELL <= 1) {
        gi = *reinterpret_cast<const floatx4*>(res_gates + g0);
        gf = *reinterpret_cast<const floatx4*>(res_gates + g0 + H);
        go = *reinterpret_cast<const floatx4*>(res_gates + g0 + 2 * H);
        gg = *reinterpret_cast<const floatx4*>(res_gates + g0 + 3 * H);
      }
      if (CELL != 1) ct = *reinterpret_cast<const floatx4*>(res_c + e);  // c_t (LSTM), h_t (single gate)
      if (CELL <= 1) {
        if (t > 0)
          cp = *reinterpret_cast<const floatx4*>(res_c + e - (size_t)B * H);
        else if (s0)
          cp = *reinterpret_cast<const floatx4*>(s0 + ((size_t)l * B + bb) * H + unit0);
        else
          cp = floatx4{0.f, 0.f, 0.f, 0.f};
      }
    }
  };
  // The upstream gradient of step t (dy, or dx of the layer above) is fetched with them when it is there:
  // `t_src` is t if it is published, else a step whose row this lane has already read (valid memory, value unused).
  auto fetch_dout = [&](int t_src) {
    if (pwv) dpre = *reinterpret_cast<const floatx4*>(dout_base + ((size_t)t_src * B + bb) * H + unit0);
  };
  fetch_step(T - 1);
  bool dpre_ok = !has_up;
  if (dpre_ok) fetch_dout(T - 1);

  int seen_up = 0;
  for (int t = T - 1; t >= 0; --t) {
    tr.mark(t, 0);
    // ---- point-wise stage of step t
    floatx4 dA4[4];
    const size_t e = ((size_t)t * B + bb) * H + unit0;
    const size_t g0 = ((size_t)t * B + bb) * G + unit0;
    if (has_up) w.wait(flag(l + 1, t), NS2, seen_up);  // dx of the layer above at step t is published
    tr.mark(t, 1);
    if (wave < 2) {
      floatx4 dout = {0.f, 0.f, 0.f, 0.f};
      if (pwv) dout = dpre_ok ? dpre : *reinterpret_cast<const floatx4*>(dout_base + e);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (pwv) {
          const float dh = dout[r] + dh_rec[r];
          if (CELL == 0) {
            const float tc = tanhf(ct[r]);
            const float dcv = dc[r] + dh * go[r] * (1.f - tc * tc);
            dA4[0][r] = dcv * gg[r] * gi[r] * (1.f - gi[r]);
            dA4[1][r] = dcv * cp[r] * gf[r] * (1.f - gf[r]);
            dA4[2][r] = dh * tc * go[r] * (1.f - go[r]);
            dA4[3][r] = dcv * gi[r] * (1.f - gg[r] * gg[r]);
            dc[r] = dcv * gf[r];
          } else if (CELL >= 2) {  // ct holds h_t
            dA4[0][r] = CELL == 3 ? dh * (1.f - ct[r] * ct[r]) : (ct[r] > 0.f ? dh : 0.f);
            dA4[1][r] = dA4[2][r] = dA4[3][r] = 0.f;
          } else {  // gi, gf, go, gg hold r, z, n, R_n h; cp holds h_{t-1}
            const float dn = dh * (1.f - gf[r]) * (1.f - go[r] * go[r]);
            dA4[0][r] = dn * gg[r] * gi[r] * (1.f - gi[r]);
            dA4[1][r] = dh * (cp[r] - go[r]) * gf[r] * (1.f - gf[r]);
            dA4[2][r] = dn;
            dA4[3][r] = dn * gi[r];
            dc[r] = dh * gf[r];
          }
#pragma unroll
          for (int g = 0; g < 4; ++g) dbsum[g][r] += dA4[g][r];
        }
        // unit u0 + 8*wave + 4*kk + r sits at k%8 = 4*kk + r of block (gate, wave): m = 2*kk + r/2, parity r%2
#pragma unroll
        for (int g = 0; g < 4; ++g)
          xs[(g * 2 + wave) * 256 + ((r & 1) * 32 + n) * 4 + 2 * kk + (r >> 1)] = pwv ? dA4[g][r] : 0.f;
      }
    }
    __syncthreads();
    {  // eight 1 KB blocks (gate x unit-octet), each contiguous in the exchange slot
      float* const xo = slot(t);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int idx = threadIdx.x + 256 * i, blk = idx >> 6, off = idx & 63;
        const int g = blk >> 1, o8 = blk & 1;
        xstore4(xo + ((size_t)(g * H + u0) / 8 + o8) * 256 + off * 4, *reinterpret_cast<const floatx4*>(xs + blk * 256 + off * 4));
      }
    }
    tr.mark(t, 2);
    signal(flag(l, t + 1) + (s2 & (kFlagSub - 1)) * kFlagStride, a.full_fences);
    tr.mark(t, 3);
    if (pwv) {
#pragma unroll
      for (int g = 0; g < 4; ++g) *reinterpret_cast<floatx4*>(dA_l + g0 + (size_t)g * H) = dA4[g];
    }

    // ---- GEMM of step t: needs dA_t of every slice of this layer and batch half.  (The first look at the counter is
    //      held back by 1024 cycles: a poll that comes before the arrivals is in their way; L = 4, H = 512, B = 64, T = 100
    //      backward 1.309 -> 1.27 ms.)
    __builtin_amdgcn_s_sleep(16);
    w.wait(flag(l, t + 1), NS2);
    tr.mark(t, 4);
    // counter of the layer above for the next point-wise stage: read now, looked at under the MFMAs
    // (the top layer reads its own, already complete counter instead, so that this is one straight line)
    seen_up = Waiter::peek_all(has_up ? flag(l + 1, t > 0 ? t - 1 : 0) : flag(l, t + 1));
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    {
      // One 16-byte exchange load feeds the four MFMAs of an 8-k group.  The loads run DEPTH groups
      // ahead of the MFMAs and are issued between them (so is the LDS part of the weights, two groups
      // ahead): issued in bulk they would hold the wave in the address unit while the matrix cores
      // idle.  The scheduling barrier after every group keeps this order.
      const float* src = slot(t) + (size_t)wave * NB8 * 256 + lane * 4;
      floatx4 bv[NB8];
      float al[NB8][4];
      int rv = rot;
      hide(rv);  // keeps the rotated offsets next to their loads
      auto ldb = [&](int g) { bv[g] = *reinterpret_cast<const floatx4*>(src + (size_t)((g + rv) & (NB8 - 1)) * 256); };
      auto ldw = [&](int g) {
        if (g * 4 >= RP) {
#pragma unroll
          for (int m = 0; m < 4; ++m) al[g][m] = wl[((size_t)wave * LP + (g * 4 + m - RP)) * 64 + lane];
        }
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
        if (g == NB8 - DEPTH) {  // behind the last exchange load of this step
          Waiter::land(seen_up);
          dpre_ok = t > 0 && (!has_up || (__all(seen_up >= NS2 / kFlagSub) && !w.dead));
          if (t > 0) fetch_step(t - 1);
          fetch_dout(dpre_ok ? t - 1 : t);
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
    tr.mark(t, 5);
    __syncthreads();
    tr.mark(t, 6);
    {
      // register r of a lane is row 8*(r/4) + 4*kk + r%4: wave w sums registers 4w..4w+3 = rows 8w+4kk+{0..3}
      float v[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = 4 * wave + r;
        v[r] = (part[(0 * 16 + row) * 64 + lane] + part[(1 * 16 + row) * 64 + lane]) +
               (part[(2 * 16 + row) * 64 + lane] + part[(3 * 16 + row) * 64 + lane]);
      }
      if (wave < 2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) dh_rec[r] = CELL == 1 ? v[r] + dc[r] : v[r];
      } else if (dxl) {
        xstore4(dx_out + ((size_t)t * B + bb) * H + unit0, floatx4{v[0], v[1], v[2], v[3]});
      }
    }
    // `part` and `xs` are next written after the barriers of the next point-wise stage
  }
  signal(flag(l, 0) + (s2 & (kFlagSub - 1)) * kFlagStride, a.full_fences);  // slot 0: dx of step 0 published
  if (pwv) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const size_t se = ((size_t)l * B + bb) * H + unit0 + r;
      if (a.dh0) a.dh0[se] = dh_rec[r];
      if (CELL == 0 && a.dc0) a.dc0[se] = dc[r];
    }
  }
  // Bias gradient (Section 2.6 lists it with the weight update): the per-lane sums over t are added
  // over the 32 batch rows of this workgroup through LDS and then into db.  Each element of db
  // receives exactly one contribution per batch half, and a + b does not depend on which of the
  // two arrives first, so the result is reproducible.
  if (a.db) {
    if (wave < 2) {
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int g = 0; g < 4; ++g) part[(g * 16 + 8 * wave + 4 * kk + r) * 32 + n] = dbsum[g][r];
    }
    __syncthreads();
    if (threadIdx.x < 16 * NG) {
      const int g = threadIdx.x >> 4, ul = threadIdx.x & 15;
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 32; ++i) sum += part[threadIdx.x * 32 + ((i + threadIdx.x) & 31)];
      atomicAdd(a.db + (size_t)l * GW + g * H + u0 + ul, sum);
    }
  }
}

template <int CELL>
hipError_t launch_fwd32(int H, int grid, const PersFwdArgs& a, hipStream_t s) {
  void* params[] = {const_cast<PersFwdArgs*>(&a)};
  const void* fn = H == 512 ? (const void*)pers_fwd32_kernel<512, CELL>
                            : (H == 256 ? (const void*)pers_fwd32_kernel<256, CELL> : (const void*)pers_fwd32_kernel<128, CELL>);
  return launch_resident(fn, grid, params, 0, s);
}

template <int HH, int CELL = 0>
hipError_t launch_bwd32(const PersBwdArgs& a, int nbh, hipStream_t s) {
  constexpr int KPW = HH / 2, LP = KPW > 128 ? KPW - 128 : 0;
  const size_t smem = (6144 + (size_t)4 * LP * 64) * sizeof(float);
  const void* fn = (const void*)pers_bwd32_kernel<HH, CELL>;
  static bool attr_set = false;
  if (hipError_t e = allow_dynamic_lds(fn, smem, attr_set); e != hipSuccess) return e;
  void* params[] = {const_cast<PersBwdArgs*>(&a), &nbh};
  const int grid = a.L * (HH / 16) * nbh;
  return launch_resident(fn, grid, params, (unsigned)smem, s);
}

}  // namespace

hipError_t launch_fwd_wide(int cell, int H, int grid, const PersFwdArgs& a, hipStream_t s) {
  return cell == 0 ? launch_fwd32<0>(H, grid, a, s)
                   : (cell == 1 ? launch_fwd32<1>(H, grid, a, s) : (cell == 2 ? launch_fwd32<2>(H, grid, a, s) : launch_fwd32<3>(H, grid, a, s)));
}

hipError_t launch_bwd_wide(int cell, int H, const PersBwdArgs& a, int nbh, hipStream_t s) {
#define LSTM_BWD_WIDE_CASE(C)                                                                                     \
  if (cell == C)                                                                                                  \
    return H == 512 ? launch_bwd32<512, C>(a, nbh, s) : (H == 256 ? launch_bwd32<256, C>(a, nbh, s) : launch_bwd32<128, C>(a, nbh, s));
  LSTM_BWD_WIDE_CASE(0)
  LSTM_BWD_WIDE_CASE(1)
  LSTM_BWD_WIDE_CASE(2)
  LSTM_BWD_WIDE_CASE(3)
#undef LSTM_BWD_WIDE_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_pack_state32(const float* h0, float* hx, int L, int T, int B, int H, int b0, int nsl, hipStream_t s) {
  const long n = (long)nsl * L * 64 * H;
  hipLaunchKernelGGL(pack_state32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, h0, hx, L, T, B, H, b0, nsl);
  return hipGetLastError();
}

hipError_t launch_pack_x32(const float* x, float* xin, int* flags, int L, int T, int B, int H, int b0, int nsl, int ready, hipStream_t s) {
  hipLaunchKernelGGL(pack_x32_kernel, dim3(H / 64, T, nsl), dim3(256), 0, s, x, xin, flags, L, T, B, H, b0, nsl, ready);
  return hipGetLastError();
}

}  // namespace lstm
