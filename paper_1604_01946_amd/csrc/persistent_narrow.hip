// Persistent recurrence, tiles of 16 batch rows: pers_fwd_kernel and pers_bwd_kernel (B <= 32, and larger batches as
// slices of 16 / 32 rows side by side while all slices fit the chip).
//
// Forward data flow per step of workgroup (l, s):
//   input half     acc  = W_l[rows, :] * h_{l-1,t}      (layers >= 1; layer 0 adds the batched P_0)
//   recurrent half acc += R_l[rows, :] * h_{l,t-1}
//   epilogue       4-way K-split summed through LDS, gates, c_t, h_t; h_t goes to the reserve
//                  and, k-major ([H][BP]), to the exchange buffer the other workgroups read.
// MFMA shape v_mfma_f32_16x16x4_f32: M = 32 weight rows (unit-major, gate-minor; two tiles),
// N = batch, K split over the four waves.  The exchange buffer is k-major so that one 16-byte
// load per lane (4 consecutive batch entries of one k) feeds the B operands of the four batch
// tiles: tile j, column n is batch 4n + j.
#include "../../include/lstm.h"
#include "persistent_dev.h"

namespace lstm {
namespace {

// KG: k-groups (of 4) per wave and per operand half = H/16.  NT: batch tiles of 16 per chain.
// NC: batch chains.  The recurrences of different batch rows are independent, so the batch is cut
// into NC chains of 16*NT rows that share the resident weights but have their own exchange slots
// and counters; a workgroup alternates between them, and while one chain's h_t is on its way to
// the other workgroups the matrix cores work on the other chain.
template <int KG, int NT, int NC>
__global__ __launch_bounds__(256) void pers_fwd_kernel(const PersFwdArgs a) {
  constexpr int H = 16 * KG, G = 4 * H, BP = 16 * NT, NS = H / 8;
  constexpr int CPL = (2 * NT + 3) / 4;  // cells finalised per lane and chain
  __shared__ float part[4][2 * NT * 4][64];
  __shared__ __attribute__((aligned(16))) float xs[8 * BP];  // this step's h slice, [unit][batch]
  __shared__ __attribute__((aligned(16))) float ro[6 * BP * 8];  // gates, c, h of the slice: [array][batch][unit]

  // The recurrences of different batch rows are independent: slices of NC*BP rows run side by side as separate groups
  // of workgroups with their own exchange slots and counters (a.nsl of them, the first at batch row a.b0).
  int l, s;
  map_block(a.L, NS * a.nsl, l, s);
  const int sl = s / NS;
  s -= sl * NS;
  const int brow0 = a.b0 + NC * BP * sl;
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, n = lane & 15;
  const int u0 = 8 * s;
  const size_t TB = (size_t)T * B;

  // Register i of a wave covers k-group (i + rot) mod KG: workgroups (and waves) that share an L2
  // walk the exchange slot from different starting points instead of all hitting one channel.
  const int rot = ((int)(blockIdx.x >> 3) + __builtin_amdgcn_readfirstlane(wave)) & (KG - 1);
  // ---- weights -> registers, as MFMA A operands: lane (q, n) holds row n of tile mt at k = kbase + 4*kg + q
  float wR[KG][2], wW[KG][2];
  {
    const float* Rl = a.R + (size_t)l * G * H;
    const float* Wl = a.W + (size_t)4 * H * a.I + (size_t)(l > 0 ? l - 1 : 0) * G * H;
    const int kbase = wave * (H / 4) + q;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const int unit = u0 + 4 * mt + (n >> 2), gate = n & 3;
      const size_t row = ((size_t)gate * H + unit) * H;
#pragma unroll
      for (int i = 0; i < KG; ++i) {
        const int kg = (i + rot) & (KG - 1);
        wR[i][mt] = Rl[row + kbase + 4 * kg];
        wW[i][mt] = (l > 0) ? Wl[row + kbase + 4 * kg] : 0.f;
      }
    }
  }

  // ---- the cells this lane finalises: pair p = (tile mt, tile j) -> unit 4*mt+q, chain-local batch NT*n+j
  int c_unit[CPL], c_lb[CPL], c_p[CPL];
  float c_bias[CPL][4];
  bool c_valid[NC][CPL];
  float c_state[NC][CPL];
#pragma unroll
  for (int ci = 0; ci < CPL; ++ci) {
    const int p = wave + 4 * ci;
    c_p[ci] = p;
    const int mt = p / NT, j = p % NT;
    c_unit[ci] = u0 + 4 * mt + q;
    c_lb[ci] = NT * n + j;
#pragma unroll
    for (int g = 0; g < 4; ++g) c_bias[ci][g] = (p < 2 * NT) ? a.bias[(size_t)l * G + g * H + c_unit[ci]] : 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int bb = brow0 + c * BP + c_lb[ci];
      c_valid[c][ci] = (p < 2 * NT) && (bb < B);
      c_state[c][ci] = (c_valid[c][ci] && a.c0) ? a.c0[((size_t)l * B + bb) * H + c_unit[ci]] : 0.f;
    }
  }

  float* const res_l = a.res + (size_t)l * TB * 6 * H;
  float* const res_gates = res_l;
  float* const res_c = res_l + TB * 4 * H;
  float* const res_h = res_l + TB * 5 * H;
  const size_t boff = (size_t)(wave * (H / 4) + q) * BP + NT * n;  // this lane's B-operand offset inside a slot
  float* const hx = a.hx + (size_t)sl * a.L * (T + 1) * NC * H * BP;
  int* const flags = a.flags + (size_t)sl * a.L * (T + 1) * NC * kFlagInts;
  auto slot = [&](int layer, int st, int c) { return hx + (((size_t)layer * (T + 1) + st) * NC + c) * H * BP; };
  auto flag = [&](int layer, int st, int c) { return flags + (((size_t)layer * (T + 1) + st) * NC + c) * kFlagInts; };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2

  int rv = rot;
  for (int t = 0; t < T; ++t) {
    if (KG >= 32) hide(rv);  // large H: keeps the rotated offsets next to their loads instead of in spilled registers
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (c == 0) tr.mark(t, 0);
      floatx4 acc[2][NT];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[mt][j] = floatx4{0.f, 0.f, 0.f, 0.f};

      // layer 0: fetch the batched input projection early, it is consumed in the epilogue
      float pin[CPL][4];
#pragma unroll
      for (int ci = 0; ci < CPL; ++ci)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          pin[ci][g] = (l == 0 && c_valid[c][ci])
                           ? a.P0[((size_t)t * B + brow0 + c * BP + c_lb[ci]) * G + g * H + c_unit[ci]] : 0.f;

      // Loads are issued in bulk ahead of the MFMAs that consume them (the scheduling barriers keep
      // the compiler from re-serialising them): a step is bound by load latency otherwise.
      const bool do_in = l > 0, do_rec = (t > 0 || a.has_h0);
      // both counters are read at once, without branches, so that their round trips overlap (a counter that
      // does not apply is replaced by one that exists; its value is not used)
      int seen_in = Waiter::peek_all(do_in ? flag(l - 1, t + 1, c) : flag(l, t > 0 ? t : 1, c));
      int seen_rec = Waiter::peek_all(flag(l, t > 0 ? t : 1, c));
      float bi[KG][NT], br[KG][NT];
      if (do_in) {  // input half: h of the layer below at this step
        Waiter::land(seen_in);
        w.wait(flag(l - 1, t + 1, c), NS, seen_in);
        const float* src = slot(l - 1, t + 1, c) + boff;
#pragma unroll
        for (int i = 0; i < KG; ++i) BVec<NT>::ld(src + (size_t)4 * ((i + rv) & (KG - 1)) * BP, bi[i]);
        if (c == 0) tr.mark(t, 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < KG / 2; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wW[i][mt], bi[i][j], acc[mt][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (do_rec) {  // recurrent half: own layer, previous step; its loads fly under the rest of the input half
        Waiter::land(seen_rec);
        if (t > 0) w.wait(flag(l, t, c), NS, seen_rec);
        if (c == 0) tr.mark(t, 2);
        const float* src = slot(l, t, c) + boff;
#pragma unroll
        for (int i = 0; i < KG; ++i) BVec<NT>::ld(src + (size_t)4 * ((i + rv) & (KG - 1)) * BP, br[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (do_in) {
#pragma unroll
        for (int i = KG / 2; i < KG; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wW[i][mt], bi[i][j], acc[mt][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (do_rec) {
#pragma unroll
        for (int i = 0; i < KG; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wR[i][mt], br[i][j], acc[mt][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }

      // ---- 4-way K-split reduction through LDS
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) part[wave][(mt * NT + j) * 4 + r][lane] = acc[mt][j][r];
      if (c == 0) tr.mark(t, 3);
      __syncthreads();
      if (c == 0) tr.mark(t, 4);

      // ---- epilogue: register r of lane (q, n) in tile (mt, j) is (unit 4*mt+q, gate r, batch NT*n+j)
      float o_gate[CPL][4], o_c[CPL], o_h[CPL];
#pragma unroll
      for (int ci = 0; ci < CPL; ++ci) {
        if (c_p[ci] < 2 * NT) {
          float sg[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = c_p[ci] * 4 + r;
            sg[r] = (part[0][row][lane] + part[1][row][lane]) + (part[2][row][lane] + part[3][row][lane]) +
                    pin[ci][r] + c_bias[ci][r];
          }
          o_gate[ci][0] = sigmoidf_dev(sg[0]);
          o_gate[ci][1] = sigmoidf_dev(sg[1]);
          o_gate[ci][2] = sigmoidf_dev(sg[2]);
          o_gate[ci][3] = tanhf_dev(sg[3]);
          o_c[ci] = o_gate[ci][1] * c_state[c][ci] + o_gate[ci][0] * o_gate[ci][3];
          o_h[ci] = o_gate[ci][2] * tanhf_dev(o_c[ci]);
          c_state[c][ci] = o_c[ci];
          xs[(c_unit[ci] - u0) * BP + c_lb[ci]] = c_valid[c][ci] ? o_h[ci] : 0.f;
        }
      }
      __syncthreads();
      if (threadIdx.x < 2 * BP)  // the slice's 8 rows are contiguous in the k-major exchange slot
        xstore4(slot(l, t + 1, c) + (size_t)u0 * BP + 4 * threadIdx.x, *reinterpret_cast<const floatx4*>(xs + 4 * threadIdx.x));
      if (c == 0) tr.mark(t, 5);
      signal(flag(l, t + 1, c) + (s & (kFlagSub - 1)) * kFlagStride, a.full_fences);  // publish h_t (the barrier also protects `part` and `xs`)
      if (c == 0) tr.mark(t, 6);
      // The reserve and the outputs are not read before the kernel ends, so they are written after
      // the signal -- staged through LDS so that each store instruction writes 16-byte runs
      // (scattered 4-byte stores keep the address unit busy for longer than the whole epilogue).
#pragma unroll
      for (int ci = 0; ci < CPL; ++ci) {
        if (c_p[ci] < 2 * NT) {
          const int ul = c_unit[ci] - u0;
#pragma unroll
          for (int g = 0; g < 4; ++g) ro[(g * BP + c_lb[ci]) * 8 + ul] = o_gate[ci][g];
          ro[(4 * BP + c_lb[ci]) * 8 + ul] = o_c[ci];
          ro[(5 * BP + c_lb[ci]) * 8 + ul] = o_h[ci];
        }
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < (12 * BP + 255) / 256; ++i) {
        const int idx = threadIdx.x + 256 * i;  // (array 0..5, chain-local batch row, half of the 8 units)
        const int arr = idx / (2 * BP), lb = (idx >> 1) % BP, hf = idx & 1;
        const int b2 = brow0 + c * BP + lb;
        if (idx < 12 * BP && b2 < B) {
          const floatx4 v = *reinterpret_cast<const floatx4*>(ro + (arr * BP + lb) * 8 + 4 * hf);
          const size_t e = ((size_t)t * B + b2) * H + u0 + 4 * hf;
          if (arr < 4) {
            *reinterpret_cast<floatx4*>(res_gates + ((size_t)t * B + b2) * G + (size_t)arr * H + u0 + 4 * hf) = v;
          } else if (arr == 4) {
            *reinterpret_cast<floatx4*>(res_c + e) = v;
            if (t == T - 1 && a.cT) *reinterpret_cast<floatx4*>(a.cT + ((size_t)l * B + b2) * H + u0 + 4 * hf) = v;
          } else {
            *reinterpret_cast<floatx4*>(res_h + e) = v;
            if (l == a.L - 1) *reinterpret_cast<floatx4*>(a.y + e) = v;
            if (t == T - 1 && a.hT) *reinterpret_cast<floatx4*>(a.hT + ((size_t)l * B + b2) * H + u0 + 4 * hf) = v;
          }
        }
      }
    }
  }
}

// h0 [L][B][H] -> exchange slot 0 of every slice, layer and chain, k-major [H][BP]; rows past the batch are zero.
__global__ void pack_state_kernel(const float* __restrict__ h0, float* __restrict__ hx, int L, int T, int B, int H,
                                  int BP, int NC, int b0, int nsl) {
  const long n = (long)nsl * L * NC * BP * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long)gridDim.x * blockDim.x) {
    const int lb = (int)(e % BP);
    long r = e / BP;
    const int k = (int)(r % H); r /= H;
    const int c = (int)(r % NC); r /= NC;
    const int l = (int)(r % L);
    const int sl = (int)(r / L);
    const int bb = b0 + (sl * NC + c) * BP + lb;
    hx[((((size_t)sl * L + l) * (T + 1)) * NC + c) * H * BP + (size_t)k * BP + lb] =
        bb < B ? h0[((size_t)l * B + bb) * H + k] : 0.f;
  }
}


// KGB: k-groups (of 4) per wave = H/4 (wave w covers the rows of gate w).  NT, NC as in the forward kernel.
template <int KGB, int NT, int NC>
__global__ __launch_bounds__(256) void pers_bwd_kernel(const PersBwdArgs a) {
  constexpr int H = 4 * KGB, G = 4 * H, BP = 16 * NT, NS = H / 8;
  __shared__ float part[4][NT * 4][64];
  __shared__ __attribute__((aligned(16))) float xs[32 * BP];  // this step's dA slice, [gate][unit][batch]

  // Slices of NC*BP batch rows side by side, as in the forward kernel: the grid holds one group of L*NS workgroups
  // per slice, the first slice starts at batch row a.b0.
  const int nsl = (int)gridDim.x / (a.L * NS);
  int l, s;
  map_block(a.L, NS * nsl, l, s);
  const int sl = s / NS;
  s -= sl * NS;
  const int brow0 = a.b0 + NC * BP * sl;
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, n = lane & 15;
  const int u0 = 8 * s;
  const size_t TB = (size_t)T * B;

  // ---- weights -> registers: A operand row n (< 8: column u0+n of R_l, >= 8: column u0+n-8 of W_l),
  //      k = wave*H + 4*kg + q
  const int rot = ((int)(blockIdx.x >> 3) * (KGB / 32) + 2 * __builtin_amdgcn_readfirstlane(wave)) & (KGB - 1);
  float wB[KGB];
  {
    const float* Rl = a.R + (size_t)l * G * H;
    const float* Wl = a.W + (size_t)4 * H * a.I + (size_t)(l > 0 ? l - 1 : 0) * G * H;
    const float* src = (n < 8) ? Rl + u0 + n : (l > 0 ? Wl : a.W) + u0 + (n - 8);  // layer 0: its own [4H][I], I == H
    const bool live = (n < 8) || (l > 0) || a.dx0;
#pragma unroll
    for (int i = 0; i < KGB; ++i)
      wB[i] = live ? src[(size_t)(wave * H + 4 * ((i + rot) & (KGB - 1)) + q) * H] : 0.f;
  }

  // ---- the cells this lane owns in the point-wise stage: wave j finalises batch tile j;
  //      lanes q < 2 hold dh_rec of units 4q..4q+3, lanes q >= 2 hold dx of units 4(q-2)..+3
  const int lb = NT * n + wave;                     // chain-local batch row
  const bool fin = wave < NT;                       // this wave finalises a tile
  const int unit0 = u0 + 4 * (q & 1);               // first of the lane's four units
  bool pw[NC], dxl[NC];
  float dc[NC][4], dh_rec[NC][4];
  int seen_up[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int bb = brow0 + c * BP + lb;
    pw[c] = fin && q < 2 && bb < B;                 // lane runs the point-wise stage
    dxl[c] = fin && q >= 2 && bb < B && (l > 0 || a.dx0);
    seen_up[c] = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const size_t se = ((size_t)l * B + bb) * H + unit0 + r;
      dc[c][r] = (pw[c] && a.dcT) ? a.dcT[se] : 0.f;
      dh_rec[c][r] = (pw[c] && a.dhT) ? a.dhT[se] : 0.f;
    }
  }

  const float* const res_l = a.res + (size_t)l * TB * 6 * H;
  const float* const res_gates = res_l;
  const float* const res_c = res_l + TB * 4 * H;
  float* const dA_l = a.dA + (size_t)l * TB * G;
  const bool has_up = l < a.L - 1;
  const float* const dout_base = has_up ? a.dxbuf + (size_t)(l + 1) * TB * H : a.dy;
  float* const dx_out = l > 0 ? a.dxbuf + (size_t)l * TB * H : a.dx0;
  const size_t boff = (size_t)(wave * H + q) * BP + NT * n;
  float* const dAx = a.dAx + (size_t)sl * a.L * T * NC * G * BP;
  int* const flags = a.flags + (size_t)sl * a.L * (T + 1) * NC * kFlagInts;
  auto slot = [&](int t, int c) { return dAx + (((size_t)l * T + t) * NC + c) * G * BP; };
  auto flag = [&](int layer, int st, int c) { return flags + (((size_t)layer * (T + 1) + st) * NC + c) * kFlagInts; };

  Waiter w{a.watchdog, a.spin_limit, false, a.full_fences};
  const Tracer tr{((int)blockIdx.x == a.trace_block) ? a.trace : nullptr};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2

  // Reserve values (and, for the top layer, dy) of the step the point-wise stage handles next.  They do
  // not depend on any counter, so they are fetched one step ahead, behind the exchange loads of the
  // previous step: loads return in order, and a miss to HBM in front of the counter polls would
  // otherwise stall every poll behind it.
  floatx4 gi[NC], gf[NC], go[NC], gg[NC], ct[NC], cp[NC], dpre[NC];
  auto fetch_step = [&](int t, int c) {
    if (pw[c]) {
      const int bb = brow0 + c * BP + lb;
      const size_t e = ((size_t)t * B + bb) * H + unit0;
      const size_t g0 = ((size_t)t * B + bb) * G + unit0;
      gi[c] = *reinterpret_cast<const floatx4*>(res_gates + g0);
      gf[c] = *reinterpret_cast<const floatx4*>(res_gates + g0 + H);
      go[c] = *reinterpret_cast<const floatx4*>(res_gates + g0 + 2 * H);
      gg[c] = *reinterpret_cast<const floatx4*>(res_gates + g0 + 3 * H);
      ct[c] = *reinterpret_cast<const floatx4*>(res_c + e);
      if (t > 0)
        cp[c] = *reinterpret_cast<const floatx4*>(res_c + e - (size_t)B * H);
      else if (a.c0)
        cp[c] = *reinterpret_cast<const floatx4*>(a.c0 + ((size_t)l * B + bb) * H + unit0);
      else
        cp[c] = floatx4{0.f, 0.f, 0.f, 0.f};
      if (!has_up) dpre[c] = *reinterpret_cast<const floatx4*>(a.dy + e);
    }
  };
#pragma unroll
  for (int c = 0; c < NC; ++c) fetch_step(T - 1, c);

  int rv = rot;
  for (int t = T - 1; t >= 0; --t) {
    hide(rv);  // keeps the rotated offsets next to their loads
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (c == 0) tr.mark(t, 0);
      const int bb = brow0 + c * BP + lb;
      // ---- point-wise stage of step t
      floatx4 dA4[4];
      const size_t e = ((size_t)t * B + bb) * H + unit0;
      const size_t g0 = ((size_t)t * B + bb) * G + unit0;
      Waiter::land(seen_up[c]);
      if (has_up) w.wait(flag(l + 1, t, c), NS, seen_up[c]);  // dx of the layer above at step t is published
      if (c == 0) tr.mark(t, 1);
      if (fin && q < 2 && !pw[c]) {  // padded batch columns of the staged tile
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int g = 0; g < 4; ++g) xs[(g * 8 + (unit0 - u0) + r) * BP + lb] = 0.f;
      }
      if (pw[c]) {
        const floatx4 dout = has_up ? *reinterpret_cast<const floatx4*>(dout_base + e) : dpre[c];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float dh = dout[r] + dh_rec[c][r];
          const float tc = tanhf_dev(ct[c][r]);
          const float dcv = dc[c][r] + dh * go[c][r] * (1.f - tc * tc);
          dA4[0][r] = dcv * gg[c][r] * gi[c][r] * (1.f - gi[c][r]);
          dA4[1][r] = dcv * cp[c][r] * gf[c][r] * (1.f - gf[c][r]);
          dA4[2][r] = dh * tc * go[c][r] * (1.f - go[c][r]);
          dA4[3][r] = dcv * gi[c][r] * (1.f - gg[c][r] * gg[c][r]);
          dc[c][r] = dcv * gf[c][r];
#pragma unroll
          for (int g = 0; g < 4; ++g) xs[(g * 8 + (unit0 - u0) + r) * BP + lb] = dA4[g][r];
        }
      }
      __syncthreads();
      {  // per gate the slice's 8 rows are contiguous in the k-major exchange slot
        float* const xo = slot(t, c);
#pragma unroll
        for (int i = 0; i < (8 * BP + 255) / 256; ++i) {
          const int idx = threadIdx.x + 256 * i;
          if (idx < 8 * BP) {
            const int g = idx / (2 * BP), rem = idx % (2 * BP);
            xstore4(xo + (size_t)(g * H + u0) * BP + 4 * rem, *reinterpret_cast<const floatx4*>(xs + 4 * idx));
          }
        }
      }
      if (c == 0) tr.mark(t, 2);
      signal(flag(l, t + 1, c) + (s & (kFlagSub - 1)) * kFlagStride, a.full_fences);
      if (c == 0) tr.mark(t, 3);
      if (pw[c]) {
#pragma unroll
        for (int g = 0; g < 4; ++g) *reinterpret_cast<floatx4*>(dA_l + g0 + (size_t)g * H) = dA4[g];
      }

      // ---- GEMM of step t: needs dA_t of every slice of this layer.  (The first look at the counter is held back by
      //      1024 cycles: a poll that comes before the arrivals is in their way.  L = 4, T = 100: H = 512, B = 32 backward
      //      1.144 -> 1.105 ms, H = 256, B = 16 0.488 -> 0.449 ms; 1536 cycles 1.080 / 0.469, 2048 cycles 1.085 / 0.490.)
      __builtin_amdgcn_s_sleep(16);
      w.wait(flag(l, t + 1, c), NS);
      if (c == 0) tr.mark(t, 4);
      // counter of the layer above for the next point-wise stage, read without a branch and consumed there
      // (the top layer reads its own, already complete counter instead)
      seen_up[c] = Waiter::peek_all(has_up ? flag(l + 1, t > 0 ? t - 1 : 0, c) : flag(l, t + 1, c));
      floatx4 acc[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
      {
        const float* src = slot(t, c) + boff;
        // double-buffered chunks of CH k-groups: the loads of chunk i+1 are in flight under the MFMAs
        // of chunk i (the scheduling barriers keep the compiler from re-serialising them)
        constexpr int CH = (KGB >= 64) ? 32 : 16, NCH = KGB / CH;
        float bv[2][CH][NT];
#pragma unroll
        for (int i = 0; i < CH; ++i) BVec<NT>::ld(src + (size_t)4 * ((i + rv) & (KGB - 1)) * BP, bv[0][i]);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          if (ch + 1 < NCH) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
              BVec<NT>::ld(src + (size_t)4 * (((ch + 1) * CH + i + rv) & (KGB - 1)) * BP, bv[(ch + 1) & 1][i]);
          }
          if (ch == (NCH > 1 ? NCH - 2 : 0) && t > 0) fetch_step(t - 1, c);  // behind this step's last exchange loads
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < CH; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wB[ch * CH + i], bv[ch & 1][i][j], acc[j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[wave][j * 4 + r][lane] = acc[j][r];
      if (c == 0) tr.mark(t, 5);
      __syncthreads();
      if (c == 0) tr.mark(t, 6);
      if (fin) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = wave * 4 + r;
          v[r] = (part[0][row][lane] + part[1][row][lane]) + (part[2][row][lane] + part[3][row][lane]);
        }
        if (q < 2) {
#pragma unroll
          for (int r = 0; r < 4; ++r) dh_rec[c][r] = v[r];
        } else if (dxl[c]) {
          xstore4(dx_out + ((size_t)t * B + bb) * H + unit0, floatx4{v[0], v[1], v[2], v[3]});
        }
      }
      // `part` is next written after the barriers of the next point-wise stage
    }
  }
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    signal(flag(l, 0, c) + (s & (kFlagSub - 1)) * kFlagStride, a.full_fences);  // slot 0: dx of step 0 published
    if (pw[c]) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const size_t se = ((size_t)l * B + brow0 + c * BP + lb) * H + unit0 + r;
        if (a.dh0) a.dh0[se] = dh_rec[c][r];
        if (a.dc0) a.dc0[se] = dc[c][r];
      }
    }
  }
}

template <int KG>
hipError_t launch_fwd(BatchPlan bp, int grid, const PersFwdArgs& a, hipStream_t s) {
  void* params[] = {const_cast<PersFwdArgs*>(&a)};
  const void* fn = nullptr;
  if (bp.NT == 1 && bp.NC == 1) fn = (const void*)pers_fwd_kernel<KG, 1, 1>;
  if (bp.NT == 1 && bp.NC == 2) fn = (const void*)pers_fwd_kernel<KG, 1, 2>;
  if (bp.NT == 2 && bp.NC == 2) fn = (const void*)pers_fwd_kernel<KG, 2, 2>;
  if (bp.NT == 2 && bp.NC == 1) fn = (const void*)pers_fwd_kernel<KG, 2, 1>;
  if (bp.NT == 4 && bp.NC == 1) fn = (const void*)pers_fwd_kernel<KG, 4, 1>;
  if (!fn) return hipErrorInvalidValue;
  return launch_resident(fn, grid, params, 0, s);
}

template <int KGB>
hipError_t launch_bwd(BatchPlan bp, int grid, const PersBwdArgs& a, hipStream_t s) {
  void* params[] = {const_cast<PersBwdArgs*>(&a)};
  const void* fn = nullptr;
  if (bp.NT == 1 && bp.NC == 1) fn = (const void*)pers_bwd_kernel<KGB, 1, 1>;
  if (bp.NT == 1 && bp.NC == 2) fn = (const void*)pers_bwd_kernel<KGB, 1, 2>;
  if (bp.NT == 2 && bp.NC == 2) fn = (const void*)pers_bwd_kernel<KGB, 2, 2>;
  if (bp.NT == 2 && bp.NC == 1) fn = (const void*)pers_bwd_kernel<KGB, 2, 1>;
  if (bp.NT == 4 && bp.NC == 1) fn = (const void*)pers_bwd_kernel<KGB, 4, 1>;
  if (!fn) return hipErrorInvalidValue;
  return launch_resident(fn, grid, params, 0, s);
}

}  // namespace

hipError_t launch_fwd_narrow(int H, BatchPlan bp, int grid, const PersFwdArgs& a, hipStream_t s) {
  if (H == 512) return launch_fwd<32>(bp, grid, a, s);
  if (H == 256) return launch_fwd<16>(bp, grid, a, s);
  if (H == 128) return launch_fwd<8>(bp, grid, a, s);
  return hipErrorInvalidValue;
}

hipError_t launch_bwd_narrow(int H, BatchPlan bp, int grid, const PersBwdArgs& a, hipStream_t s) {
  if (H == 512) return launch_bwd<128>(bp, grid, a, s);
  if (H == 256) return launch_bwd<64>(bp, grid, a, s);
  if (H == 128) return launch_bwd<32>(bp, grid, a, s);
  return hipErrorInvalidValue;
}

hipError_t launch_pack_state(const float* h0, float* hx, int L, int T, int B, int H, int BP, int NC, int b0, int nsl, hipStream_t s) {
  const long n = (long)nsl * L * NC * BP * H;
  hipLaunchKernelGGL(pack_state_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, h0, hx, L, T, B, H, BP, NC, b0, nsl);
  return hipGetLastError();
}

}  // namespace lstm
