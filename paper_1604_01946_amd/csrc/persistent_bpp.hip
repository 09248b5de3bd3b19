// Persistent backward recurrence with two chains of 16 batch rows taking turns inside every wave
// (pers_bwd_pp_kernel), for 32 < B <= 64 per slice, H = 128 / 256 / 512, LSTM.
//
// Why.  In pers_bwd32_kernel a step is one dependent sequence per wave: point-wise stage, publication of the gate
// gradients dA_t, the wait until every other workgroup of the layer has published, the matrix instructions, the
// K-split reduction -- and for everything but the fourth item the matrix core idles (about 45 % of a step at
// H = 512).  The recurrences of different batch rows are independent, so here the 32 rows of a workgroup are two
// chains of 16 that alternate, and the product of a step is split in two phases.  Section 4 of arXiv 1604.01946 names
// the underlying idea (weights stay on chip for the whole sequence); Section 2.4's wavefront over layers runs inside
// the grid through per-(layer, step, chain) counters; Section 2.1's remark on the backward pass (four gate gradients
// map to one output through the stacked matrices) is the K = 4H contraction.
//
// Tile.  v_mfma_f32_16x16x4_f32 (the same rate as the 32x32x2 shape).  A workgroup owns 16 hidden units of one
// batch half, as in pers_bwd32_kernel: two M tiles of 16 rows (dh_{t-1} of its units through R_l, and the gradient
// dx_t for the same units of the layer below through W_l), N = the chain's 16 batch rows, K = 4H split over the four
// waves (wave w: the four gate gradients of units [w*H/4, (w+1)*H/4)).  The weight slice [32 x 4H] is shared by both
// chains: 128 registers per lane, the rest (H = 512) in LDS.
//
// Phases of a chain's step t, per wave:
//   A     dh_{t-1} = R_l^T dA_t (tile 0): 4H/16 matrix instructions and nothing else; the operands were requested
//         during the other chain's phase B and stay in registers for this chain's phase B.  Partial sums -> LDS, barrier.
//   post  K-split sums, point-wise stage of step t-1, dA_{t-1} published (exchange slot, standard array).
//   B     dx_t = W_l^T dA_t (tile 1) from the same operand registers.  Nothing waits for it soon (the layer below
//         runs behind), so every round trip of the kernel happens under it: the counters of the other chain's
//         next phase A and of the layer above are looked at, the reserve values of the next point-wise stage (the
//         other chain's, half a period away: the layers of a stack finish one behind the other, each by as much as
//         it has to see of the layer above ahead of time, so nothing is asked for earlier than its round trip needs)
//         and all operands of that phase A are requested.  Its partial sums are added up after the next barrier
//         (the other chain's).
// Order in time: A0 post0 B0 A1 post1 B1 A0 ...: between the publication of a chain's dA_{t-1} and the first
// matrix instruction that needs everybody's dA_{t-1} lie two phases B and one phase A of pure arithmetic, three
// times the exchange round trip; no phase A ever waits.
//
// What one wave can overlap.  With one wave per SIMD (the register budget allows no second) a wave that runs matrix
// instructions back to back pays the full issue time of every other vector instruction: measured on this chip, 31
// cycles per 16-byte global load, 18 per ds_read_b128, 4 to 9 per vector ALU instruction, against 32 per matrix
// instruction; scalar instructions are free.  Hence: addresses are scalar base + fixed lane offset + immediate,
// operand requests are as few and as wide as possible, and post() is kept short.  Its LDS round trips and its
// dependent arithmetic are filled with the first groups of phase B (matrix instructions placed between its pieces).
//
// Exchange layout of one (layer, step, chain) slot, 4H x 16 floats: the four gate gradients (i, f, o, g) of unit u
// and batch row n are one 16-byte piece at piece index (u/4)*64 + (n/4)*16 + (u%4)*4 + n%4.  A lane (kq, n) of the
// B operand fetches its piece of a 4-unit group with one 16-byte load (1 KB per wave and instruction) and feeds
// four matrix instructions per tile from it (K index = gate, k row of the matrices = gate*H + 4*(u/4) + kq).  The
// point-wise stage runs on all four waves, one (unit, row) per lane: wave w has rows 4w..4w+3 of the chain and all
// 16 units, so that the reserve is read and dA / dx are written in runs of 64 bytes; its 64 pieces are transposed
// through a corner of LDS that only this wave touches and leave as four stores of 256 contiguous bytes.
//
// Counters.  One per (layer, index, batch half, chain), T + 2 indices, spread over NL = H/16 lines of 128 bytes;
// every wave arrives on its own (line (4*s + w) % NL: four arrivals per line) once ITS stores are acknowledged.
// Index t+2 = "dA_t of the chain published".  dx_t of chain 0 is stored in chain 1's post() of step t, dx_t of chain 1
// in chain 0's post() of step t-1 (after the barrier that follows the phase B), each in front of that post()'s
// publication, so by issue order: dx_t of chain 0 is covered by index t+1 of chain 1, dx_t of chain 1 by index t of
// chain 0 (index 0: the arrival after the last step).  The only workgroup barrier of a chain-step is the one of the
// K-split reduction (partial sums double-buffered by chain).
//
// Memory requests retire in issue order, loads and stores alike, and every request of this kernel is visible to the
// compiler (no load or store in inline assembly, no request under a branch that the fast path takes): a wait for a
// loaded register therefore waits for exactly the requests up to that load.  A chain's publication is counted at the
// start of the other chain's next phase A: that phase's operands were requested after the stores, so once its first
// operand has arrived the stores are acknowledged.  When a counter was not complete at the point where phase B
// looked, the requests go to an address that is certainly valid and are repeated at the start of the phase that
// needs them (a path that ends with every request complete, so that the compiler's counts stay those of the fast
// path).
#include "../../include/lstm.h"
#include "persistent_dev.h"

namespace lstm {
namespace {

// One of two global addresses, as a value the optimiser cannot look into: a store through `c ? p : q` is otherwise
// turned into two stores under a branch, and a branch ends the region in which matrix instructions and the
// instructions of the point-wise stage can be interleaved.
typedef __attribute__((address_space(1))) float gfloat;
__device__ __forceinline__ gfloat* pick(bool c, const float* p, const float* q) {
  unsigned long long x = c ? reinterpret_cast<unsigned long long>(p) : reinterpret_cast<unsigned long long>(q);
  asm volatile("" : "+v"(x));
  return reinterpret_cast<gfloat*>(x);
}

// CELL = 1: GRU, as in pers_bwd32_kernel.  The four K groups are then the gradients with respect to the r and z
// pre-activations, to W_n x + b_n and to R_n h (the third has no recurrent weights, the fourth no input weights);
// dh_{t-1} also receives the direct term dh_t o z_t (carried in `dc`); the reserve is h [T][B][H] followed by r, z, n,
// R_n h as [T][B][4H]; `h0` takes the place of `c0`, dcT / dc0 are unused, R, W and db have 3H rows.
// CELL = 2 / 3: single-gate RNN (ReLU / tanh): only the first K group is non-zero; the reserve holds h alone.
template <int HH, int GA_, int PL_, int KH_, int FUSE_N_, bool TRACE, int CELL = 0>
__global__ __launch_bounds__(256) void pers_bwd_pp_kernel(const PersBwdArgs a, const int NBH) {
  constexpr int H = HH, G = 4 * H, NS2 = H / 16, NL = NS2;
  constexpr int NGW = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1), GW = NGW * H;  // gate blocks and rows of R, W, db
  constexpr int NU = H / 16;             // groups of four units per wave (its K quarter)
  constexpr int RG = NU < 16 ? NU : 16;  // groups whose weights live in registers
  constexpr int LG = NU - RG;            // groups whose weights live in LDS
  constexpr int GA = GA_;                // group of phase B at which the chain's publication is completed
  constexpr int PL = PL_;                // group of phase B from which the next phase A's operands are requested
  constexpr int KH = KH_;                // groups of phase B that are issued in between the instructions of post()
  constexpr int FUSE_N = FUSE_N_;        // instructions of post() per matrix instruction there
  constexpr int KM = KH - 3;             // groups in between the arithmetic of the point-wise stage
  static_assert(GA >= 1 && GA < NU && PL >= KH && PL < NU && KH >= 4 && KH < NU && (LG == 0 ? KH <= RG : KH + 2 <= RG), "schedule");
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* const part = smem;          // [2 tiles: dh, dx][2 chains][4 waves][64 lanes][4]
  float* const stage = smem + 4096;  // [4 waves][256]
  float* const wl = smem + 5120;     // [4 waves][LG][2 tiles][64 lanes][4 gates]

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
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int u0 = 16 * s2;
  if constexpr (TRACE) {  // (slots 1 and 5 of the first step processed: kernel entry, weights in place; of step 0: last step done, exit)
    if (a.trace && (int)blockIdx.x == a.trace_block && threadIdx.x == 0) a.trace[(size_t)(T - 1) * 8 + 1] = wall_clock64();
  }
  const size_t TB = (size_t)T * B;
  const int NQ = 2 * NBH;
  // The waves of a layer read a slot's K quarter in orders rotated against each other (all of them would otherwise ask
  // the same L2 lines at the same time).  The rotation is a multiple of four groups, so that the address of a request is
  // a scalar base (scalar arithmetic costs the wave no matrix-instruction time, vector arithmetic does) plus the lane's
  // fixed offset plus an immediate.
  const int rot = 4 * (((int)(blockIdx.x >> 3) + w) & (NU / 4 - 1));

  // ---- weights.  A operand of processed group i (unit group ug = w*NU + (i + rot) % NU), gate g, tile tl:
  //      lane (kq = lane / 16, row = lane % 16) holds M_tl[g*H + 4*ug + kq][u0 + row], M_0 = R_l, M_1 = W_l
  float wreg[RG][4][2];
  {
    const int kq = lane >> 4, row = lane & 15;
    const float* Rl = a.R + (size_t)l * GW * H + u0 + row;
    const float* Wl = (l > 0 ? a.W + (size_t)GW * a.I + (size_t)(l - 1) * GW * H : a.W) + u0 + row;  // layer 0: [GW][I], I == H
    const bool live1 = l > 0 || a.dx0;
#pragma unroll
    for (int i = 0; i < NU; ++i) {
      const int ug = w * NU + ((i + rot) & (NU - 1));
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int gm = CELL >= 2 ? 0 : ((CELL == 1 && g == 3) ? 2 : g);  // matrix row block behind K group g
        const size_t k = (size_t)(gm * H + 4 * ug + kq) * H;
        const float v0 = (CELL == 0 || (CELL == 1 ? g != 2 : g == 0)) ? Rl[k] : 0.f;
        const float v1 = (live1 && (CELL == 0 || (CELL == 1 ? g != 3 : g == 0))) ? Wl[k] : 0.f;
        if (i < RG) {
          wreg[i < RG ? i : 0][g][0] = v0;
          wreg[i < RG ? i : 0][g][1] = v1;
        } else {
          wl[((((size_t)w * LG + (i - RG)) * 2 + 0) * 64 + lane) * 4 + g] = v0;
          wl[((((size_t)w * LG + (i - RG)) * 2 + 1) * 64 + lane) * 4 + g] = v1;
        }
      }
    }
  }

  // ---- point-wise role: one (unit, batch row) per lane and chain: unit u0 + m, row 4*w + nl of the chain
  const int nl = lane >> 4, m = lane & 15;
  const int n = 4 * w + nl;
  const int u = u0 + m;
  bool valid[2];
  size_t eoff[2], goff[2];  // offsets of (row, unit) inside a [B][H] and a [B][4H] step (rows past the batch: the last row)
  float dc[2], dh_rec[2], dbsum[2][4];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    const int bb = a.b0 + 32 * bh + 16 * c + n;
    valid[c] = bb < B;
    const int bc = valid[c] ? bb : B - 1;
    eoff[c] = (size_t)bc * H + u;
    goff[c] = (size_t)bc * G + u;
    const size_t se = (size_t)l * B * H + eoff[c];
    dc[c] = (CELL == 0 && valid[c] && a.dcT) ? a.dcT[se] : 0.f;  // GRU: the direct term dh_t o z_t
    dh_rec[c] = (valid[c] && a.dhT) ? a.dhT[se] : 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g) dbsum[c][g] = 0.f;
  }
  // B operand role: lane (kq, nn) fetches piece (nn/4)*16 + kq*4 + nn%4 of every 4-unit group of its K quarter
  const unsigned loff = (unsigned)(((lane & 15) >> 2) * 16 + (lane >> 4) * 4 + (lane & 3)) * 16;  // bytes

  const float* const res_l = a.res + (size_t)l * TB * (CELL == 0 ? 6 : (CELL == 1 ? 5 : 1)) * H;
  const float* const res_gates = CELL == 0 ? res_l : res_l + TB * H;
  const float* const res_c = CELL == 0 ? res_l + TB * 4 * H : res_l;  // c (LSTM) or h: the state array the step reads
  const float* const s0 = CELL == 0 ? a.c0 : a.h0;
  float* const dA_l = a.dA + (size_t)l * TB * G;
  const bool has_up = l < a.L - 1;
  const float* const dout_base = has_up ? a.dxbuf + (size_t)(l + 1) * TB * H : a.dy;
  float* const dx_out = l > 0 ? a.dxbuf + (size_t)l * TB * H : a.dx0;
  const bool dx_wanted = l > 0 || a.dx0;
  float* const dummy = a.dummy + (size_t)blockIdx.x * 32 + (lane & 31);  // a line of this workgroup's own
  // (lq, bq: the layer and batch half as values that the optimiser meets anew in every phase -- the slot and counter
  // addresses are then worked out where they are used, with scalar instructions that cost the wave nothing, instead of
  // being kept in registers across the whole step: the kernel is short of scalar registers, and each one that spills
  // comes back through a vector instruction)
  int lq = l, bq = bh;
  auto rehide = [&]() {
    hide(lq);
    hide(bq);
  };
  auto slot = [&](int t, int c) { return a.dAx + (((size_t)lq * T + t) * NQ + 2 * bq + c) * G * 16; };
  // a slot that no step uses (the exchange array holds T + 1 slots per layer, the steps use T)
  auto spare = [&](int c) { return a.dAx + (((size_t)a.L * T + lq) * NQ + 2 * bq + c) * G * 16; };
  auto flag = [&](int layer, int st, int c) {
    return a.flags + ((((size_t)layer * (T + 2) + st) * NQ + 2 * bq + c) * NL) * kFlagStride;
  };
  const int arrive_line = ((4 * s2 + w) & (NL - 1)) * kFlagStride;

  PpWaiter<NL> wt{a.watchdog, a.spin_limit, false};
  // time stamps of one workgroup's phases (diagnostic hook; a kernel of its own, so that the normal one carries
  // neither the branches nor the registers): per (chain, step) slot 0 = start of phase A, 2 = its end, 3 = past the
  // barrier, 4 = post() and the head of phase B done, 6 = end of phase B
  const PpTracer tr{(TRACE && a.trace && (int)blockIdx.x == a.trace_block) ? a.trace : nullptr, T};
  auto mark = [&](const int c, const int t, const int slot) {
    if constexpr (TRACE) tr.mark(c, t, slot);
  };
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2
  __syncthreads();                                    // LDS weights are in place
  mark(0, T - 1, 5);

  // ---- reserve values and upstream gradient of a chain's next point-wise stage
  float gi[2], gf[2], go[2], gg[2], ct[2], cp[2], dpre[2];
  bool cp_real[2];
  auto fetch_res = [&](const int c, const int t) {
    if (CELL <= 1) {
      const float* const pg = res_gates + (size_t)t * B * G + goff[c];
      gi[c] = pg[0];
      gf[c] = pg[H];
      go[c] = pg[2 * H];
      gg[c] = pg[3 * H];
    }
    if (CELL != 1) ct[c] = res_c[(size_t)t * B * H + eoff[c]];  // c_t (LSTM), h_t (single gate)
    const float* const pc = t > 0 ? res_c + (size_t)(t - 1) * B * H + eoff[c]
                                  : (s0 ? s0 + (size_t)l * B * H + eoff[c] : res_c + eoff[c]);
    cp[c] = *pc;
    cp_real[c] = t > 0 || s0;
  };
  auto fetch_dout = [&](const int c, const int t) { dpre[c] = dout_base[(size_t)t * B * H + eoff[c]]; };

  // ---- point-wise stage of chain c, step t: gate gradients -> exchange slot (published), standard dA array
  //      (`real` false: the stage after step 0, executed so that every step issues the same requests -- its stores go
  //      to a spare slot and a scratch line, and the carried state stays as it is)
  //      In three pieces, so that the matrix instructions of phase B can be placed between them (pw_math ends with a
  //      write to LDS, pw_read with the reads of the transposed values, pw_store issues the stores).
  float pw_d[4], pw_s[4];
  auto pw_math = [&](const int c, const bool real) {
    const float dh = dpre[c] + dh_rec[c];
    const float cpv = cp_real[c] ? cp[c] : 0.f;
    if (CELL == 0) {
      const float tc = tanhf_dev(ct[c]);
      const float dcv = dc[c] + dh * go[c] * (1.f - tc * tc);
      pw_d[0] = dcv * gg[c] * gi[c] * (1.f - gi[c]);
      pw_d[1] = dcv * cpv * gf[c] * (1.f - gf[c]);
      pw_d[2] = dh * tc * go[c] * (1.f - go[c]);
      pw_d[3] = dcv * gi[c] * (1.f - gg[c] * gg[c]);
      dc[c] = real ? dcv * gf[c] : dc[c];
    } else if (CELL >= 2) {  // ct holds h_t
      pw_d[0] = CELL == 3 ? dh * (1.f - ct[c] * ct[c]) : (ct[c] > 0.f ? dh : 0.f);
      pw_d[1] = pw_d[2] = pw_d[3] = 0.f;
    } else {  // gi, gf, go, gg hold r, z, n, R_n h; cpv is h_{t-1}
      const float dn = dh * (1.f - gf[c]) * (1.f - go[c] * go[c]);
      pw_d[0] = dn * gg[c] * gi[c] * (1.f - gi[c]);
      pw_d[1] = dh * (cpv - go[c]) * gf[c] * (1.f - gf[c]);
      pw_d[2] = dn;
      pw_d[3] = dn * gi[c];
      dc[c] = real ? dh * gf[c] : dc[c];
    }
    const bool keep = valid[c] && real;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      pw_d[g] = keep ? pw_d[g] : 0.f;
      dbsum[c][g] += pw_d[g];
    }
    *reinterpret_cast<floatx4*>(stage + w * 256 + (m * 4 + nl) * 4) = floatx4{pw_d[0], pw_d[1], pw_d[2], pw_d[3]};
  };
  auto pw_read = [&]() {
#pragma unroll
    for (int j = 0; j < 4; ++j) pw_s[j] = stage[w * 256 + 64 * j + lane];
  };
  auto pw_store = [&](const int c, const int t, const bool real) {
    const bool keep = valid[c] && real;
    float* const xo = (real ? slot(t, c) : spare(c)) + (size_t)(4 * s2) * 256 + w * 64 + lane;
#pragma unroll
    for (int j = 0; j < 4; ++j) __hip_atomic_store(xo + j * 256, pw_s[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    float* const pd = dA_l + (size_t)t * B * G + goff[c];
#pragma unroll
    for (int g = 0; g < 4; ++g) *pick(keep, pd + g * H, dummy) = pw_d[g];
  };
  auto pointwise = [&](const int c, const int t, const bool real) {
    pw_math(c, real);
    pw_read();
    pw_store(c, t, real);
  };

  // ---- arrival of this wave on the counter of chain c, slot st (its stores up to here are acknowledged)
  auto arrive = [&](const int c, const int st) {
    if (lane == 0) __hip_atomic_fetch_add(flag(lq, st, c) + arrive_line, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };

  int seen_next = 0, seen_up = 0;
  floatx4 op[2][NU];               // B operands of a chain's step: requested during the other chain's phase B, kept until its own
  int rv = rot >> 2;
  // The lane offset as a 32-bit register that the optimiser meets anew in every phase (fresh_lo): next to the scalar base
  // it then becomes the offset operand of the request instead of one 64-bit vector addition per request.
  unsigned lo = loff;
  auto fresh_lo = [&]() {
    lo = loff;
    asm volatile("" : "+v"(lo));
  };
  auto ldx = [&](const float* src, int i) {  // src: the slot (wave-uniform)
    const char* const sb = reinterpret_cast<const char*>(src) + ((size_t)w * NU + 4 * (((i >> 2) + rv) & (NU / 4 - 1))) * 1024;
    return *reinterpret_cast<const floatx4*>(sb + lo + (i & 3) * 1024);
  };
  // counter that stands for "dx of (chain c, step t) of the layer above is published" (see the phases below)
  auto up_flag = [&](const int c, const int t) { return c == 0 ? flag(lq + 1, t + 1, 1) : flag(lq + 1, t, 0); };

  // ---- phase A of chain c, step t: the recurrent half of the product, dh_{t-1} = R_l^T dA_t for the workgroup's
  //      units (the half that the chain's next point-wise stage waits for); no memory request at all
  auto phaseA = [&](const int c, const int t) {
    rehide();
    mark(c, t, 0);
    floatx4 acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f};
    floatx4 al[NU > RG ? NU - RG : 1];
    auto ldw = [&](int g) {
      if (g >= RG && g < NU) al[g - RG] = *reinterpret_cast<const floatx4*>(wl + ((((size_t)w * LG + (g - RG)) * 2 + 0) * 64 + lane) * 4);
    };
    const int o = 1 - c;
    const int tb = c == 0 ? t + 1 : t;  // the phase B before this phase was (o, tb), after post(o, tb): X(o, tb - 1)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < NU; ++g) {
      if (g + 2 >= RG) ldw(g + 2);  // LDS part of the weights, two groups ahead
      if (g == 0 && RG < 2) ldw(RG);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a0 = g < RG ? wreg[g % RG][j][0] : al[g < RG ? 0 : g - RG][j];
        if (j & 1) acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, op[c][g][j], acc2, 0, 0, 0);
        else acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, op[c][g][j], acc, 0, 0, 0);
      }
      if (g == GA) {
        // The other chain's publication (the stores of its post()) was issued before this phase's operands were
        // requested: an operand that has arrived means those stores are acknowledged.
        asm volatile("" : "+v"(op[c][0]));
        if (lane == 0 && tb < T)
          __hip_atomic_fetch_add(flag(lq, tb + 1, o) + arrive_line, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    acc += acc2;
    // counters for phase B (the next phase A's operands, the layer above): read here, ahead of the stores of post(),
    // so that looking at them does not wait for those stores to reach memory
    {
      const int o = 1 - c, tn = c == 0 ? t : t - 1;
      seen_next = PpWaiter<NL>::peek(tn >= 0 ? flag(lq, tn + 2, o) : flag(lq, t + 2, c));
      seen_up = PpWaiter<NL>::peek((has_up && tn > 0) ? up_flag(o, tn - 1) : flag(lq, t + 2, c));
    }
    *reinterpret_cast<floatx4*>(part + (c * 4 + w) * 256 + lane * 4) = acc;
    mark(c, t, 2);
    __syncthreads();
    mark(c, t, 3);
  };

  // ---- after the barrier: K-split sums of dh; dx of the other chain's last phase B (its partial sums were written
  //      before that barrier) goes out; then the chain's point-wise stage of step t-1
  // ---- phase B of chain c, step t: the other half of the product, dx_t = W_l^T dA_t, from the operands still in
  //      registers.  Nothing waits for it soon, so everything with a round trip happens under it: the counters that
  //      phase A read are looked at, the reserve values and the upstream gradient of the next point-wise stage and the
  //      operands of the next phase A (both the other chain's) are requested.  Its first KH groups carry no request: they are issued in
  //      between the pieces of post() -- the K-split sums of dh, dx of the other chain's last phase B (its partial sums
  //      were written before the barrier), the chain's point-wise stage of step t-1 -- which has no matrix instruction
  //      of its own to hide its LDS round trips and its arithmetic behind.
  floatx4 bacc = {0.f, 0.f, 0.f, 0.f}, bacc2 = {0.f, 0.f, 0.f, 0.f};
  auto b_groups = [&](const int c, const int g0, const int g1) {
#pragma unroll
    for (int g = g0; g < g1; ++g) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (j & 1) bacc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(wreg[g][j][1], op[c][g][j], bacc2, 0, 0, 0);
        else bacc = __builtin_amdgcn_mfma_f32_16x16x4f32(wreg[g][j][1], op[c][g][j], bacc, 0, 0, 0);
      }
    }
  };
  auto interleave = [&](const int mfmas) {
#pragma unroll
    for (int i = 0; i < mfmas; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // one matrix instruction
      __builtin_amdgcn_sched_group_barrier(0x7f7, FUSE_N, 0);  // up to FUSE_N of anything else
    }
  };
  auto fused = [&](const int c, const int t) {
    rehide();
    const int o = 1 - c;
    const bool real = t > 0;
    const int tdx = c == 0 ? t + 1 : t;  // step of the other chain's last phase B (none before the very first phase A)
    __builtin_amdgcn_sched_barrier(0);
    // 1: the partial sums are requested; one group of matrix instructions covers the round trip
    const int ri = ((m >> 2) * 16 + n) * 4 + (m & 3);
    const float* const pb = part + c * 1024 + ri;
    const float* const px = part + 2048 + o * 1024 + ri;
    const float h0 = pb[0], h1 = pb[256], h2 = pb[512], h3 = pb[768];
    const float x0 = px[0], x1 = px[256], x2 = px[512], x3 = px[768];
    bacc = floatx4{0.f, 0.f, 0.f, 0.f};
    bacc2 = floatx4{0.f, 0.f, 0.f, 0.f};
    __builtin_amdgcn_sched_barrier(0);
    b_groups(c, 0, 1);
    __builtin_amdgcn_sched_barrier(0);
    // 2: sums, dx out, the arithmetic of the point-wise stage, its gate gradients into LDS -- in between KM groups
    dh_rec[c] = CELL == 1 ? ((h0 + h1) + (h2 + h3)) + dc[c] : (h0 + h1) + (h2 + h3);
    const float dxv = (x0 + x1) + (x2 + x3);
    // (every step issues the same requests, whatever is wanted: what is not goes to the workgroup's scratch line)
    __hip_atomic_store(pick(dx_wanted && valid[o] && tdx < T, dx_out + (size_t)tdx * B * H + eoff[o], dummy), dxv, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    pw_math(c, real);
    b_groups(c, 1, 1 + KM);
    interleave(4 * KM);
    __builtin_amdgcn_sched_barrier(0);
    // 3: the transposed values are requested; one group covers the round trip
    pw_read();
    __builtin_amdgcn_sched_barrier(0);
    b_groups(c, 1 + KM, 2 + KM);
    __builtin_amdgcn_sched_barrier(0);
    // 4: the stores, in between the remaining groups
    pw_store(c, real ? t - 1 : 0, real);
    b_groups(c, 2 + KM, KH);
    interleave(4 * (KH - 2 - KM));
    __builtin_amdgcn_sched_barrier(0);
    mark(c, t, 4);
  };
  auto b_rest = [&](const int c, const int t) {
    rehide();
    const int o = 1 - c;
    const int tn = c == 0 ? t : t - 1;  // the next phase A is (o, tn)
    const bool has_next = tn >= 0;
    // the next point-wise stage is the other chain's, in post(o, tn), of step tn - 1 (if any): what it needs from the
    // reserve and from the layer above is requested here, half a period ahead of its use
    const int tq = tn > 0 ? tn - 1 : 0;
    const bool has_pw = tn > 0;
    fetch_res(o, tq);
    // operands of the next phase A; when there is none, this chain's own slot once more (valid memory, values unused),
    // so that every step issues the same requests
    const float* const nsrc = has_next ? slot(tn, o) : slot(t, c);
    floatx4 al[NU > RG ? NU - RG : 1];
    auto ldw = [&](int g) {
      if (g >= RG && g < NU) al[g - RG] = *reinterpret_cast<const floatx4*>(wl + ((((size_t)w * LG + (g - RG)) * 2 + 1) * 64 + lane) * 4);
    };
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = KH; g < NU; ++g) {
      if (g + 2 >= RG) ldw(g + 2);
      if (g == PL) {
        // The counters were read before this chain's post(); they are almost always complete (the publications they
        // count are two phases old).  When one is not, the wave polls right here: nothing that it could do instead
        // would get it past the next barrier any sooner, and no other workgroup waits for this one meanwhile (every
        // counter that it feeds was fed before this phase).
        PpWaiter<NL>::land(seen_next);
        PpWaiter<NL>::land(seen_up);
        if (has_next) wt.wait(flag(lq, tn + 2, o), 4, seen_next);
        if (has_up && has_pw) wt.wait(up_flag(o, tq), 4, seen_up);
        fetch_dout(o, tq);
        fresh_lo();
      }
      if (g >= PL) {  // operand groups [lo, hi) of the next phase A, spread evenly over groups PL..NU-1
        constexpr int span = NU - PL, HB = NU;
        const int lo = ((g - PL) * HB) / span, hi = ((g - PL + 1) * HB) / span;
#pragma unroll
        for (int j = lo; j < hi; ++j) op[o][j] = ldx(nsrc, j);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a1 = g < RG ? wreg[g % RG][j][1] : al[g < RG ? 0 : g - RG][j];
        if (j & 1) bacc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, op[c][g][j], bacc2, 0, 0, 0);
        else bacc = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, op[c][g][j], bacc, 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    bacc += bacc2;
    *reinterpret_cast<floatx4*>(part + 2048 + (c * 4 + w) * 256 + lane * 4) = bacc;
    mark(c, t, 6);
  };

  // ---- the last step's point-wise stage of both chains
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    fetch_res(c, T - 1);
    if (has_up) wt.wait(up_flag(c, T - 1), 4, 0);
    fetch_dout(c, T - 1);
    pointwise(c, T - 1, true);
  }
  drain_vmem();
  arrive(0, T + 1);
  arrive(1, T + 1);
  // what the first phases need and later ones find requested by the phase B before them: the reserve values and the
  // upstream gradient of step T-2 for the point-wise stage in chain 0's first post(), and chain 0's operands
  {
    fetch_res(0, T > 1 ? T - 2 : 0);
    if (has_up && T > 1) wt.wait(up_flag(0, T - 2), 4, 0);
    fetch_dout(0, T > 1 ? T - 2 : 0);
  }
  wt.wait(flag(lq, T + 1, 0), 4, 0);
  fresh_lo();
#pragma unroll
  for (int i = 0; i < NU; ++i) op[0][i] = ldx(slot(T - 1, 0), i);
  for (int t = T - 1; t >= 0; --t) {
    hide(rv);
    phaseA(0, t);
    fused(0, t);
    b_rest(0, t);
    hide(rv);
    phaseA(1, t);
    fused(1, t);
    b_rest(1, t);
  }
  // the last phase B's publication (the stage after step 0 of chain 1: nothing but dx of chain 0, step 0, rides on it)
  drain_vmem();
  arrive(1, 1);
  // dx of chain 1, step 0
  __syncthreads();
  {
    const float* const px = part + 2048 + 1024 + ((m >> 2) * 16 + n) * 4 + (m & 3);
    const float dxv = (px[0] + px[256]) + (px[512] + px[768]);
    if (dx_wanted && valid[1]) __hip_atomic_store(dx_out + eoff[1], dxv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  drain_vmem();
  arrive(0, 0);
  mark(0, 0, 1);

#pragma unroll
  for (int c = 0; c < 2; ++c) {
    if (valid[c]) {
      const size_t se = (size_t)l * B * H + eoff[c];
      if (a.dh0) a.dh0[se] = dh_rec[c];
      if (CELL == 0 && a.dc0) a.dc0[se] = dc[c];
    }
  }
  // Bias gradient (Section 2.6 lists it with the weight update): the per-lane sums over t are added over the 32
  // batch rows of this workgroup through LDS, in a fixed order, and then into db.  Each element of db receives exactly
  // one contribution per batch half, and a + b does not depend on which of the two arrives first.
  if (a.db) {
    __syncthreads();
#pragma unroll
    for (int g = 0; g < 4; ++g) part[(g * 16 + m) * 16 + n] = dbsum[0][g] + dbsum[1][g];
    __syncthreads();
    if (threadIdx.x < 16 * NGW) {
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) sum += part[threadIdx.x * 16 + ((i + threadIdx.x) & 15)];
      atomicAdd(a.db + (size_t)l * GW + (threadIdx.x >> 4) * H + u0 + (threadIdx.x & 15), sum);
    }
  }
  mark(0, 0, 5);
}

template <int HH, int CELL>
hipError_t launch_bpp(const PersBwdArgs& a, int nbh, hipStream_t s) {
  constexpr int NU = HH / 16, LG = NU > 16 ? NU - 16 : 0;
  const size_t smem = (5120 + (size_t)4 * LG * 2 * 64 * 4) * sizeof(float);
  // Schedule (measured at H = 512; the alternatives within 1 %): the other chain's publication is counted one group
  // into phase A; a quarter of phase B runs in between the pieces of post(), six of its instructions per matrix
  // instruction; the next phase A's operands are requested during the rest of phase B, from group PL on.
  // At H = 512 the counters are looked at, and the requests begin, at group 12 of the 32 (cfg3 backward recurrence by
  // that group: 8 1.047 ms, 10 1.038, 12 1.032, 13 1.031, 14 1.042, 16 1.058: looking later also lets a layer follow
  // the one above more closely).
  constexpr int KH = NU / 4 < 4 ? 4 : NU / 4;
  constexpr int PL = HH == 512 ? 12 : KH;
  const bool trace = a.trace != nullptr;
  const void* fn = trace ? (const void*)pers_bwd_pp_kernel<HH, 1, PL, KH, 6, true, CELL>
                         : (const void*)pers_bwd_pp_kernel<HH, 1, PL, KH, 6, false, CELL>;
  static bool attr_set[2] = {false, false};
  if (hipError_t e = allow_dynamic_lds(fn, smem, attr_set[trace ? 1 : 0]); e != hipSuccess) return e;
  void* params[] = {const_cast<PersBwdArgs*>(&a), &nbh};
  const int grid = a.L * (HH / 16) * nbh;
  return launch_resident(fn, grid, params, (unsigned)smem, s);
}

}  // namespace

template <int CELL>
hipError_t launch_bpp_h(int H, const PersBwdArgs& a, int nbh, hipStream_t s) {
  if (H == 512) return launch_bpp<512, CELL>(a, nbh, s);
  if (H == 256) return launch_bpp<256, CELL>(a, nbh, s);
  if (H == 128) return launch_bpp<128, CELL>(a, nbh, s);
  return hipErrorInvalidValue;
}

hipError_t launch_bwd_pp(int cell, int H, const PersBwdArgs& a, int nbh, hipStream_t s) {  // cell 0: LSTM, 1: GRU, 2: ReLU, 3: tanh
  if (cell == 1) return launch_bpp_h<1>(H, a, nbh, s);
  if (cell == 2) return launch_bpp_h<2>(H, a, nbh, s);
  if (cell == 3) return launch_bpp_h<3>(H, a, nbh, s);
  if (cell != 0) return hipErrorInvalidValue;
  if (H == 512) return launch_bpp<512, 0>(a, nbh, s);
  if (H == 256) return launch_bpp<256, 0>(a, nbh, s);
  if (H == 128) return launch_bpp<128, 0>(a, nbh, s);
  return hipErrorInvalidValue;
}

}  // namespace lstm
