// Persistent forward recurrence with two half-slices of 32 batch rows taking turns inside every wave
// (pers_fwd_pp_kernel), for 32 < B <= 64 per slice, H = 128 / 256 / 512, LSTM, every layer multiplying its input
// itself (layers >= 1 always do; layer 0 when I == H and x arrives in exchange layout).
//
// Why.  In pers_fwd32_kernel a step of 64 rows is one dependent sequence per wave: matrix instructions, K-split
// reduction, gates, publication of h_t, and then the wait until every other workgroup of the layer has published
// -- for the last part of that list the matrix core idles (about 30 % of a step at H = 512).  The recurrences of
// different batch rows are independent, so here the slice is two chains of 32 rows that alternate: while the
// h_t of one chain is on its way to the other workgroups (store acknowledgement, counter, propagation, the
// fetch of the operand), the wave multiplies for the other chain.  The acknowledgement of a chain's store is
// awaited, and its counter bumped, some groups of matrix instructions into the other chain's block; a chain's gates
// are computed in between the first matrix instructions of the other chain's next block; the whole input half of
// a chain's next operand is requested during the other chain's block: none of these round trips
// has the matrix core waiting.  Section 4 of arXiv 1604.01946 names the underlying idea (weights stay on chip
// for the whole sequence); Section 2.4's wavefront over layers runs inside the grid through per-(layer, step,
// chain) counters.
//
// Tile.  v_mfma_f32_32x32x2_f32, M = 32 weight rows, N = the chain's 32 batch rows, K = 2H split over the
// workgroup's four waves (one per SIMD; the weights are in registers once, shared by both chains).  Row rho of
// the A operand holds (gate rho/8, unit 2*(rho%4) + (rho/4)%2): in the D layout a lane (kk, n) then holds, for
// each gate, units kk, 2+kk, 4+kk, 6+kk of batch row n, which is one 16-byte piece of the exchange layout
// below, and after the transposition through LDS every wave publishes two whole 128-byte lines with one
// coalesced 4-byte-per-lane store.
//
// Exchange layout of one (layer, step, chain) slot, H x 32 floats: element for k = 8*k8 + 2*i + kk and batch
// row n at ((k8*2 + kk)*32 + n)*4 + i.  A lane (kk, n) fetches the four k-pairs of an 8-k group with one
// 16-byte load (1 KB per wave and instruction); the 8 units of slice s are the contiguous KB k8 = s.
//
// Counters.  One per (slice group, layer, step, chain), spread over NL = H/16 lines of 128 bytes; every wave
// arrives on its own (line (4*s + q) % NL: eight arrivals per line) once ITS store of h_t is acknowledged, so
// publishing needs no workgroup barrier.  The only barrier of a chain-step is the one of the K-split reduction;
// the partial sums are double-buffered so that this one suffices.
//
// The wait for a store's acknowledgement relies on the counter of outstanding vector-memory operations
// retiring in issue order: "at most N outstanding" means everything but the N youngest requests is complete, and
// at least N loads always follow a publication before that wait.  Operations with a run-time count (the polls of
// a wait that really has to spin) are followed by a full drain.  The kernel must not spill registers to scratch
// memory (spill traffic would be counted too; it could only make the wait longer, never shorter).
#include "../../include/lstm.h"
#include "persistent_dev.h"

namespace lstm {
namespace {

constexpr int pp_count(int lo, int hi, int upto) { return upto < lo ? 0 : ((upto < hi ? upto : hi) - lo + 1); }

// CELL = 1 runs a GRU on the same machinery, as pers_fwd32_kernel does (convention of rnn.h: gates r, z, n; the reset
// gate multiplies the recurrent product): the four row groups of a workgroup's tile are then r, z, the input half of
// n (W_n x, no recurrent weights) and the recurrent half of n (R_n h, no input weights); its reserve is h [T][B][H]
// followed by r, z, n, R_n h as [T][B][4H], and `c0` is not used (the carried state is h).
// CELL = 2 / 3: single-gate RNN with ReLU / tanh: only the first row group carries weights; the reserve is h [T][B][H].
template <int HH, int GA_, int PF_, bool TRACE, int CELL = 0>
__global__ __launch_bounds__(256) void pers_fwd_pp_kernel(const PersFwdArgs a) {
  constexpr int NGT = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1);  // gate blocks of W, R, b
  constexpr int H = HH, G = NGT * H, NS = H / 8, NL = H / 16;  // G: rows of W, R, b
  constexpr int NK8 = H / 32;        // 8-k groups per wave and operand half (K-quarter of H)
  constexpr int NG = 2 * NK8;        // groups of a block: input half, then recurrent half
  constexpr int LAG = NK8 / 4;       // group at which the recurrent operand's fetch begins (its counter is looked at there)
  constexpr int GA = GA_;            // group at which the other chain's previous publication is completed
  constexpr int PF = PF_;            // group at which the fetch of the other chain's next input begins
  // requests certainly issued between a publication and its completion: recurrent groups and input groups up to GA
  constexpr int NYOUNG = pp_count(LAG, LAG + NK8 - 1, GA) + pp_count(PF, PF + NK8 - 1, GA);
  static_assert(NYOUNG >= 1 && NYOUNG < 60 && PF + NK8 <= NG && GA < NG, "schedule");
  __shared__ __attribute__((aligned(16))) float part[2][4][1024];  // [buffer][wave][gate][kk][n][4]
  __shared__ __attribute__((aligned(16))) float stage[4][6 * 64];  // per wave: i, f, o, c', c, h of its 8 rows x 8 units

  int l, s;
  map_block(a.L, NS * a.nsl, l, s);
  const int sl = s / NS;
  s -= sl * NS;
  const int T = a.T, B = a.B;
  const int lane = threadIdx.x & 63;
  const int q = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kk = lane >> 5, n = lane & 31;
  const int u0 = 8 * s;
  const size_t TB = (size_t)T * B;
  // The waves of a layer read a slot in orders rotated against each other (all of them would otherwise ask the same
  // L2 lines at the same time).  The rotation is a multiple of four groups, so that the address of a request is a scalar
  // base plus the lane's fixed offset plus an immediate: scalar arithmetic costs a wave that runs matrix instructions
  // back to back nothing, every vector instruction costs its full issue time (one wave per SIMD: nothing else to issue).
  constexpr int NR4 = NK8 / 4 > 0 ? NK8 / 4 : 1;
  const int rot = NK8 >= 4 ? 4 * (((int)(blockIdx.x >> 3) + q) & (NR4 - 1)) : 0;

  if constexpr (TRACE) {  // (slot 5 of step 0: kernel entry under chain 1, weights in place under chain 0)
    if (a.trace && (int)blockIdx.x == a.trace_block && threadIdx.x == 0) a.trace[((size_t)T + 0) * 8 + 5] = wall_clock64();
  }
  // ---- weights -> registers.  A operand of group register i (k8 = (i + rot) % NK8), k-pair j:
  //      row rho = lane % 32 = 8*gate + 4*par + cc holds unit 2*cc + par; k = q*H/4 + 8*k8 + 2*j + kk
  float wR[NK8][4], wW[NK8][4];
  {
    const float* Rl = a.R + (size_t)l * G * H;
    const float* Wl = l > 0 ? a.W + (size_t)G * a.I + (size_t)(l - 1) * G * H : a.W;  // layer 0: [G][I] with I <= H
    const int Il = l > 0 ? H : a.I;  // columns of Wl (x comes zero-padded to H columns)
    const int grp = n >> 3, par = (n >> 2) & 1, cc = n & 3;
    const int gate = CELL >= 2 ? 0 : ((CELL == 1 && grp == 3) ? 2 : grp);  // matrix row block behind tile row group grp
    const bool useR = CELL == 0 || (CELL == 1 ? grp != 2 : grp == 0), useW = CELL == 0 || (CELL == 1 ? grp != 3 : grp == 0);
    const size_t row = ((size_t)gate * H + u0 + 2 * cc + par) * H;
    const size_t rowW = ((size_t)gate * H + u0 + 2 * cc + par) * Il;
#pragma unroll
    for (int i = 0; i < NK8; ++i) {
      const int k8 = (i + rot) & (NK8 - 1);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = q * (H / 4) + 8 * k8 + 2 * j + kk;
        wR[i][j] = useR ? Rl[row + k] : 0.f;
        wW[i][j] = (useW && k < Il) ? Wl[rowW + k] : 0.f;
      }
    }
  }

  // ---- the cell this lane finalises after the transposition (the same position in both chains): exchange
  //      position p = lane % 32 of the wave's quarter, i.e. batch row 8*q + p/4 of the chain, unit 2*(p%4) + kk
  const int p = lane & 31;
  const int nr = 8 * q + (p >> 2);
  const int unit = u0 + 2 * (p & 3) + kk;
  int bb[2];
  bool valid[2];
  float c_state[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    bb[c] = a.b0 + 64 * sl + 32 * c + nr;
    valid[c] = bb[c] < B;
    const float* const s0 = CELL == 0 ? a.c0 : (CELL == 1 ? a.h0 : nullptr);  // the carried state: c (LSTM), h (GRU)
    c_state[c] = (valid[c] && s0) ? s0[((size_t)l * B + bb[c]) * H + unit] : 0.f;
  }
  float bias[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) bias[g] = g < NGT ? a.bias[(size_t)l * G + g * H + unit] : 0.f;

  float* const res_l = a.res + (size_t)l * TB * (CELL == 0 ? 6 : (CELL == 1 ? 5 : 1)) * H;
  float* const res_gates = CELL == 0 ? res_l : res_l + TB * H;  // LSTM, GRU
  float* const res_c = res_l + TB * 4 * H;  // LSTM only
  float* const res_h = CELL == 0 ? res_l + TB * 5 * H : res_l;
  float* const hx = a.hx + (size_t)sl * a.L * (T + 1) * H * 64;
  int* const flags = a.flags + (size_t)sl * a.L * (T + 1) * 2 * NL * kFlagStride;
  auto slot = [&](int layer, int st, int c) { return hx + (((size_t)layer * (T + 1) + st) * 2 + c) * H * 32; };
  auto flag = [&](int layer, int st, int c) { return flags + (((size_t)layer * (T + 1) + st) * 2 + c) * NL * kFlagStride; };
  const int arrive_line = ((4 * s + q) & (NL - 1)) * kFlagStride;
  // the layer below is, for layer 0, the input sequence itself: x in exchange layout, all of it there before the launch
  const bool in_is_x = l == 0;
  const float* const in_base = in_is_x ? a.xin + (size_t)sl * (T + 1) * H * 64 : slot(l - 1, 0, 0);
  auto in_slot = [&](int st, int c) { return in_base + ((size_t)st * 2 + c) * H * 32; };
  auto in_flag = [&](int st, int c) { return in_is_x ? flag(0, 0, c) : flag(l - 1, st, c); };  // x: never waited for

  PpWaiter<NL> w{a.watchdog, a.spin_limit, false};
  // time stamps of one workgroup's phases (diagnostic hook; a kernel instance of its own, so that the normal one carries
  // neither the branches nor the registers)
  const PpTracer trc{(TRACE && a.trace && (int)blockIdx.x == a.trace_block) ? a.trace : nullptr, T};
  struct {
    const PpTracer& t;
    __device__ __forceinline__ void mark(int c, int step, int slot) const {
      if constexpr (TRACE) t.mark(c, step, slot);
    }
  } tr{trc};
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2

  int rv = rot >> 2;
  // The lane offset as a 32-bit register that the optimiser meets anew in every block (fresh_lo): next to the scalar
  // base it then becomes the offset operand of the request instead of one 64-bit vector addition per request.
  unsigned lo = lane * 16;
  auto fresh_lo = [&]() {
    lo = lane * 16;
    asm volatile("" : "+v"(lo));
  };
  auto ldx = [&](const float* src, int i) {  // src: the slot (wave-uniform); group i of this wave's K quarter
    const char* const sb = reinterpret_cast<const char*>(src) +
                           ((size_t)q * NK8 + (NK8 >= 4 ? 4 * (((i >> 2) + rv) & (NR4 - 1)) : 0)) * 1024;
    return *reinterpret_cast<const floatx4*>(sb + lo + (NK8 >= 4 ? (i & 3) : i) * 1024);
  };
  auto mma4 = [&](floatx16& acc, const float (&wgt)[4], const floatx4& bv) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wgt[j], bv[j], acc, 0, 0, 0);
  };

  // Operands of a chain, one register quad per group: at the start of the chain's block its ring holds the whole
  // input half (requested during the other chain's block); slot i is refilled with recurrent group i as soon as
  // input group i has been consumed, LAG groups behind.
  floatx4 ring[2][NK8];
  int seen_rec = 1 << 30;              // the next block's own-layer counter, read during the block before it

  // ---- completes the publication of chain c's step t: the store is acknowledged once at most NYOUNG younger
  //      requests are outstanding (none for the very last one); then the counter
  auto complete = [&](const int c, const int t, const bool last) {
    if (last) drain_vmem();
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NYOUNG) : "memory");
    if (lane == 0) __hip_atomic_fetch_add(flag(l, t + 1, c) + arrive_line, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    tr.mark(c, t, 6);
  };

  // ---- one block: the matrix instructions of chain c's step t, then its reduction, gates and the store of h_t.
  //      Memory requests of a block, in order: the counter of the other chain's next input; recurrent groups from
  //      group LAG on; from group NK8 on the other chain's next input (its own if the layer below has published,
  //      else this chain's recurrent slot once more: valid memory, values unused, real fetch at the end of the
  //      block); the next block's own-layer counter; the store of h_t.  Nothing with a run-time count follows the
  //      store before the next block completes it.
  floatx16 acc;
  // ---- the first LAG groups of a block: operands long in registers, no memory request; issued together with the
  //      other chain's gates (see fused below)
  auto head = [&](const int c) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int g = 0; g < LAG; ++g) mma4(acc, wW[g], ring[c][g]);
  };
  auto block = [&](const int c, const int t) {
    tr.mark(c, t, 0);
    const int tn = c == 0 ? t + 1 : t + 2;  // input slot of the other chain's next block: its step t (c == 0) or t + 1
    const bool other_next = tn <= T;        // that block exists
    int seen_in = PpWaiter<NL>::peek(in_flag(other_next ? tn : T, 1 - c));
    const float* const rsrc = slot(l, t, c);
    fresh_lo();
    const float* nsrc = rsrc;
    bool fetched = false;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = LAG; g < NG; ++g) {
      if (g == LAG) {  // h_{l,t-1} of this chain must be published (slot 0 was written before the launch)
        PpWaiter<NL>::land(seen_rec);
        w.wait(flag(l, t, c), 8, t > 0 ? seen_rec : 8);
        tr.mark(c, t, 2);
        fresh_lo();  // (after every branch: the offset has to be defined in the basic block of the requests)
      }
      if (g == PF) {
        PpWaiter<NL>::land(seen_in);
        fetched = other_next && !w.dead && (in_is_x || __all(seen_in >= 8));
        if (fetched) nsrc = in_slot(tn, 1 - c);
      }
      const floatx4 cur = ring[c][g % NK8];
      if (g >= LAG && g < LAG + NK8) ring[c][g - LAG] = ldx(rsrc, g - LAG);
      if (g >= PF && g < PF + NK8) ring[1 - c][g - PF] = ldx(nsrc, g - PF);
      if (g < NK8) mma4(acc, wW[g], cur);
      else mma4(acc, wR[g - NK8], cur);
      if (g == GA) {
        if (c == 1 || t > 0) complete(1 - c, c == 1 ? t : t - 1, false);  // the other chain's previous step
        fresh_lo();
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    tr.mark(c, t, 1);
    if (other_next && !fetched) {  // the layer below was late: wait for it now (before this chain's store)
      w.wait(in_flag(tn, 1 - c), 8, 0);
      const float* src = in_slot(tn, 1 - c);
#pragma unroll
      for (int i = 0; i < NK8; ++i) ring[1 - c][i] = ldx(src, i);
    }
    float* const mine = &part[(2 * t + c) & 1][q][0];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<floatx4*>(mine + ((g * 2 + kk) * 32 + n) * 4) =
          floatx4{acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
    // the own-layer counter that the next block (the other chain's) waits for: read now, looked at LAG groups into it
    {
      const int st = c == 0 ? t : t + 1;  // that block is (1, t) or (0, t + 1): it needs h of step st - 1
      seen_rec = PpWaiter<NL>::peek(flag(l, (st > 0 && st < T) ? st : 1, 1 - c));
    }
    tr.mark(c, t, 3);
    __syncthreads();
    tr.mark(c, t, 4);
  };
  // ---- after the barrier, first part (straight-line code): K-split sums, gates, the store of h_t, the six values
  //      of the cell into the wave's corner of LDS
  auto post_a = [&](const int c, const int t) {
    const float* const all = &part[(2 * t + c) & 1][0][0] + kk * 128 + 32 * q + p;
    float sg[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      sg[g] = (all[g * 256] + all[1024 + g * 256]) + (all[2048 + g * 256] + all[3072 + g * 256]) + bias[g];
    float gi, gf, go, gc, cn, hn;
    if (CELL == 0) {
      gi = sigmoidf_dev(sg[0]), gf = sigmoidf_dev(sg[1]), go = sigmoidf_dev(sg[2]), gc = tanhf_dev(sg[3]);
      cn = gf * c_state[c] + gi * gc;
      hn = go * tanhf_dev(cn);
      c_state[c] = cn;
    } else if (CELL >= 2) {
      gi = gf = go = gc = cn = 0.f;
      hn = CELL == 3 ? tanhf_dev(sg[0]) : fmaxf(sg[0], 0.f);
    } else {  // sg: r and z pre-activations, W_n x + b_n, R_n h; the four saved values: r, z, n, R_n h
      gi = sigmoidf_dev(sg[0]), gf = sigmoidf_dev(sg[1]);
      go = tanhf_dev(sg[2] + gi * sg[3]);
      gc = sg[3];
      hn = (1.f - gf) * go + gf * c_state[c];
      cn = 0.f;
      c_state[c] = hn;
    }
    // publish: the wave's 64 values are two whole 128-byte lines of the slot
    __hip_atomic_store(slot(l, t + 1, c) + (size_t)s * 256 + kk * 128 + 32 * q + p, valid[c] ? hn : 0.f, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    // The reserve and the outputs (nobody reads them before the kernel ends) go out right behind it, as 16-byte
    // pieces: the wave's 8 rows x 8 units of each of the six arrays are transposed through a corner of LDS that only
    // this wave touches.  Stores to memory retire slowly and in order with the loads: anywhere later they would sit
    // in front of operands that the next block is about to need.
    {
      float* const st = &stage[q][0];
      const int so = (p >> 2) * 8 + 2 * (p & 3) + kk;  // (row of the wave's eight, unit of the slice)
      st[so] = gi; st[64 + so] = gf; st[128 + so] = go; st[192 + so] = gc; st[256 + so] = cn; st[320 + so] = hn;
    }
  };
  // ---- second part: the reserve and the outputs as 16-byte pieces.  Every wave issues the same three stores in
  //      every step, whatever its rows and the call want written: a piece that is not wanted goes to a scratch line.
  //      With no branch around them the compiler knows how many requests are outstanding behind the counter that the
  //      next block looks at, and waits for that counter alone instead of for these stores to reach memory.
  auto post_b = [&](const int c, const int t) {
    const float* const st = &stage[q][0];
    const bool lastt = t == T - 1, top = l == a.L - 1;
    float* const scratch_line = a.dummy + 4 * (lane & 7);
    const int row = (lane >> 1) & 7, hf = lane & 1;
    const int br = a.b0 + 64 * sl + 32 * c + 8 * q + row;
    const bool in_batch = br < B;
    const size_t e = ((size_t)t * B + br) * H + u0 + 4 * hf;
    const size_t se = ((size_t)l * B + br) * H + u0 + 4 * hf;
    {  // gates: piece (array lane/16, row, half)
      const int arr = lane >> 4;
      const floatx4 v = *reinterpret_cast<const floatx4*>(st + arr * 64 + row * 8 + 4 * hf);
      float* const dst = (in_batch && a.keep && CELL <= 1) ? res_gates + ((size_t)t * B + br) * 4 * H + (size_t)arr * H + u0 + 4 * hf : scratch_line;
      *reinterpret_cast<floatx4*>(dst) = v;
    }
    {  // lanes 0-15: c, lanes 16-31: h (upper lanes repeat them into the scratch line)
      const int arr = 4 + ((lane >> 4) & 1);
      const floatx4 v = *reinterpret_cast<const floatx4*>(st + arr * 64 + row * 8 + 4 * hf);
      const bool mine = in_batch && lane < 32;
      float* const dst = (mine && a.keep && (CELL == 0 || arr == 5)) ? (arr == 4 ? res_c : res_h) + e : scratch_line;
      *reinterpret_cast<floatx4*>(dst) = v;
      float* const dsty = (mine && top && arr == 5) ? a.y + e : scratch_line;
      *reinterpret_cast<floatx4*>(dsty) = v;
      if (lastt && mine) {
        if (CELL == 0 && arr == 4 && a.cT) *reinterpret_cast<floatx4*>(a.cT + se) = v;
        if (arr == 5 && a.hT) *reinterpret_cast<floatx4*>(a.hT + se) = v;
      }
    }
  };
  // ---- a chain's gates and stores have no matrix instruction of their own chain to hide behind, but the other
  //      chain's next block has: its first LAG groups are issued in between (one matrix instruction, then a
  //      handful of the other instructions, and so on)
  auto fused = [&](const int cp, const int tp, const int cn) {
    post_a(cp, tp);
    head(cn);
#pragma unroll
    for (int i = 0; i < 4 * LAG; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one matrix instruction
      __builtin_amdgcn_sched_group_barrier(0x7f7, 8, 0);   // up to eight of anything else
    }
    __builtin_amdgcn_sched_barrier(0);
    post_b(cp, tp);
  };

  tr.mark(0, 0, 5);
  // ---- chain 0's first input operand (chain 1's is requested by chain 0's first block)
  {
    if (!in_is_x) w.wait(in_flag(1, 0), 8, 0);
    const float* src = in_slot(1, 0);
#pragma unroll
    for (int i = 0; i < NK8; ++i) ring[0][i] = ldx(src, i);
  }
  // (the loop is rotated so that every look at a counter follows the stores before it in straight-line code)
  head(0);
  hide(rv);
  block(0, 0);
  for (int t = 0; t < T; ++t) {
    fused(0, t, 1);
    block(1, t);
    if (t + 1 < T) {
      hide(rv);
      fused(1, t, 0);
      block(0, t + 1);
    }
  }
  post_a(1, T - 1);
  post_b(1, T - 1);
  complete(1, T - 1, true);  // chain 0's last publication was completed inside chain 1's last block
}

// h0 [L][B][H] (zeros if null) -> exchange slot 0 of every (slice, layer, chain) in the layout above; rows past the
// batch hold zeros.
__global__ void pack_state_pp_kernel(const float* __restrict__ h0, float* __restrict__ hx, int L, int T, int B, int H, int b0,
                                     int nsl) {
  const long cnt = (long)nsl * L * 64 * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < cnt; e += (long)gridDim.x * blockDim.x) {
    const int k = (int)(e % H), lb = (int)((e / H) % 64), l = (int)((e / ((long)H * 64)) % L);
    const int sl = (int)(e / ((long)H * 64 * L));
    const int c = lb >> 5, n = lb & 31, k8 = k >> 3, i = (k >> 1) & 3, kk = k & 1;
    const int bb = b0 + 64 * sl + lb;
    hx[((((size_t)sl * L + l) * (T + 1)) * 2 + c) * H * 32 + ((size_t)(k8 * 2 + kk) * 32 + n) * 4 + i] =
        (h0 && bb < B) ? h0[((size_t)l * B + bb) * H + k] : 0.f;
  }
}

// x [T][B][I] (I <= H) -> slots 1..T of xin [nsl][T+1][2][H*32] in the layout above, rows past the batch and columns
// past I zero (layer 0 then multiplies H columns like every other layer; its weights beyond column I are zero as well).
// Block (kb, t, sl) moves the 64 batch rows x 64 inputs [64*kb, 64*kb+64) of one step through LDS: whole rows in,
// one contiguous 8 KB piece of each chain's slot out.
__global__ __launch_bounds__(256) void pack_x_pp_kernel(const float* __restrict__ x, float* __restrict__ xin, int T, int B,
                                                        int I, int H, int b0, int nsl) {
  __shared__ float tile[64][65];
  const int kb = blockIdx.x, t = blockIdx.y, sl = blockIdx.z;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int e = threadIdx.x + 256 * i, lb = e >> 6, kc = e & 63;
    const int bb = b0 + 64 * sl + lb;
    tile[lb][kc] = (bb < B && 64 * kb + kc < I) ? x[((size_t)t * B + bb) * I + 64 * kb + kc] : 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int o = threadIdx.x + 256 * i;  // 16-byte piece (chain, k8 local, kk, n): 2 x 8 x 2 x 32
    const int n = o & 31, kk = (o >> 5) & 1, k8 = (o >> 6) & 7, c = o >> 9;
    floatx4 v;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = tile[32 * c + n][8 * k8 + 2 * j + kk];
    float* const dst = xin + (((size_t)sl * (T + 1) + t + 1) * 2 + c) * H * 32 + (size_t)kb * 2048;
    *reinterpret_cast<floatx4*>(dst + (size_t)((k8 * 2 + kk) * 32 + n) * 4) = v;
  }
}

template <int HH, int CELL>
hipError_t launch_pp(int grid, const PersFwdArgs& a, hipStream_t s) {
  constexpr int NK8 = HH / 32;
  // the other chain's publication is completed half an operand half into a block (H = 512, group 8; cfg3 forward
  // recurrence by that group: 6 0.964 ms -- the acknowledgement is not there yet --, 7 0.902, 8 0.906, 9 0.910,
  // 10 0.911, 12 0.921), the fetch of its next input starts there as well (from group 10 or 12 on: 0.953)
  constexpr int GA = HH == 512 ? NK8 / 2 : NK8 / 2 + NK8 / 4;
  const void* fn = a.trace ? (const void*)pers_fwd_pp_kernel<HH, GA, NK8 / 2, true, CELL>
                           : (const void*)pers_fwd_pp_kernel<HH, GA, NK8 / 2, false, CELL>;
  void* params[] = {const_cast<PersFwdArgs*>(&a)};
  return launch_resident(fn, grid, params, 0, s);
}

}  // namespace

template <int CELL>
hipError_t launch_pp_h(int H, int grid, const PersFwdArgs& a, hipStream_t s) {
  if (H == 512) return launch_pp<512, CELL>(grid, a, s);
  if (H == 256) return launch_pp<256, CELL>(grid, a, s);
  if (H == 128) return launch_pp<128, CELL>(grid, a, s);
  return hipErrorInvalidValue;
}

hipError_t launch_fwd_pp(int cell, int H, int grid, const PersFwdArgs& a, hipStream_t s) {  // cell 0: LSTM, 1: GRU, 2: ReLU, 3: tanh
  if (cell == 1) return launch_pp_h<1>(H, grid, a, s);
  if (cell == 2) return launch_pp_h<2>(H, grid, a, s);
  if (cell == 3) return launch_pp_h<3>(H, grid, a, s);
  if (cell != 0) return hipErrorInvalidValue;
  if (H == 512) return launch_pp<512, 0>(grid, a, s);
  if (H == 256) return launch_pp<256, 0>(grid, a, s);
  if (H == 128) return launch_pp<128, 0>(grid, a, s);
  return hipErrorInvalidValue;
}

hipError_t launch_pack_state_pp(const float* h0, float* hx, int L, int T, int B, int H, int b0, int nsl, hipStream_t s) {
  const long n = (long)nsl * L * 64 * H;
  hipLaunchKernelGGL(pack_state_pp_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, h0, hx, L, T, B, H, b0, nsl);
  return hipGetLastError();
}

hipError_t launch_pack_x_pp(const float* x, float* xin, int T, int B, int I, int H, int b0, int nsl, hipStream_t s) {
  hipLaunchKernelGGL(pack_x_pp_kernel, dim3(H / 64, T, nsl), dim3(256), 0, s, x, xin, T, B, I, H, b0, nsl);
  return hipGetLastError();
}

}  // namespace lstm
