// Persistent forward recurrence of one LSTM layer with H = 2048 (the kernel is written for H = 1024 as well), the slice of 32 batch
// rows as two chains of 16 rows that take turns inside every wave: pers_fwdLpp_kernel.
//
// Why.  pers_fwdL_kernel runs a step as one dependent sequence: wait until every workgroup has published h_{t-1}, fetch
// it, multiply, reduce, gates, publish -- about a quarter of a step the matrix cores wait for the exchange (Section 4
// of arXiv 1604.01946 names the price of keeping the weights on chip: the workgroups have to meet after every step).
// The recurrences of different batch rows are independent, so here a chain's exchange (store, acknowledgement,
// counter, propagation, the fetch of the operand) runs while the wave multiplies for the other chain, as in the
// alternating kernels for H <= 512.
//
// Tile.  v_mfma_f32_16x16x4_f32: N = the chain's 16 batch rows, M = 16 of the workgroup's 32 weight rows (two tiles:
// tile m holds units 4 m ... 4 m + 3 with their four gates, row 4 u' + gate, so that a lane of the result holds the
// four gates of one (unit, batch row)), K = H split over the four waves.  The weights of a wave (2 tiles x H/16 groups
// of four k) live in registers up to 64 groups and in LDS beyond (H = 2048: half and half), read from LDS once per
// chain-step, two groups x two tiles per 16-byte read.
//
// Exchange layout of one (step, chain) slot, H x 16 floats: element (k, n) at (k/16)*256 + (((k%16)/4)*16 + n)*4 + k%4.
// A lane (kq, n) of the B operand fetches the four values k = 16 Q + 4 kq + j, j = 0..3, of a 16-k block Q with one
// 16-byte load (1 KB per wave and request), and matrix instruction j of the block takes value j: its four k are
// {16 Q + 4 kq + j}.  A workgroup's 8 units are 512 contiguous bytes of the slot, written by its two finalising waves
// with one 4-byte store per lane (a wave covers 256 contiguous bytes).
//
// Roles.  Waves 2 c and 2 c + 1 finalise chain c (tile m = wave % 2): K-split sums from LDS, gates, cell update,
// publication of h_t, reserve.  Counters: one per (step, chain), 16 lines, two arrivals per workgroup.
//
// Order in a wave: block(0, t), block(1, t), block(0, t + 1) ...; a block = the chain-step's matrix instructions.
// The point-wise stage of a chain sits at the start of the other chain's block; that block completes the
// publication (acknowledgement + counter) at request GA, looks at the counter at request QP (by then every workgroup
// has usually arrived; if not, the wave polls there) and requests all operands of the published chain's next block
// during its remaining requests.
#include "../../include/lstm.h"
#include "persistent_dev.h"

namespace lstm {
namespace {

// CELL as in pers_fwdL_kernel (0 LSTM, 1 GRU, 2 / 3 single gate with ReLU / tanh): only recurrent weights live here, so
// the GRU's third row of a unit (W_n x + b_n) has none and arrives with the batched projection P [T*B][3H], its fourth
// (R_n h) has no projection; `c0` carries h0 for the GRU; reserve layouts as in that kernel.
template <int HH, int GA_, int QP_, int RG_, bool TRACE, int CELL = 0>
__global__ __launch_bounds__(256) void pers_fwdLpp_kernel(const PersFwdLArgs a) {
  constexpr int NGT = CELL == 0 ? 4 : (CELL == 1 ? 3 : 1), GP = NGT * HH;  // gate blocks and rows of R, bias, P
  constexpr int H = HH, G = 4 * H, NS = H / 8;
  constexpr int KQ = H / 4;                 // k per wave
  constexpr int NQ = KQ / 16;               // operand requests per wave and chain-step
  constexpr int NGR = KQ / 4;               // groups (one matrix instruction per tile) per wave and chain-step
  constexpr int RG = NGR < RG_ ? NGR : RG_;  // groups whose weights live in registers (a multiple of four)
  constexpr int LG = NGR - RG;              // groups whose weights live in LDS
  constexpr int RQ = RG / 4;                // requests served from registers
  constexpr int GA = GA_, QP = QP_;
  constexpr int NEED = NS / 8;              // arrivals per counter line: two per workgroup, 16 lines
  static_assert(GA >= 1 && GA < QP && QP >= 4 && QP < NQ && NQ % 4 == 0, "schedule");
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* const part = smem;         // [2 chains][4 waves][2 tiles][64 lanes][4]
  float* const wl = smem + 4096;    // [4 waves][LG / 2][64 lanes][4]: (group, tile) = (2 p, 0), (2 p, 1), (2 p + 1, 0), (2 p + 1, 1)

  const int sl = blockIdx.x / NS, s = blockIdx.x % NS, u0 = 8 * s;
  const int T = a.T, B = a.B, b0 = a.b0 + 32 * sl;
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const size_t TB = (size_t)T * B;
  float* const hx = a.hx + (size_t)sl * (T + 1) * H * 32;
  int* const flags = a.flags + (size_t)sl * (T + 1) * 2 * 16 * kFlagStride;
  auto slot = [&](int st, int c) { return hx + ((size_t)st * 2 + c) * H * 16; };
  auto flag = [&](int st, int c) { return flags + ((size_t)st * 2 + c) * 16 * kFlagStride; };
  // the waves read a slot in orders rotated against each other, in steps of four requests (the address of a request is
  // then a scalar base + the lane's fixed offset + an immediate)
  const int rot = 4 * (((int)(blockIdx.x >> 3) + w) & (NQ / 4 - 1));

  // ---- weights.  Processed request p covers block Q(p) = p % 4 + 4 * ((p / 4 + rot / 4) % (NQ / 4)); group 4 p + j,
  //      tile m: lane (kq = lane / 16, row = lane % 16) holds R[gate row % 4 of unit u0 + 4 m + row / 4][w KQ + 16 Q + 4 kq + j]
  float wreg[RG][2];
  {
    const int kq = lane >> 4, row = lane & 15;
#pragma unroll
    for (int p = 0; p < NQ; ++p) {
      const int Q = (p & 3) + 4 * (((p >> 2) + (rot >> 2)) & (NQ / 4 - 1));
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = 4 * p + j;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
          const int grp = row & 3, gate = CELL >= 2 ? 0 : ((CELL == 1 && grp == 3) ? 2 : grp);
          const bool live = CELL == 0 || (CELL == 1 ? grp != 2 : grp == 0);
          const float v = live ? a.R[((size_t)gate * H + u0 + 4 * m + (row >> 2)) * H + (size_t)w * KQ + 16 * Q + 4 * kq + j] : 0.f;
          if (i < RG)
            wreg[i < RG ? i : 0][m] = v;
          else
            wl[(((size_t)w * (LG / 2) + ((i - RG) >> 1)) * 64 + lane) * 4 + ((i - RG) & 1) * 2 + m] = v;
        }
      }
    }
  }

  // ---- the cell this lane finalises: chain cf = w / 2, tile mf = w % 2, unit u0 + 4 mf + lane / 16, batch row lane % 16
  const int cf = w >> 1, mf = w & 1;
  const int q4 = lane >> 4, n = lane & 15;
  const int unit = u0 + 4 * mf + q4;
  const int bb = b0 + 16 * cf + n;
  const bool valid = bb < B;
  const int bc = valid ? bb : B - 1;  // rows past the batch read the last row (their results are not stored)
  float c_state = (CELL <= 1 && valid && a.c0) ? a.c0[(size_t)bb * H + unit] : 0.f;  // c_{t-1} (LSTM), h_{t-1} (GRU)
  float bias[4], pin[4];  // pin: the input product of the chain's next point-wise stage
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    bias[g] = g < NGT ? a.bias[g * H + unit] : 0.f;
    pin[g] = g < NGT ? a.P[(size_t)bc * GP + g * H + unit] : 0.f;
  }
  // Addresses of the point-wise stage's requests: a scalar base per array and step (scalar arithmetic costs a wave that
  // runs matrix instructions back to back nothing) plus one of two per-lane 32-bit offsets.
  const unsigned off_g = (unsigned)(((size_t)bc * G + unit) * 4), off_h = (unsigned)(((size_t)bc * H + unit) * 4);
  const unsigned off_p = (unsigned)(((size_t)bc * GP + unit) * 4);
  const char* const p_base = reinterpret_cast<const char*>(a.P);
  char* const res_gates = reinterpret_cast<char*>(CELL == 0 ? a.res : a.res + TB * H);  // the four saved arrays (LSTM, GRU)
  char* const res_c = reinterpret_cast<char*>(a.res + TB * 4 * H);                       // LSTM only
  char* const res_h = reinterpret_cast<char*>(CELL == 0 ? a.res + TB * 5 * H : a.res);
  char* const y_base = reinterpret_cast<char*>(a.y);

  PpWaiter<16> wt{a.watchdog, a.spin_limit, false};
  const PpTracer trc{(TRACE && a.trace && (int)blockIdx.x == a.trace_block) ? a.trace : nullptr, T};
  auto mark = [&](const int c, const int t, const int sl2) {
    if constexpr (TRACE) trc.mark(c, t, sl2);
  };
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // once: drop whatever earlier launches left in L1/L2
  __syncthreads();                                    // LDS weights are in place

  int rv = rot >> 2;
  unsigned lo = lane * 16;
  auto fresh_lo = [&]() {
    lo = lane * 16;
    asm volatile("" : "+v"(lo));
  };
  auto ldx = [&](const float* src, int p) {  // src: the slot (wave-uniform); processed request p of this wave's K quarter
    const char* const sb = reinterpret_cast<const char*>(src) + ((size_t)w * NQ + 4 * (((p >> 2) + rv) & (NQ / 4 - 1))) * 1024;
    return *reinterpret_cast<const floatx4*>(sb + lo + (p & 3) * 1024);
  };

  floatx4 op[2][NQ];     // B operands of a chain's block: requested during the other chain's block
  int seen_next = 0;

  // ---- point-wise stage of chain cf, step t (the two finalising waves of the chain; after the barrier that follows
  //      the chain's block): sums, gates, h_t out, next step's input product requested, reserve and outputs
  float probe = 0.f, pw[6];
  auto post = [&](const int t) {
    const float* const src = part + ((size_t)cf * 4 * 2 + mf) * 256 + lane * 4;
    const floatx4 s0 = *reinterpret_cast<const floatx4*>(src), s1 = *reinterpret_cast<const floatx4*>(src + 512);
    const floatx4 s2 = *reinterpret_cast<const floatx4*>(src + 1024), s3 = *reinterpret_cast<const floatx4*>(src + 1536);
    float sg[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) sg[g] = ((s0[g] + s1[g]) + (s2[g] + s3[g])) + pin[g] + bias[g];
    float gi, gf, go, gc, cn, hn;
    if (CELL == 0) {
      gi = sigmoidf_dev(sg[0]), gf = sigmoidf_dev(sg[1]), go = sigmoidf_dev(sg[2]), gc = tanhf_dev(sg[3]);
      cn = gf * c_state + gi * gc;
      hn = go * tanhf_dev(cn);
      c_state = cn;
    } else if (CELL == 1) {  // sg: r, z pre-activations; W_n x + b_n (from P); R_n h.  Saved: r, z, n, R_n h
      gi = sigmoidf_dev(sg[0]), gf = sigmoidf_dev(sg[1]);
      go = tanhf_dev(sg[2] + gi * sg[3]);
      gc = sg[3];
      hn = (1.f - gf) * go + gf * c_state;
      cn = 0.f;
      c_state = hn;
    } else {
      gi = gf = go = gc = cn = 0.f;
      hn = CELL == 3 ? tanhf_dev(sg[0]) : fmaxf(sg[0], 0.f);
    }
    __hip_atomic_store(slot(t + 1, cf) + (size_t)s * 128 + (mf * 16 + n) * 4 + q4, valid ? hn : 0.f, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    // A load requested behind the publication (a word that is in the L2 cache anyway): requests retire in issue order,
    // so once it has arrived the publication is acknowledged.
    probe = __builtin_nontemporal_load(a.bias + unit);
    pw[0] = gi; pw[1] = gf; pw[2] = go; pw[3] = gc; pw[4] = cn; pw[5] = hn;
  };
  // ---- its second part: the reserve and the outputs (nobody reads them before the kernel ends)
  auto post_b = [&](const int t) {
    const float gi = pw[0], gf = pw[1], go = pw[2], gc = pw[3], cn = pw[4], hn = pw[5];
    if (valid) {
      unsigned og = off_g, oh = off_h;
      asm volatile("" : "+v"(og), "+v"(oh));  // (32-bit offsets met anew here: they become the offset operands of the stores)
      if (CELL <= 1) {
        char* const rg = res_gates + (size_t)t * B * G * 4;
        *reinterpret_cast<float*>(rg + og) = gi;
        *reinterpret_cast<float*>(rg + (size_t)H * 4 + og) = gf;
        *reinterpret_cast<float*>(rg + (size_t)2 * H * 4 + og) = go;
        *reinterpret_cast<float*>(rg + (size_t)3 * H * 4 + og) = gc;
      }
      const size_t eb = (size_t)t * B * H * 4;
      if (CELL == 0) *reinterpret_cast<float*>(res_c + eb + oh) = cn;
      *reinterpret_cast<float*>(res_h + eb + oh) = hn;
      if (a.y) *reinterpret_cast<float*>(y_base + eb + oh) = hn;
      if (t == T - 1) {
        if (a.hT) a.hT[(size_t)bb * H + unit] = hn;
        if (CELL == 0 && a.cT) a.cT[(size_t)bb * H + unit] = cn;
      }
    }
  };

  // ---- one block: the matrix instructions of chain c's step t.  have_prev: the other chain has a point-wise stage
  //      pending (its block was the one before this one).
  auto block = [&](const int c, const int t, const bool have_prev) {
    const int o = 1 - c;
    const int tp = c == 0 ? t - 1 : t;   // step of the pending point-wise stage (chain o)
    const int tn = c == 0 ? t : t + 1;   // the next block is (o, tn)
    const bool has_next = tn < T;
    hide(rv);
    mark(c, t, 0);
    floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    // (the stores to the reserve right behind the stage, ahead of the operand requests of this block: requests retire
    // in issue order, and stores issued behind those requests would be waited for with them)
    if (have_prev && cf == o) {
      post(tp);
      post_b(tp);
    }
    floatx4 alw[LG > 0 ? LG / 2 : 1];
    auto ldw = [&](int p) {
      if (p >= RQ && p < NQ) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
          alw[2 * (p - RQ) + h] = *reinterpret_cast<const floatx4*>(wl + (((size_t)w * (LG / 2) + 2 * (p - RQ) + h) * 64 + lane) * 4);
      }
    };
    // operands of the next block; when there is none, this chain's own slot once more (valid memory, values unused)
    const float* const nsrc = has_next ? slot(tn, o) : slot(t, c);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int p = 0; p < NQ; ++p) {
      ldw(p + 1);
      if (p == QP - 3) seen_next = PpWaiter<16>::peek((has_next && tn > 0) ? flag(tn, o) : flag(t > 0 ? t : 1, c));
      if (p == QP) {
        mark(c, t, 1);
        PpWaiter<16>::land(seen_next);
        if (has_next && tn > 0) wt.wait(flag(tn, o), NEED, seen_next);
        mark(c, t, 2);
        fresh_lo();
      }
      if (p >= QP) {  // requests [lo2, hi2) of the next block, spread evenly over the requests QP .. NQ-1 of this one
        constexpr int span = NQ - QP;
        const int lo2 = ((p - QP) * NQ) / span, hi2 = ((p - QP + 1) * NQ) / span;
#pragma unroll
        for (int r = lo2; r < hi2; ++r) op[o][r] = ldx(nsrc, r);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int g = 4 * p + j;
        const float a0 = g < RG ? wreg[g < RG ? g : 0][0] : alw[g < RG ? 0 : (g - RG) >> 1][((g - RG) & 1) * 2 + 0];
        const float a1 = g < RG ? wreg[g < RG ? g : 0][1] : alw[g < RG ? 0 : (g - RG) >> 1][((g - RG) & 1) * 2 + 1];
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, op[c][p][j], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, op[c][p][j], acc1, 0, 0, 0);
      }
      if (p == GA) {
        // completion of the pending publication: the input product requested behind it has arrived, so the store
        // before it is acknowledged (requests retire in issue order)
        if (have_prev && cf == o) {
          asm volatile("" : "+v"(probe));
          if (lane == 0)
            __hip_atomic_fetch_add(flag(tp + 1, o) + (s & 15) * kFlagStride, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          // the input product of the chain's next point-wise stage, a whole step ahead of its use
          const size_t tq = tp + 1 < T ? tp + 1 : tp;
          unsigned og = off_p;
          asm volatile("" : "+v"(og));
          const char* const pb = p_base + tq * B * GP * 4;
#pragma unroll
          for (int g = 0; g < NGT; ++g) pin[g] = *reinterpret_cast<const float*>(pb + (size_t)g * H * 4 + og);
        }
        fresh_lo();
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    float* const mine = part + (((size_t)c * 4 + w) * 2) * 256 + lane * 4;
    *reinterpret_cast<floatx4*>(mine) = acc0;
    *reinterpret_cast<floatx4*>(mine + 256) = acc1;
    mark(c, t, 3);
    __syncthreads();
    mark(c, t, 4);
  };

  // ---- chain 0's first operand (slot 0 was written before the launch)
  fresh_lo();
#pragma unroll
  for (int p = 0; p < NQ; ++p) op[0][p] = ldx(slot(0, 0), p);
  for (int t = 0; t < T; ++t) {
    block(0, t, t > 0);
    block(1, t, true);
  }
  if (cf == 1) {
    post(T - 1);
    post_b(T - 1);
  }
}

// h0 [B][H] of one layer (zeros if null) -> slot 0 of both chains of every slice, in the layout above
__global__ void pack_stateLpp_kernel(const float* __restrict__ h0, float* __restrict__ hx, int T, int B, int H, int b0, int nsl) {
  const long cnt = (long)nsl * 32 * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < cnt; e += (long)gridDim.x * blockDim.x) {
    const int k = (int)(e % H), lb = (int)((e / H) % 32), sl = (int)(e / ((long)H * 32));
    const int bb = b0 + 32 * sl + lb, c = lb >> 4, n = lb & 15;
    hx[(size_t)sl * (T + 1) * H * 32 + (size_t)c * H * 16 + (size_t)(k >> 4) * 256 + ((((k & 15) >> 2) * 16 + n) << 2) + (k & 3)] =
        (h0 && bb < B) ? h0[(size_t)bb * H + k] : 0.f;
  }
}

template <int HH, int GA, int QP, int RG, int CELL>
hipError_t launch_fwdLpp_t(const PersFwdLArgs& a, hipStream_t s) {
  constexpr int NGR = HH / 16, LG = NGR > RG ? NGR - RG : 0;
  const size_t smem = (4096 + (size_t)4 * (LG / 2) * 64 * 4) * sizeof(float);
  const bool trace = a.trace != nullptr;
  const void* fn = trace ? (const void*)pers_fwdLpp_kernel<HH, GA, QP, RG, true, CELL> : (const void*)pers_fwdLpp_kernel<HH, GA, QP, RG, false, CELL>;
  static bool attr_set[2] = {false, false};
  if (hipError_t e = allow_dynamic_lds(fn, smem, attr_set[trace ? 1 : 0]); e != hipSuccess) return e;
  void* params[] = {const_cast<PersFwdLArgs*>(&a)};
  return launch_resident(fn, a.nsl * (HH / 8), params, (unsigned)smem, s);
}

}  // namespace

// Counter ints per (slice, step): two chains x 16 lines
size_t fwdLpp_flag_ints() { return (size_t)2 * 16 * kFlagStride; }

hipError_t launch_fwdLpp(int cell, int H, const PersFwdLArgs& a, hipStream_t s) {  // cell: 0 LSTM, 1 GRU, 2 ReLU, 3 tanh
  // Schedule, measured at B = 32, T = 50 (ms per launch): (GA, QP) = (14, 22) 3.60, (10, 24) 2.97, (8, 26) 2.14,
  // (4, 26) 1.97, (4, 28) 1.98, (2, 26) 1.97 -- the earlier a publication is completed and the later its counter is
  // looked at, the fewer polls get in the way of the arrivals they wait for; 64 groups of weights in registers (96:
  // 2.08, all 128: 2.24; the one-chain kernel: 2.40).  At H = 1024 a block is too short to cover the exchange (best
  // schedule 1.44 ms against 1.31 for the one-chain kernel at L = 4, B = 32): that size stays on pers_fwdL_kernel.
  if (H == 2048) {
    return cell == 0 ? launch_fwdLpp_t<2048, 4, 26, 64, 0>(a, s) : (cell == 1 ? launch_fwdLpp_t<2048, 4, 26, 64, 1>(a, s)
                     : (cell == 2 ? launch_fwdLpp_t<2048, 4, 26, 64, 2>(a, s) : launch_fwdLpp_t<2048, 4, 26, 64, 3>(a, s)));
  }
  return hipErrorInvalidValue;
}

hipError_t launch_pack_stateLpp(const float* h0, float* hx, int T, int B, int H, int b0, int nsl, hipStream_t s) {
  hipLaunchKernelGGL(pack_stateLpp_kernel, dim3((unsigned)((32L * nsl * H + 255) / 256)), dim3(256), 0, s, h0, hx, T, B, H, b0, nsl);
  return hipGetLastError();
}

}  // namespace lstm
