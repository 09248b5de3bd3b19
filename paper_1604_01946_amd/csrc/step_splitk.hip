// Split-K variant of the fused backward step kernel, for hidden sizes whose recurrent matrix cannot
// stay on chip (H >= 1024).
//
// At such sizes a step is bound by streaming R once from memory (4*4H*H bytes, Section 2.1's
// [4H x H] operand of arXiv 1604.01946) and by the matrix cores at about the same time.  In the
// backward step the contraction runs over K = 4H: with the hidden units alone dealt over the
// workgroups (step.hip), every workgroup re-reads the whole dA_{t+1} (B x 4H values), and that L2
// traffic, not R, becomes the limit.  Here a workgroup owns a (unit slice, K slice) tile instead:
// it streams its tile of the packed R^T, reads only its K slice of dA_{t+1}, and writes a partial
// sum.  The workgroup that finishes a unit slice last (an agent-scope counter per unit slice and
// step) adds the partial sums in fixed K-slice order -- no floating-point atomics, so results stay
// bit-wise repeatable -- and runs the fused point-wise gate-gradient update for that unit slice.
// K slices are dealt so that workgroups sharing a dA slice run on the same XCD.  (The forward step
// contracts over K = H only; there the same scheme measured slower than step.hip's kernel and is
// not used.)
#include "internal.h"
#include "knobs.h"

#include <stdlib.h>

namespace lstm {
namespace {

template <bool VEC>
__device__ __forceinline__ floatx4 ld4(const float* __restrict__ row, int k, int K, bool valid) {
  floatx4 v = {0.f, 0.f, 0.f, 0.f};
  if (VEC) {
    if (valid && k < K) v = *reinterpret_cast<const floatx4*>(row + k);
  } else {
    if (valid) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (k + e < K) v[e] = row[k + e];
    }
  }
  return v;
}

// Write-through (agent-scope) 16-byte store.  The data operand must not come straight out of an
// MFMA: inline assembly is opaque to the compiler's hazard handling, so an accumulator could be
// read before its last pass has been written.  The partial sums are therefore staged through LDS
// first (which also turns them into long contiguous runs).  For the same reason the statement ends in
// idle cycles: a store of more than 8 bytes still reads its data registers after it has issued, and
// the compiler, not knowing this is a store, may overwrite them with the very next instruction.
__device__ __forceinline__ void xstore4(float* p, floatx4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 3" ::"v"(p), "v"(v) : "memory");
}

// True in exactly one workgroup per (row slice, launch): the one whose partial arrived last.
// `s_last`: one int of LDS that no thread touches otherwise from here on.
__device__ __forceinline__ bool last_arrival(int* counter, int expected, int* s_last) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's write-through partial stores are acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_last = (old == expected - 1);
  }
  __syncthreads();
  // The partial sums were written through to memory before each arrival was counted, and this
  // workgroup has not touched those lines since the launch began (a launch starts with clean
  // caches), so its first reads fetch the published values: no cache invalidate is needed.
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  return *s_last != 0;
}

// ------------------------------------------------------------------ pack (once per pass)
// k-steps (of 16) of a K slice that one wave takes: the four waves of a workgroup split the slice
__host__ __device__ inline int sk_per_wave(int per) { return (per + 3) / 4; }

// backward: [unit slice of 64][K slice][wave][k-step of the wave][m-tile of 16 units][lane][4] over R^T
// (row = hidden unit, K = 4H); zero where the slice, the wave's share or K runs out.
__global__ void pack_bwd_sk_kernel(const float* __restrict__ R, floatx4* __restrict__ Rp, int H, int KS, int per,
                                   long per_layer) {
  const int K = 4 * H, NUS = (H + 63) / 64, perw = sk_per_wave(per);
  const long total = (long)NUS * KS * 4 * perw * 4 * 64;
  const float* Rl = R + (size_t)blockIdx.y * 4 * H * H;
  floatx4* out = Rp + (size_t)blockIdx.y * per_layer;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int lane = (int)(i & 63);
    long r = i >> 6;
    const int mt = (int)(r & 3); r >>= 2;
    const int ksl = (int)(r % perw); r /= perw;
    const int w = (int)(r & 3); r >>= 2;
    const int ks = (int)(r % KS);
    const int us = (int)(r / KS);
    const int q = lane >> 4, n = lane & 15;
    const int unit = us * 64 + 16 * mt + n;
    const int kstep = w * perw + ksl;  // within the K slice
    const int k = (ks * per + kstep) * 16 + 4 * q;
    floatx4 v = {0.f, 0.f, 0.f, 0.f};
    if (unit < H && kstep < per) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (k + e < K) v[e] = Rl[(size_t)(k + e) * H + unit];
    }
    out[i] = v;
  }
}

// ------------------------------------------------------------------ backward
// grid.x = NUS * KS (K slice fastest), grid.y = batch tiles.  A workgroup owns 64 hidden units (four m-tiles of 16)
// and one K slice; its four waves split the slice, so each wave reads only its quarter of the dA slice (the B operand)
// and every element of the packed R^T tile exactly once, and the four partial sums meet in LDS.
// TWO: short load chunks and at most 256 registers, so that two waves share a SIMD (64 batch rows in one tile: the
// step is bound by the matrix cores, and one wave per SIMD leaves them waiting on its own loads).
template <int NT, bool VEC, bool TWO = false>
__global__ __launch_bounds__(256, TWO ? 2 : 1) void step_bwd_sk_kernel(const StepBwdArgs a, const SplitK sk) {
  constexpr int MT = 4;
  __shared__ __attribute__((aligned(16))) float part[4][MT * NT * 4][64];
  const int H = a.H, B = a.B, K = 4 * a.H, KS = sk.KS, per = sk.per, perw = sk_per_wave(per);
  const int us = blockIdx.x / KS, ks = blockIdx.x % KS;
  const int u0 = us * 64, b0 = blockIdx.y * 16 * NT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, n = lane & 15;
  const int NUS = gridDim.x / KS;
  // partial sums: [batch tile][K slice][batch row in tile][H]
  float* const pbase = sk.partial + ((size_t)blockIdx.y * KS) * (16 * NT) * H;

  floatx4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[mt][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  if (a.dA_next) {
    const floatx4* ap = reinterpret_cast<const floatx4*>(a.RTp) + ((size_t)((us * KS + ks) * 4 + wave) * perw) * MT * 64 + lane;
    const float* brow[NT];
    bool bvalid[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int bb = b0 + 16 * j + n;
      bvalid[j] = bb < B;
      brow[j] = a.dA_next + (long)(bvalid[j] ? bb : 0) * K;
    }
    // Chunks of U k-steps, double-buffered: the loads of chunk c+1 are in flight while chunk c feeds the MFMAs.
    constexpr int U = TWO ? 2 : 4;
    const int klim = min(K, (ks + 1) * per * 16);
    const int mine = max(0, min(perw, per - wave * perw));  // k-steps of this wave inside the slice
    floatx4 av[2][U][MT], bv[2][U][NT];
    auto load_chunk = [&](int c, floatx4 (&ava)[U][MT], floatx4 (&bva)[U][NT]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int ksl = c * U + u;
        const bool in = ksl < mine;
        const int k = (ks * per + wave * perw + ksl) * 16 + 4 * q;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) ava[u][mt] = in ? ap[(size_t)(ksl * MT + mt) * 64] : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NT; ++j) bva[u][j] = ld4<VEC>(brow[j], k, klim, bvalid[j] && in);
      }
    };
    auto mma_chunk = [&](const floatx4 (&ava)[U][MT], const floatx4 (&bva)[U][NT]) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < NT; ++j)
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(ava[u][mt][e], bva[u][j][e], acc[mt][j], 0, 0, 0);
    };
    const int nch = (perw + U - 1) / U;
    load_chunk(0, av[0], bv[0]);
    for (int c = 0; c < nch; c += 2) {
      load_chunk(c + 1, av[1], bv[1]);
      __builtin_amdgcn_sched_barrier(0);
      mma_chunk(av[0], bv[0]);
      __builtin_amdgcn_sched_barrier(0);
      load_chunk(c + 2, av[0], bv[0]);
      __builtin_amdgcn_sched_barrier(0);
      if (c + 1 < nch) mma_chunk(av[1], bv[1]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // The waves' partial sums meet in LDS.  D layout: register r of lane (q, n) in tile (mt, j) is
  // (unit u0 + 16*mt + 4q + r, batch 16j + n); H % 64 == 0 here.
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) part[wave][(mt * NT + j) * 4 + r][lane] = acc[mt][j][r];
  __syncthreads();
  floatx4 sum[NT];  // wave w adds up m-tile w
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = (wave * NT + j) * 4 + r;
      sum[j][r] = (part[0][row][lane] + part[1][row][lane]) + (part[2][row][lane] + part[3][row][lane]);
    }
  __syncthreads();
  // Staged as [batch row][64 units]: 256 contiguous bytes per batch row (the staging area reuses `part`).
  float* const stage = &part[0][0][0];
#pragma unroll
  for (int j = 0; j < NT; ++j) *reinterpret_cast<floatx4*>(stage + (16 * j + n) * 64 + 16 * wave + 4 * q) = sum[j];
  __syncthreads();
  for (int idx = threadIdx.x; idx < 16 * NT * 16; idx += 256) {
    const int lb = idx >> 4, c4 = idx & 15;
    xstore4(pbase + ((size_t)ks * (16 * NT) + lb) * H + u0 + 4 * c4, *reinterpret_cast<const floatx4*>(stage + idx * 4));
  }

  // (the flag lives in the last quarter of `part`, past the staging area)
  if (!last_arrival(sk.counters + (size_t)blockIdx.y * NUS + us, KS, reinterpret_cast<int*>(&part[3][0][0]))) return;

  // ---- fix-up: sum the K slices in order, then the point-wise gate gradients of this unit slice
  for (int idx = threadIdx.x; idx < 16 * 16 * NT; idx += 256) {
    const int u4 = idx & 15, lb = idx >> 4;
    const int unit = u0 + 4 * u4, bb = b0 + lb;
    if (bb >= B) continue;
    floatx4 dh = *reinterpret_cast<const floatx4*>(pbase + (size_t)lb * H + unit);
    for (int k2 = 1; k2 < KS; ++k2) dh += *reinterpret_cast<const floatx4*>(pbase + ((size_t)k2 * (16 * NT) + lb) * H + unit);
    const long e = (long)bb * H + unit, g0 = (long)bb * 4 * H + unit;
    if (a.dh_extra) dh += *reinterpret_cast<const floatx4*>(a.dh_extra + e);
    if (!a.pointwise) {
      *reinterpret_cast<floatx4*>(a.dh_out + e) = dh;
      continue;
    }
    dh += *reinterpret_cast<const floatx4*>(a.dout + e);
    const floatx4 gi = *reinterpret_cast<const floatx4*>(a.gates + g0);
    const floatx4 gf = *reinterpret_cast<const floatx4*>(a.gates + g0 + H);
    const floatx4 go = *reinterpret_cast<const floatx4*>(a.gates + g0 + 2L * H);
    const floatx4 gg = *reinterpret_cast<const floatx4*>(a.gates + g0 + 3L * H);
    const floatx4 ct = *reinterpret_cast<const floatx4*>(a.c_t + e);
    floatx4 cp = {0.f, 0.f, 0.f, 0.f}, dci = {0.f, 0.f, 0.f, 0.f};
    if (a.c_prev) cp = *reinterpret_cast<const floatx4*>(a.c_prev + e);
    if (a.dc_in) dci = *reinterpret_cast<const floatx4*>(a.dc_in + e);
    floatx4 o0, o1, o2, o3, dco;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float tc = tanhf_dev(ct[r]);
      const float dc = dci[r] + dh[r] * go[r] * (1.f - tc * tc);
      o0[r] = dc * gg[r] * gi[r] * (1.f - gi[r]);
      o1[r] = dc * cp[r] * gf[r] * (1.f - gf[r]);
      o2[r] = dh[r] * tc * go[r] * (1.f - go[r]);
      o3[r] = dc * gi[r] * (1.f - gg[r] * gg[r]);
      dco[r] = dc * gf[r];
    }
    *reinterpret_cast<floatx4*>(a.dA + g0) = o0;
    *reinterpret_cast<floatx4*>(a.dA + g0 + H) = o1;
    *reinterpret_cast<floatx4*>(a.dA + g0 + 2L * H) = o2;
    *reinterpret_cast<floatx4*>(a.dA + g0 + 3L * H) = o3;
    *reinterpret_cast<floatx4*>(a.dc_out + e) = dco;
  }
}

inline int batch_tiles_y(int B) { return B <= 64 ? 1 : (B + 63) / 64; }
inline int tile_nt(int B) { return B <= 16 ? 1 : (B <= 32 ? 2 : 4); }
inline int pow2_floor(int v) {
  int p = 1;
  while (2 * p <= v) p *= 2;
  return p;
}

}  // namespace

// Split-K is used when H is large and a multiple of 64 (the fix-up then needs no unit guards).
bool splitk_supported(int H) {
  const int min_h = knobs().splitk_min_h > 0 ? knobs().splitk_min_h : 1024;  // tests lower the threshold to reach these kernels with small shapes
  return H >= min_h && (H % 64) == 0;
}

// K slices: enough to put about 256 workgroups in flight, at most 8 (a power of two so that the K
// slice of a workgroup follows from the XCD it is dealt to).
int splitk_bwd_slices(int H, int B) {
  const int nus = (H + 63) / 64 * batch_tiles_y(B);
  int ks = pow2_floor(nus >= 256 ? 1 : 256 / nus);
  return ks > 8 ? 8 : ks;
}
int splitk_bwd_per(int H, int B) { const int nks = (4 * H + 15) / 16, ks = splitk_bwd_slices(H, B); return (nks + ks - 1) / ks; }

size_t splitk_pack_floats(int H) {
  // upper bound for any slice count: each of up to 8 K slices pads to whole k-steps and then to four equal shares for the waves
  return (size_t)((H + 63) / 64) * 4 * (((4 * H + 15) / 16) + 32) * 256;
}
size_t splitk_partial_floats(int H, int B) { return (size_t)8 * batch_tiles_y(B) * 64 * H; }
size_t splitk_counter_ints(int H, int B) { return (size_t)((H + 63) / 64) * batch_tiles_y(B); }

hipError_t launch_pack_bwd_sk(const float* R, float* RTp, int L, int H, int B, size_t per_layer_floats, hipStream_t s) {
  hipLaunchKernelGGL(pack_bwd_sk_kernel, dim3(512, L), dim3(256), 0, s, R, reinterpret_cast<floatx4*>(RTp), H,
                     splitk_bwd_slices(H, B), splitk_bwd_per(H, B), (long)(per_layer_floats / 4));
  return hipGetLastError();
}

hipError_t launch_step_bwd_sk(const StepBwdArgs& a, float* partial, int* counters, hipStream_t s) {
  SplitK sk{partial, counters, splitk_bwd_slices(a.H, a.B), splitk_bwd_per(a.H, a.B)};
  if (a.dA_next) prof_flops(2.0 * a.B * 4.0 * a.H * a.H, "step_bwd_sk_kernel");
  const dim3 grid(((a.H + 63) / 64) * sk.KS, batch_tiles_y(a.B));
  const bool vec = (a.dA_next == nullptr) || (reinterpret_cast<uintptr_t>(a.dA_next) & 15u) == 0;
  const int nt = tile_nt(a.B);
#define LSTM_SK_CASE(NT_)                                                                              \
  if (nt == NT_) {                                                                                     \
    if (vec) hipLaunchKernelGGL((step_bwd_sk_kernel<NT_, true>), grid, dim3(256), 0, s, a, sk);        \
    else hipLaunchKernelGGL((step_bwd_sk_kernel<NT_, false>), grid, dim3(256), 0, s, a, sk);           \
  }
  if (nt == 4 && grid.y == 1) {
    if (vec) hipLaunchKernelGGL((step_bwd_sk_kernel<4, true, true>), grid, dim3(256), 0, s, a, sk);
    else hipLaunchKernelGGL((step_bwd_sk_kernel<4, false, true>), grid, dim3(256), 0, s, a, sk);
    return hipGetLastError();
  }
  LSTM_SK_CASE(1) LSTM_SK_CASE(2) LSTM_SK_CASE(4)
#undef LSTM_SK_CASE
  return hipGetLastError();
}

}  // namespace lstm
