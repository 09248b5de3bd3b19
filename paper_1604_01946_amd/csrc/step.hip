// Fused per-step kernels: recurrent GEMM over the four stacked gates with the point-wise
// cell update as its epilogue (forward), and the mirrored backward step.
//
// Section 2.1 of arXiv 1604.01946 stacks the four gate matrices that share an input into
// one [4H x H] operand; Section 2.2.2 fuses all point-wise work of a cell into one kernel.
// Here both live in one kernel: a workgroup owns a slice of hidden units *with all four
// gate rows of that slice*, so the gate pre-activations never leave the chip.
//
// Mapping (forward): workgroup = 8 hidden units x (16*NT) batch rows; the 32 weight rows
// (unit-major, gate-minor) are the M side of v_mfma_f32_16x16x4_f32, the batch is the N
// side, and K = H is split over the 4 waves (wave w takes the k-steps w, w+4, ...).  Both
// operands are read straight from memory as 16-byte runs along K -- lane (q = lane/16,
// n = lane%16) fetches k = 16*ks + 4q .. +3 of row n, and element e of that fetch feeds the
// e-th MFMA of the k-step -- so no LDS staging is needed.  The four partial sums meet in
// LDS; in the D layout a lane already holds all four gates of one (unit, batch) cell.
// Backward: workgroup = 16 hidden units x (16*NT) batch rows, K = 4H over the transposed
// recurrent matrix; the epilogue is the point-wise gate-gradient computation.
#include "internal.h"

namespace lstm {
namespace {

template <bool VEC>
__device__ __forceinline__ floatx4 load4(const float* __restrict__ row, int k, int K, bool valid) {
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

template <int NT, bool VEC>
__global__ __launch_bounds__(256) void step_fwd_kernel(const StepFwdArgs a) {
  __shared__ float part[4][2 * NT * 4][64];
  const int H = a.H, B = a.B;
  const int u0 = blockIdx.x * 8, b0 = blockIdx.y * 16 * NT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, n = lane & 15;

  floatx4 acc[2][NT];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[mt][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  if (a.h_prev) {
    const float* arow[2];
    bool avalid[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const int unit = u0 + 4 * mt + (n >> 2), gate = n & 3;
      avalid[mt] = unit < H;
      arow[mt] = a.R + ((long)gate * H + (avalid[mt] ? unit : 0)) * H;
    }
    const float* brow[NT];
    bool bvalid[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int bb = b0 + 16 * j + n;
      bvalid[j] = bb < B;
      brow[j] = a.h_prev + (long)(bvalid[j] ? bb : 0) * H;
    }
    // U k-steps per trip: all of their loads are issued before the first MFMA so that enough bytes
    // are in flight to stream the weights at memory speed (k-steps past the end load zeros)
    constexpr int U = (NT == 4) ? 4 : 8;
    for (int ks = wave; ks * 16 < H; ks += 4 * U) {
      floatx4 av[U][2], bv[U][NT];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = (ks + 4 * u) * 16 + 4 * q;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) av[u][mt] = load4<VEC>(arow[mt], k, H, avalid[mt]);
#pragma unroll
        for (int j = 0; j < NT; ++j) bv[u][j] = load4<VEC>(brow[j], k, H, bvalid[j]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int j = 0; j < NT; ++j)
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][mt][e], bv[u][j][e], acc[mt][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) part[wave][(mt * NT + j) * 4 + r][lane] = acc[mt][j][r];
  __syncthreads();

  // D layout: register r of lane (q, n) is row 4q + r = (unit_local q, gate r), column n (batch).
  for (int p = wave; p < 2 * NT; p += 4) {
    const int mt = p / NT, j = p % NT;
    const int unit = u0 + 4 * mt + q, bb = b0 + 16 * j + n;
    float s[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
      s[r] = (part[0][p * 4 + r][lane] + part[1][p * 4 + r][lane]) + (part[2][p * 4 + r][lane] + part[3][p * 4 + r][lane]);
    if (unit < H && bb < B) {
      const long g0 = (long)bb * 4 * H + unit, e = (long)bb * H + unit;
#pragma unroll
      for (int r = 0; r < 4; ++r) s[r] += a.P[g0 + (long)r * H] + a.bias[r * H + unit];
      const float ig = sigmoidf_dev(s[0]), fg = sigmoidf_dev(s[1]), og = sigmoidf_dev(s[2]), gg = tanhf(s[3]);
      const float cp = a.c_prev ? a.c_prev[e] : 0.f;
      const float c = fg * cp + ig * gg;
      const float h = og * tanhf(c);
      a.gates_out[g0] = ig; a.gates_out[g0 + H] = fg; a.gates_out[g0 + 2L * H] = og; a.gates_out[g0 + 3L * H] = gg;
      a.c_out[e] = c; a.h_out[e] = h;
      if (a.h_out2) a.h_out2[e] = h;
      if (a.c_out2) a.c_out2[e] = c;
    }
  }
}

template <int NT, bool VEC>
__global__ __launch_bounds__(256) void step_bwd_kernel(const StepBwdArgs a) {
  __shared__ float part[4][NT * 4][64];
  const int H = a.H, B = a.B, K = 4 * a.H;
  // upw = 16 fills the MFMA tile; upw = 8 (rows 8..15 idle) doubles the number of workgroups when
  // the grid would otherwise leave CUs without work (the step is bound by streaming R, not by MFMA)
  const int upw = a.units_per_wg;
  const int u0 = blockIdx.x * upw, b0 = blockIdx.y * 16 * NT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, n = lane & 15;

  floatx4 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};

  if (a.dA_next) {
    const bool avalid = n < upw && (u0 + n) < H;
    const float* arow = a.RT + (long)(avalid ? u0 + n : 0) * K;
    const float* brow[NT];
    bool bvalid[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int bb = b0 + 16 * j + n;
      bvalid[j] = bb < B;
      brow[j] = a.dA_next + (long)(bvalid[j] ? bb : 0) * K;
    }
    constexpr int U = (NT == 4) ? 4 : 8;
    for (int ks = wave; ks * 16 < K; ks += 4 * U) {
      floatx4 av[U], bv[U][NT];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = (ks + 4 * u) * 16 + 4 * q;
        av[u] = load4<VEC>(arow, k, K, avalid);
#pragma unroll
        for (int j = 0; j < NT; ++j) bv[u][j] = load4<VEC>(brow[j], k, K, bvalid[j]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int j = 0; j < NT; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][e], bv[u][j][e], acc[j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) part[wave][j * 4 + r][lane] = acc[j][r];
  __syncthreads();

  // D layout: register r of lane (q, n) is row 4q + r (hidden unit u0 + 4q + r), column n (batch).
  for (int j = wave; j < NT; j += 4) {
    const int bb = b0 + 16 * j + n;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int unit = u0 + 4 * q + r;
      if (4 * q + r >= upw || unit >= H || bb >= B) continue;
      const long e = (long)bb * H + unit, g0 = (long)bb * 4 * H + unit;
      float dh = (part[0][j * 4 + r][lane] + part[1][j * 4 + r][lane]) + (part[2][j * 4 + r][lane] + part[3][j * 4 + r][lane]);
      if (a.dh_extra) dh += a.dh_extra[e];
      if (!a.pointwise) {
        a.dh_out[e] = dh;
        continue;
      }
      dh += a.dout[e];
      const float ig = a.gates[g0], fg = a.gates[g0 + H], og = a.gates[g0 + 2L * H], gg = a.gates[g0 + 3L * H];
      const float tc = tanhf(a.c_t[e]);
      const float dc = (a.dc_in ? a.dc_in[e] : 0.f) + dh * og * (1.f - tc * tc);
      const float cp = a.c_prev ? a.c_prev[e] : 0.f;
      a.dA[g0] = dc * gg * ig * (1.f - ig);
      a.dA[g0 + H] = dc * cp * fg * (1.f - fg);
      a.dA[g0 + 2L * H] = dh * tc * og * (1.f - og);
      a.dA[g0 + 3L * H] = dc * ig * (1.f - gg * gg);
      a.dc_out[e] = dc * fg;
    }
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <bool VEC>
hipError_t launch_fwd_nt(const StepFwdArgs& a, hipStream_t s) {
  const int gx = (a.H + 7) / 8;
  if (a.B <= 16)
    hipLaunchKernelGGL((step_fwd_kernel<1, VEC>), dim3(gx, 1), dim3(256), 0, s, a);
  else if (a.B <= 32)
    hipLaunchKernelGGL((step_fwd_kernel<2, VEC>), dim3(gx, 1), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((step_fwd_kernel<4, VEC>), dim3(gx, (a.B + 63) / 64), dim3(256), 0, s, a);
  return hipGetLastError();
}
template <bool VEC>
hipError_t launch_bwd_nt(const StepBwdArgs& a0, hipStream_t s) {
  StepBwdArgs a = a0;
  const int bt = a.B <= 64 ? 1 : (a.B + 63) / 64;
  a.units_per_wg = (((a.H + 15) / 16) * bt < 192) ? 8 : 16;
  const int gx = (a.H + a.units_per_wg - 1) / a.units_per_wg;
  if (a.B <= 16)
    hipLaunchKernelGGL((step_bwd_kernel<1, VEC>), dim3(gx, 1), dim3(256), 0, s, a);
  else if (a.B <= 32)
    hipLaunchKernelGGL((step_bwd_kernel<2, VEC>), dim3(gx, 1), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((step_bwd_kernel<4, VEC>), dim3(gx, (a.B + 63) / 64), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_step_fwd(const StepFwdArgs& a, hipStream_t stream) {
  const bool vec = (a.H % 4 == 0) && aligned16(a.R) && (a.h_prev == nullptr || aligned16(a.h_prev));
  return vec ? launch_fwd_nt<true>(a, stream) : launch_fwd_nt<false>(a, stream);
}

hipError_t launch_step_bwd(const StepBwdArgs& a, hipStream_t stream) {
  const bool vec = aligned16(a.RT) && (a.dA_next == nullptr || aligned16(a.dA_next));  // K = 4H is a multiple of 4
  return vec ? launch_bwd_nt<true>(a, stream) : launch_bwd_nt<false>(a, stream);
}

}  // namespace lstm
