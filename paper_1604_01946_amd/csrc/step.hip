// Fused per-step kernels: recurrent GEMM over the four stacked gates with the point-wise
// cell update as its epilogue (forward), the mirrored backward step, and the weight pack
// kernels that feed them.
//
// Section 2.1 of arXiv 1604.01946 stacks the four gate matrices that share an input into
// one [4H x H] operand; Section 2.2.2 fuses all point-wise work of a cell into one kernel;
// Section 2.3 re-lays the weight matrices out once per pass because they are reused by every
// step.  Here a workgroup owns a slice of hidden units *with all four gate rows of that
// slice*, so the gate pre-activations never leave the chip, and the per-pass re-layout goes
// further than a transpose: the recurrent matrix is packed into exactly the order in which
// the step kernel's waves consume it, so that a step streams it with whole 1 KB loads at
// consecutive addresses (at large H the step is bound by reading R once, nothing else).
//
// Mapping (forward): workgroup = 4*MT hidden units x (16*NT) batch rows; the 16*MT weight rows
// (unit-major, gate-minor) are the M side of v_mfma_f32_16x16x4_f32, the batch is the N side,
// and K = H is split into four contiguous quarters, one per wave.  Lane (q = lane/16,
// n = lane%16) holds k = 16*ks + 4q .. +3 of row n for k-step ks, and element e of that
// 16-byte value feeds the e-th MFMA of the k-step; the B operand (h_{t-1}, [B][H]) is read
// straight from memory the same way.  The four partial sums meet in LDS; in the D layout a
// lane already holds all four gates of one (unit, batch) cell.
// Backward: workgroup = upw (8 or 16) hidden units x (16*NT) batch rows, K = 4H over the
// transposed recurrent matrix; the epilogue is the point-wise gate-gradient computation.
#include "internal.h"
#include "knobs.h"

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

// k-steps (of 16) per wave for a contraction length K
__host__ __device__ inline int ksteps_per_wave(int K) { return (((K + 15) / 16) + 3) / 4; }

// ------------------------------------------------------------------ weight pack (once per pass)
// Forward order: [slice][wave][k-step][m-tile][lane][4]; zero where the slice or K runs out.
__global__ void pack_fwd_kernel(const float* __restrict__ R, floatx4* __restrict__ Rp, int H, int MT, long per_layer) {
  const int per = ksteps_per_wave(H);
  const int NS = (H + 4 * MT - 1) / (4 * MT);
  const long total = (long)NS * 4 * per * MT * 64;
  const float* Rl = R + (size_t)blockIdx.y * 4 * H * H;
  floatx4* out = Rp + (size_t)blockIdx.y * per_layer;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int lane = (int)(i & 63);
    long r = i >> 6;
    const int mt = (int)(r % MT); r /= MT;
    const int ksl = (int)(r % per); r /= per;
    const int w = (int)(r & 3);
    const int s = (int)(r >> 2);
    const int q = lane >> 4, n = lane & 15;
    const int unit = s * 4 * MT + 4 * mt + (n >> 2), gate = n & 3;
    const int k = (w * per + ksl) * 16 + 4 * q;
    floatx4 v = {0.f, 0.f, 0.f, 0.f};
    if (unit < H) {
      const float* row = Rl + ((size_t)gate * H + unit) * H;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (k + e < H) v[e] = row[k + e];
    }
    out[i] = v;
  }
}

// Backward order: [slice][wave][k-step][lane][4] over R^T (row = hidden unit, K = 4H).
__global__ void pack_bwd_kernel(const float* __restrict__ R, floatx4* __restrict__ Rp, int H, int upw, long per_layer) {
  const int K = 4 * H, per = ksteps_per_wave(K);
  const int NS = (H + upw - 1) / upw;
  const long total = (long)NS * 4 * per * 64;
  const float* Rl = R + (size_t)blockIdx.y * 4 * H * H;
  floatx4* out = Rp + (size_t)blockIdx.y * per_layer;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    // lanes of one output block differ in n fastest: the source reads run along the unit axis
    const int lane = (int)(i & 63);
    long r = i >> 6;
    const int ksl = (int)(r % per); r /= per;
    const int w = (int)(r & 3);
    const int s = (int)(r >> 2);
    const int q = lane >> 4, n = lane & 15;
    const int unit = s * upw + n;
    const int k = (w * per + ksl) * 16 + 4 * q;
    floatx4 v = {0.f, 0.f, 0.f, 0.f};
    if (n < upw && unit < H) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (k + e < K) v[e] = Rl[(size_t)(k + e) * H + unit];
    }
    out[i] = v;
  }
}

// ------------------------------------------------------------------ forward step
// TWO: short load chunks and at most 256 registers, so that two waves share a SIMD (the host asks for it where the
// step is bound by the matrix cores and one workgroup per CU would leave them waiting on its own loads).
template <int NT, int MT, bool VEC, bool TWO = false>
__global__ __launch_bounds__(256, TWO ? 2 : 1) void step_fwd_kernel(const StepFwdArgs a) {
  __shared__ float part[4][MT * NT * 4][64];
  const int H = a.H, B = a.B;
  const int u0 = blockIdx.x * 4 * MT, b0 = blockIdx.y * 16 * NT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, n = lane & 15;

  floatx4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[mt][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  if (a.h_prev) {
    const int per = ksteps_per_wave(H);
    const floatx4* ap = reinterpret_cast<const floatx4*>(a.Rp) + ((size_t)(blockIdx.x * 4 + wave) * per) * MT * 64 + lane;
    const float* brow[NT];
    bool bvalid[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int bb = b0 + 16 * j + n;
      bvalid[j] = bb < B;
      brow[j] = a.h_prev + (long)(bvalid[j] ? bb : 0) * H;
    }
    // Chunks of U k-steps, double-buffered: the loads of chunk c+1 are issued before the MFMAs of
    // chunk c, so with one wave per SIMD the weight stream still overlaps the matrix work (the
    // scheduling barriers keep the compiler from re-serialising loads and MFMAs).
    constexpr int U = TWO ? 2 : 4;
    const int klim = min(H, (wave + 1) * per * 16);
    floatx4 av[2][U][MT], bv[2][U][NT];
    auto load_chunk = [&](int c, floatx4 (&ava)[U][MT], floatx4 (&bva)[U][NT]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int ksl = c * U + u;
        const bool in = ksl < per;
        const int k = (wave * per + ksl) * 16 + 4 * q;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) ava[u][mt] = in ? ap[(size_t)(ksl * MT + mt) * 64] : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NT; ++j) bva[u][j] = load4<VEC>(brow[j], k, klim, bvalid[j] && in);
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
    const int nch = (per + U - 1) / U;
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
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) part[wave][(mt * NT + j) * 4 + r][lane] = acc[mt][j][r];
  __syncthreads();

  // D layout: register r of lane (q, n) is row 4q + r = (unit_local q, gate r), column n (batch).
  for (int p = wave; p < MT * NT; p += 4) {
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
      const float ig = sigmoidf_dev(s[0]), fg = sigmoidf_dev(s[1]), og = sigmoidf_dev(s[2]), gg = tanhf_dev(s[3]);
      const float cp = a.c_prev ? a.c_prev[e] : 0.f;
      const float c = fg * cp + ig * gg;
      const float h = og * tanhf_dev(c);
      a.gates_out[g0] = ig; a.gates_out[g0 + H] = fg; a.gates_out[g0 + 2L * H] = og; a.gates_out[g0 + 3L * H] = gg;
      a.c_out[e] = c; a.h_out[e] = h;
      if (a.h_out2) a.h_out2[e] = h;
      if (a.c_out2) a.c_out2[e] = c;
    }
  }
}

// ------------------------------------------------------------------ backward step
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
    const int per = ksteps_per_wave(K);
    const floatx4* ap = reinterpret_cast<const floatx4*>(a.RTp) + ((size_t)(blockIdx.x * 4 + wave) * per) * 64 + lane;
    const float* brow[NT];
    bool bvalid[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int bb = b0 + 16 * j + n;
      bvalid[j] = bb < B;
      brow[j] = a.dA_next + (long)(bvalid[j] ? bb : 0) * K;
    }
    constexpr int U = 4;
    const int klim = min(K, (wave + 1) * per * 16);
    floatx4 av[2][U], bv[2][U][NT];
    auto load_chunk = [&](int c, floatx4 (&ava)[U], floatx4 (&bva)[U][NT]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int ksl = c * U + u;
        const bool in = ksl < per;
        const int k = (wave * per + ksl) * 16 + 4 * q;
        ava[u] = in ? ap[(size_t)ksl * 64] : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NT; ++j) bva[u][j] = load4<VEC>(brow[j], k, klim, bvalid[j] && in);
      }
    };
    auto mma_chunk = [&](const floatx4 (&ava)[U], const floatx4 (&bva)[U][NT]) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int j = 0; j < NT; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(ava[u][e], bva[u][j][e], acc[j], 0, 0, 0);
    };
    const int nch = (per + U - 1) / U;
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
      const float tc = tanhf_dev(a.c_t[e]);
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
inline int batch_tiles_y(int B) { return B <= 64 ? 1 : (B + 63) / 64; }

template <int MT, bool VEC>
hipError_t launch_fwd_mt(const StepFwdArgs& a, hipStream_t s) {
  const int gx = (a.H + 4 * MT - 1) / (4 * MT);
  if (a.B <= 16)
    hipLaunchKernelGGL((step_fwd_kernel<1, MT, VEC>), dim3(gx, 1), dim3(256), 0, s, a);
  else if (a.B <= 32)
    hipLaunchKernelGGL((step_fwd_kernel<2, MT, VEC>), dim3(gx, 1), dim3(256), 0, s, a);
  else if (MT == 4 && a.B <= 64)
    hipLaunchKernelGGL((step_fwd_kernel<4, MT, VEC, MT == 4>), dim3(gx, 1), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((step_fwd_kernel<4, MT, VEC>), dim3(gx, (a.B + 63) / 64), dim3(256), 0, s, a);
  return hipGetLastError();
}
template <bool VEC>
hipError_t launch_bwd_nt(const StepBwdArgs& a, hipStream_t s) {
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

// Every workgroup reads all of h_{t-1} for its batch rows: 8 units per workgroup halve those re-reads against 4,
// 16 halve them again (at H = 4096 they are otherwise twice the stream of R itself); fewer units per workgroup
// where more would leave CUs idle.
int step_fwd_mtiles(int H, int B) {
  const int forced = knobs().step_mt;
  if (forced == 1 || forced == 2 || forced == 4) return forced;
  if (((H + 15) / 16) * batch_tiles_y(B) >= 200) return 4;
  return (((H + 7) / 8) * batch_tiles_y(B) < 200) ? 1 : 2;
}
int step_bwd_units(int H, int B) { return (((H + 15) / 16) * batch_tiles_y(B) < 192) ? 8 : 16; }

size_t step_pack_floats(int H) {
  // upper bound of both packed layouts for one layer, in floats
  // forward: ceil(H / (4 MT)) slices of MT m-tiles, MT <= 4: at most (H + 3) / 4 + 3 m-tiles of 4 waves x per x 256 floats
  const size_t fwd = (size_t)((H + 3) / 4 + 3) * 4 * ksteps_per_wave(H) * 256;
  const size_t bwd = (size_t)((H + 7) / 8) * 4 * ksteps_per_wave(4 * H) * 256;
  return fwd > bwd ? fwd : bwd;
}

hipError_t launch_pack_fwd(const float* R, float* Rp, int L, int H, int B, size_t per_layer_floats, hipStream_t s) {
  const int MT = step_fwd_mtiles(H, B);
  hipLaunchKernelGGL(pack_fwd_kernel, dim3(512, L), dim3(256), 0, s, R, reinterpret_cast<floatx4*>(Rp), H, MT,
                     (long)(per_layer_floats / 4));
  return hipGetLastError();
}

hipError_t launch_pack_bwd(const float* R, float* RTp, int L, int H, int B, size_t per_layer_floats, hipStream_t s) {
  const int upw = step_bwd_units(H, B);
  hipLaunchKernelGGL(pack_bwd_kernel, dim3(512, L), dim3(256), 0, s, R, reinterpret_cast<floatx4*>(RTp), H, upw,
                     (long)(per_layer_floats / 4));
  return hipGetLastError();
}

hipError_t launch_step_fwd(const StepFwdArgs& a, hipStream_t stream) {
  const bool vec = (a.H % 4 == 0) && (a.h_prev == nullptr || aligned16(a.h_prev));
  const int MT = step_fwd_mtiles(a.H, a.B);
  if (a.h_prev) prof_flops(2.0 * a.B * 4.0 * a.H * a.H, "step_fwd_kernel");
  if (MT == 1) return vec ? launch_fwd_mt<1, true>(a, stream) : launch_fwd_mt<1, false>(a, stream);
  if (MT == 4) return vec ? launch_fwd_mt<4, true>(a, stream) : launch_fwd_mt<4, false>(a, stream);
  return vec ? launch_fwd_mt<2, true>(a, stream) : launch_fwd_mt<2, false>(a, stream);
}

hipError_t launch_step_bwd(const StepBwdArgs& a0, hipStream_t stream) {
  StepBwdArgs a = a0;
  a.units_per_wg = step_bwd_units(a.H, a.B);
  if (a.dA_next) prof_flops(2.0 * a.B * 4.0 * a.H * a.H, "step_bwd_kernel");
  const bool vec = (a.dA_next == nullptr || aligned16(a.dA_next));  // K = 4H is a multiple of 4
  return vec ? launch_bwd_nt<true>(a, stream) : launch_bwd_nt<false>(a, stream);
}

}  // namespace lstm
