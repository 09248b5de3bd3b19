// fp32 matrix-core GEMM for gfx950: C[M][N] (+)= A*B, grouped launches.
//
// Used for the time-batched input projection (Section 2.3 of arXiv 1604.01946: the
// inputs of many steps concatenated into one larger product), for the batched
// input-gradient product of the backward pass, and for the weight-gradient products
// that Section 2.6 describes (one large, dependency-free product per matrix).
//
// Design: 256 threads = 4 wave64 in a 2x2 arrangement; each wave owns WM x WN tiles of
// v_mfma_f32_32x32x2_f32.  Operand tiles are staged through LDS k-major ([k][row]) so the
// MFMA operand fetch (lane -> row = lane%32, k = lane/32) is bank-conflict free, with
// register-staged double buffering of the global loads.  Operands may be stored with the
// unit stride along K or along the row dimension; unaligned / odd shapes take a scalar
// guarded loader, so every positive shape works.
#include "internal.h"

namespace lstm {
namespace {

constexpr int KT = 16;   // k extent of one LDS tile
constexpr int PAD = 4;   // row padding (floats) of the LDS tiles; keeps 16-byte alignment

struct GemmGroupArgs {
  GemmProblem p[kMaxGemmGroup];
  int tile_start[kMaxGemmGroup + 1];
  int nprob;
};

enum LoadMode : int { LM_SCALAR = 0, LM_KCONTIG = 1, LM_RCONTIG = 2 };

__host__ __device__ inline int pick_mode(const float* base, long s_r, long s_k, int R, int K) {
  const bool aligned = (reinterpret_cast<uintptr_t>(base) & 15u) == 0;
  if (aligned && s_k == 1 && (K % 4) == 0 && (s_r % 4) == 0) return LM_KCONTIG;
  if (aligned && s_r == 1 && (R % 4) == 0 && (s_k % 4) == 0) return LM_RCONTIG;
  return LM_SCALAR;
}

template <int ROWS>
struct TileIO {
  static constexpr int PER_THREAD = ROWS * KT / 256;
  static constexpr int NVEC = PER_THREAD / 4;
  static constexpr int LDS_STRIDE = ROWS + PAD;

  __device__ static void load(float (&reg)[PER_THREAD], const float* __restrict__ base, long s_r, long s_k, int r0,
                              int k0, int R, int K, int mode, int tid) {
    if (mode == LM_KCONTIG) {
#pragma unroll
      for (int v = 0; v < NVEC; ++v) {
        const int idx = tid + 256 * v;
        const int row = r0 + idx / (KT / 4), k = k0 + 4 * (idx % (KT / 4));
        float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < R && k < K) val = *reinterpret_cast<const float4*>(base + (long)row * s_r + k);
        reg[4 * v + 0] = val.x; reg[4 * v + 1] = val.y; reg[4 * v + 2] = val.z; reg[4 * v + 3] = val.w;
      }
    } else if (mode == LM_RCONTIG) {
#pragma unroll
      for (int v = 0; v < NVEC; ++v) {
        const int idx = tid + 256 * v;
        const int k = k0 + idx / (ROWS / 4), row = r0 + 4 * (idx % (ROWS / 4));
        float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < R && k < K) val = *reinterpret_cast<const float4*>(base + (long)k * s_k + row);
        reg[4 * v + 0] = val.x; reg[4 * v + 1] = val.y; reg[4 * v + 2] = val.z; reg[4 * v + 3] = val.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < PER_THREAD; ++i) {
        const int e = tid + 256 * i;
        const int row = r0 + e % ROWS, k = k0 + e / ROWS;
        reg[i] = (row < R && k < K) ? base[(long)row * s_r + (long)k * s_k] : 0.f;
      }
    }
  }

  __device__ static void store(const float (&reg)[PER_THREAD], float* __restrict__ S, int mode, int tid) {
    if (mode == LM_KCONTIG) {
#pragma unroll
      for (int v = 0; v < NVEC; ++v) {
        const int idx = tid + 256 * v;
        const int row = idx / (KT / 4), k = 4 * (idx % (KT / 4));
#pragma unroll
        for (int j = 0; j < 4; ++j) S[(k + j) * LDS_STRIDE + row] = reg[4 * v + j];
      }
    } else if (mode == LM_RCONTIG) {
#pragma unroll
      for (int v = 0; v < NVEC; ++v) {
        const int idx = tid + 256 * v;
        const int k = idx / (ROWS / 4), row = 4 * (idx % (ROWS / 4));
        *reinterpret_cast<float4*>(S + k * LDS_STRIDE + row) =
            make_float4(reg[4 * v + 0], reg[4 * v + 1], reg[4 * v + 2], reg[4 * v + 3]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < PER_THREAD; ++i) {
        const int e = tid + 256 * i;
        S[(e / ROWS) * LDS_STRIDE + (e % ROWS)] = reg[i];
      }
    }
  }
};

// MA / MB: load mode of the A / B operand, fixed at compile time (LM_SCALAR handles anything).
template <int WM, int WN, int MA, int MB>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmGroupArgs g) {
  constexpr int MT = 64 * WM, NT = 64 * WN;
  using IOA = TileIO<MT>;
  using IOB = TileIO<NT>;
  __shared__ __attribute__((aligned(16))) float As[2][KT * IOA::LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) float Bs[2][KT * IOB::LDS_STRIDE];

  // which problem, which tile
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): remap so that one XCD
  // works on a contiguous run of tiles, which share operand panels.
  int pi = 0;
  int bid = blockIdx.x;
  if ((gridDim.x & 7) == 0) bid = (bid & 7) * (gridDim.x >> 3) + (bid >> 3);
  while (pi + 1 < g.nprob && bid >= g.tile_start[pi + 1]) ++pi;
  const GemmProblem& P = g.p[pi];
  const int local = bid - g.tile_start[pi];
  const int tiles_n = (P.N + NT - 1) / NT;
  const int m0 = (local / tiles_n) * MT, n0 = (local % tiles_n) * NT;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float ra[IOA::PER_THREAD], rb[IOB::PER_THREAD];
  const int nk = (P.K + KT - 1) / KT;
  IOA::load(ra, P.A, P.sAm, P.sAk, m0, 0, P.M, P.K, MA, tid);
  IOB::load(rb, P.B, P.sBn, P.sBk, n0, 0, P.N, P.K, MB, tid);
  IOA::store(ra, As[0], MA, tid);
  IOB::store(rb, Bs[0], MB, tid);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      IOA::load(ra, P.A, P.sAm, P.sAk, m0, (kt + 1) * KT, P.M, P.K, MA, tid);
      IOB::load(rb, P.B, P.sBn, P.sBk, n0, (kt + 1) * KT, P.N, P.K, MB, tid);
    }
    const float* as = As[cur] + (lane >> 5) * IOA::LDS_STRIDE + wm * 32 * WM + (lane & 31);
    const float* bs = Bs[cur] + (lane >> 5) * IOB::LDS_STRIDE + wn * 32 * WN + (lane & 31);
    // all operand fragments of the k-tile are fetched from LDS first; the MFMAs then start as soon as
    // the first fragments arrive and the remaining LDS latency hides under them
    float a[KT / 2][WM], b[KT / 2][WN];
#pragma unroll
    for (int kk = 0; kk < KT / 2; ++kk) {
#pragma unroll
      for (int i = 0; i < WM; ++i) a[kk][i] = as[2 * kk * IOA::LDS_STRIDE + 32 * i];
#pragma unroll
      for (int j = 0; j < WN; ++j) b[kk][j] = bs[2 * kk * IOB::LDS_STRIDE + 32 * j];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < KT / 2; ++kk)
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk][i], b[kk][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (kt + 1 < nk) {
      IOA::store(ra, As[cur ^ 1], MA, tid);
      IOB::store(rb, Bs[cur ^ 1], MB, tid);
    }
    __syncthreads();
  }

  // D layout of the 32x32 tile: register r of lane holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      const int col = n0 + wn * 32 * WN + 32 * j + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 32 * WM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < P.M && col < P.N) {
          float* c = P.C + (long)row * P.ldc + col;
          *c = P.accumulate ? (*c + acc[i][j][r]) : acc[i][j][r];
        }
      }
    }
}

template <int WM, int WN>
void launch_tile(int ma, int mb, int grid, const GemmGroupArgs& g, hipStream_t s) {
#define LSTM_GEMM_CASE(A_, B_)                                                                        \
  if (ma == A_ && mb == B_) {                                                                         \
    hipLaunchKernelGGL((gemm_f32_kernel<WM, WN, A_, B_>), dim3(grid), dim3(256), 0, s, g);            \
    return;                                                                                           \
  }
  LSTM_GEMM_CASE(LM_KCONTIG, LM_KCONTIG)
  LSTM_GEMM_CASE(LM_KCONTIG, LM_RCONTIG)
  LSTM_GEMM_CASE(LM_RCONTIG, LM_RCONTIG)
  LSTM_GEMM_CASE(LM_RCONTIG, LM_KCONTIG)
#undef LSTM_GEMM_CASE
  hipLaunchKernelGGL((gemm_f32_kernel<WM, WN, LM_SCALAR, LM_SCALAR>), dim3(grid), dim3(256), 0, s, g);
}

}  // namespace

hipError_t launch_gemm_group(const GemmProblem* probs, int nprob, hipStream_t stream) {
  if (nprob <= 0) return hipSuccess;
  if (nprob > kMaxGemmGroup) return hipErrorInvalidValue;
  GemmGroupArgs g;
  bool big = true;
  long total_big = 0;
  // one kernel instance serves the whole group: operands that cannot all take the same vector
  // loader fall back to the scalar one
  int ma = -1, mb = -1;
  for (int i = 0; i < nprob; ++i) {
    g.p[i] = probs[i];
    if (probs[i].M < 96 || probs[i].N < 96) big = false;
    total_big += (long)((probs[i].M + 127) / 128) * ((probs[i].N + 127) / 128);
    const int a = pick_mode(probs[i].A, probs[i].sAm, probs[i].sAk, probs[i].M, probs[i].K);
    const int b = pick_mode(probs[i].B, probs[i].sBn, probs[i].sBk, probs[i].N, probs[i].K);
    ma = (i == 0 || ma == a) ? a : LM_SCALAR;
    mb = (i == 0 || mb == b) ? b : LM_SCALAR;
  }
  if (ma == LM_SCALAR || mb == LM_SCALAR) ma = mb = LM_SCALAR;
  // Few large tiles leave most of the 256 CUs idle; fall back to 64x64 tiles then.
  if (total_big < 128) big = false;
  const int mt = big ? 128 : 64;
  int start = 0;
  for (int i = 0; i < nprob; ++i) {
    g.tile_start[i] = start;
    start += ((probs[i].M + mt - 1) / mt) * ((probs[i].N + mt - 1) / mt);
  }
  for (int i = nprob; i <= kMaxGemmGroup; ++i) g.tile_start[i] = start;
  g.nprob = nprob;
  if (start == 0) return hipSuccess;
  if (big)
    launch_tile<2, 2>(ma, mb, start, g, stream);
  else
    launch_tile<1, 1>(ma, mb, start, g, stream);
  return hipGetLastError();
}

}  // namespace lstm
