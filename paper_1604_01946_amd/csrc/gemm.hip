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
#include "knobs.h"

#include <stdlib.h>
#include <algorithm>
#include <type_traits>

namespace lstm {
namespace {

constexpr int KT = 16;   // k extent of one LDS tile
constexpr int PAD = 4;   // row padding (floats) of the LDS tiles; keeps 16-byte alignment

struct GemmGroupArgs {
  GemmProblem p[kMaxGemmGroup];
  int tile_start[kMaxGemmGroup + 1];
  int nprob;
  int n_main;  // tiles [0, n_main) are dispatched before the rest (launch_gemm_split: whole tiles before K slices)
};

// blockIdx -> tile index.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): remap so that one
// XCD works on a contiguous run of tiles, which share operand panels -- separately for the tiles before and from
// n_main on, so that the hardware's dispatch order (ascending blockIdx) still reaches every tile of the first part
// before any of the second.
__device__ __forceinline__ int tile_index(const GemmGroupArgs& g) {
  int bid = blockIdx.x, lo = 0, n = g.n_main;
  if (bid >= n) {
    lo = n;
    n = (int)gridDim.x - n;
    bid -= lo;
  }
  if ((n & 7) == 0 && (lo & 7) == 0) bid = (bid & 7) * (n >> 3) + (bid >> 3);
  return lo + bid;
}

enum LoadMode : int { LM_SCALAR = 0, LM_KCONTIG = 1, LM_RCONTIG = 2 };

__host__ __device__ inline int pick_mode(const float* base, long s_r, long s_k, int R, int K) {
  const bool aligned = (reinterpret_cast<uintptr_t>(base) & 15u) == 0;
  if (aligned && s_k == 1 && (K % 4) == 0 && (s_r % 4) == 0) return LM_KCONTIG;
  if (aligned && s_r == 1 && (R % 4) == 0 && (s_k % 4) == 0) return LM_RCONTIG;
  return LM_SCALAR;
}

// Moves one operand's [ROWS x KT] tiles from global memory to LDS (k-major) in slots of four
// floats per thread.  The k-tiles of a slot are loaded in order 0, 1, 2, ...; `cur` is the address
// of the next one and advances by one 64-bit add, so that the address arithmetic between the MFMAs
// of the main loop stays a handful of instructions.  Every load is unconditional and reads a valid
// address (past the last k-tile it re-reads the last one, a row outside the matrix reads the
// matrix base) and the value is then replaced by zero where it lies outside: a guarded load would
// put branches into the main loop, and with them the compiler moves the accumulators between
// register files on every iteration.
template <int ROWS, int MODE>
struct TileMover {
  static constexpr int PER_THREAD = ROWS * KT / 256;
  static constexpr int SLOTS = PER_THREAD / 4;
  static constexpr int LDS_STRIDE = ROWS + PAD;

  const float* cur[SLOTS];  // vector modes: address of the slot in the next k-tile to load
  int ktiles[SLOTS];        // vector modes: k-tiles for which the slot is inside the matrix (0: row outside)
  int lds[SLOTS];           // vector modes: LDS offset of the slot
  long step;                // elements between consecutive k-tiles
  // scalar mode keeps the full description
  const float* base;
  long s_r, s_k;
  int r0, R, K, tid;

  __device__ void init(const float* b, long sr, long sk, int r0_, int R_, int K_, int tid_) {
    base = b; s_r = sr; s_k = sk; r0 = r0_; R = R_; K = K_; tid = tid_;
    step = (long)KT * sk;
#pragma unroll
    for (int v = 0; v < SLOTS; ++v) {
      const int idx = tid + 256 * v;
      int row, k;
      if (MODE == LM_KCONTIG) {
        row = idx / (KT / 4); k = 4 * (idx % (KT / 4));
      } else {
        k = idx / (ROWS / 4); row = 4 * (idx % (ROWS / 4));
      }
      lds[v] = k * LDS_STRIDE + row;
      const bool inside = r0 + row < R && k < K;
      cur[v] = b + (inside ? (long)(r0 + row) * sr + (long)k * sk : 0);
      ktiles[v] = inside ? (K - k + KT - 1) / KT : 0;
    }
  }

  // slot v of k-tile kt -> reg[4v .. 4v+3], raw (store() zeroes what lies outside the matrix: doing
  // it here would make the wave wait for the data at once); the k-tiles of a slot must be requested
  // in order from 0
  __device__ __forceinline__ void load(float (&reg)[PER_THREAD], int v, int kt) {
    if (MODE == LM_SCALAR) {
#pragma unroll
      for (int i = 4 * v; i < 4 * v + 4; ++i) {
        const int e = tid + 256 * i;
        const int row = r0 + e % ROWS, k = kt * KT + e / ROWS;
        reg[i] = base[(row < R && k < K) ? (long)row * s_r + (long)k * s_k : 0];
      }
    } else {
      const float4 val = *reinterpret_cast<const float4*>(cur[v]);
      reg[4 * v + 0] = val.x; reg[4 * v + 1] = val.y; reg[4 * v + 2] = val.z; reg[4 * v + 3] = val.w;
      cur[v] += (kt + 1 < ktiles[v]) ? step : 0;
    }
  }

  // reg[4v .. 4v+3], loaded for k-tile kt -> LDS tile S
  __device__ __forceinline__ void store(const float (&reg)[PER_THREAD], int v, int kt, float* __restrict__ S) const {
    if (MODE == LM_SCALAR) {
#pragma unroll
      for (int i = 4 * v; i < 4 * v + 4; ++i) {
        const int e = tid + 256 * i;
        const int row = r0 + e % ROWS, k = kt * KT + e / ROWS;
        S[(e / ROWS) * LDS_STRIDE + (e % ROWS)] = (row < R && k < K) ? reg[i] : 0.f;
      }
    } else {
      const bool inside = kt < ktiles[v];
      const float4 val = make_float4(inside ? reg[4 * v + 0] : 0.f, inside ? reg[4 * v + 1] : 0.f,
                                     inside ? reg[4 * v + 2] : 0.f, inside ? reg[4 * v + 3] : 0.f);
      if (MODE == LM_KCONTIG) {
        S[lds[v]] = val.x; S[lds[v] + LDS_STRIDE] = val.y;
        S[lds[v] + 2 * LDS_STRIDE] = val.z; S[lds[v] + 3 * LDS_STRIDE] = val.w;
      } else {
        *reinterpret_cast<float4*>(S + lds[v]) = val;
      }
    }
  }
};

// MA / MB: load mode of the A / B operand, fixed at compile time (LM_SCALAR handles anything).
template <int WM, int WN, int MA, int MB>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmGroupArgs g) {
  constexpr int MT = 64 * WM, NT = 64 * WN;
  using IOA = TileMover<MT, MA>;
  using IOB = TileMover<NT, MB>;
  constexpr int SA = IOA::SLOTS, SB = IOB::SLOTS, SLOTS = SA + SB, KP = KT / 2;
  static_assert(SLOTS + 3 <= KP && KP % 4 == 0, "the k-pairs of one tile must have room for the store slots before the barrier");
  __shared__ __attribute__((aligned(16))) float As[2][KT * IOA::LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) float Bs[2][KT * IOB::LDS_STRIDE];

  // which problem, which tile
  int pi = 0;
  const int bid = tile_index(g);
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

  // Software pipeline over k-tiles of KT, all stages in one instruction stream so that a single wave
  // keeps the matrix pipe busy without relying on other waves to cover its waits:
  //   G(t)  global -> registers, two tiles ahead (two register sets, so a miss to HBM has two tiles
  //         of MFMA time to return), one slot per k-pair at the start of a tile;
  //   S(t)  registers -> LDS, one tile ahead, one slot per k-pair before the barrier;
  //   F     LDS -> operand fragments, two k-pairs ahead of the MFMAs that use them (a ring of four);
  //   one barrier per tile, before the last two k-pairs: it publishes S(t+1) and closes the reads of
  //   tile t (the fragments of its last k-pairs are fetched before it), so the first fragments of
  //   tile t+1 are fetched under the last MFMAs of tile t.
  // Spreading G and S over the k-pairs matters: their address arithmetic issued in one clump holds
  // the wave between two MFMAs for longer than an MFMA lasts.  Loads past K give zeros, so the
  // stages run unconditionally.
  IOA ia;
  IOB ib;
  ia.init(P.A, P.sAm, P.sAk, m0, P.M, P.K, tid);
  ib.init(P.B, P.sBn, P.sBk, n0, P.N, P.K, tid);
  float ra[2][IOA::PER_THREAD], rb[2][IOB::PER_THREAD];
  const int nk = (P.K + KT - 1) / KT;
  const int aoff = (lane >> 5) * IOA::LDS_STRIDE + wm * 32 * WM + (lane & 31);
  const int boff = (lane >> 5) * IOB::LDS_STRIDE + wn * 32 * WN + (lane & 31);
  constexpr int AHEAD = 2;  // k-pairs between the fetch of a fragment pair and the MFMAs that use it
  float fa[4][WM], fb[4][WN];
  auto fetch = [&](int buf, int kk, int slot) {
#pragma unroll
    for (int i = 0; i < WM; ++i) fa[slot][i] = As[buf][aoff + 2 * kk * IOA::LDS_STRIDE + 32 * i];
#pragma unroll
    for (int j = 0; j < WN; ++j) fb[slot][j] = Bs[buf][boff + 2 * kk * IOB::LDS_STRIDE + 32 * j];
  };
#pragma unroll
  for (int t = 0; t < 2; ++t) {
#pragma unroll
    for (int v = 0; v < SA; ++v) ia.load(ra[t], v, t);
#pragma unroll
    for (int v = 0; v < SB; ++v) ib.load(rb[t], v, t);
  }
#pragma unroll
  for (int v = 0; v < SA; ++v) ia.store(ra[0], v, 0, As[0]);
#pragma unroll
  for (int v = 0; v < SB; ++v) ib.store(rb[0], v, 0, Bs[0]);
  __syncthreads();
#pragma unroll
  for (int kk = 0; kk < AHEAD; ++kk) fetch(0, kk, kk);

  // one k-tile; PAR = parity of kt (LDS buffer and register set), a compile-time constant so that
  // the register arrays keep static indices
  auto tile = [&](auto par, int kt) {
    constexpr int PAR = decltype(par)::value;
    constexpr int BAR = KP - 1 - AHEAD;  // the barrier follows the MFMAs of this k-pair
#pragma unroll
    for (int kk = 0; kk < KP; ++kk) {
      if (kk < SLOTS) {  // G(kt + 2), slot kk
        if (kk < SA) ia.load(ra[PAR], kk < SA ? kk : 0, kt + 2);
        else ib.load(rb[PAR], kk >= SA ? kk - SA : 0, kt + 2);
      }
      constexpr int S0 = BAR + 1 - SLOTS;  // first k-pair of the store stage; the last one is BAR
      if (kk >= S0 && kk <= BAR) {  // S(kt + 1), slot kk - S0
        const int v = kk - S0;
        if (v < SA) ia.store(ra[PAR ^ 1], v < SA ? v : 0, kt + 1, As[PAR ^ 1]);
        else ib.store(rb[PAR ^ 1], v >= SA ? v - SA : 0, kt + 1, Bs[PAR ^ 1]);
      }
      if (kk + AHEAD < KP) fetch(PAR, kk + AHEAD, (kk + AHEAD) & 3);
      else fetch(PAR ^ 1, kk + AHEAD - KP, (kk + AHEAD) & 3);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[kk & 3][i], fb[kk & 3][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (kk == BAR) __syncthreads();
    }
  };
  // an odd tile count is rounded up (the extra tile multiplies zeros): the loop body stays one
  // straight line of code
  for (int kt = 0; kt < nk; kt += 2) {
    tile(std::integral_constant<int, 0>{}, kt);
    tile(std::integral_constant<int, 1>{}, kt + 1);
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

// ------------------------------------------------------------------ direct-to-LDS variant
// The kernel above spends about a fifth of its time on the instructions that move operand tiles
// through registers (address arithmetic, zero selects, LDS stores): on this hardware they are not
// hidden behind the MFMAs of the same wave.  This variant takes them out of the main loop:
//   * global_load_lds_dwordx4 writes 16 bytes per lane straight into LDS (one instruction per KB,
//     scalar base + constant per-lane offset, so advancing to the next k-tile is scalar arithmetic);
//   * three LDS stages, tiles requested two ahead, one barrier per tile;
//   * an operand with unit stride along K keeps its natural [row][16 k] layout in LDS with the four
//     16-byte pieces of a row XOR-swizzled by (row/2)%4, and a lane fetches four MFMA steps' worth of
//     operand with one conflict-free ds_read_b128; an operand with unit stride along the row dimension
//     lands k-major ([k][row]) and is fetched with ds_read_b32 as before.
// MFMA step (blk, s) of a k-tile multiplies k = 8*blk + 4*h + s for the lane half h = lane/32, the
// same pairing for both operands.  Requirements (else the kernel above runs): both operands in a
// vector mode, K a multiple of KT, byte offsets inside an operand below 2^31.  Rows past the end of
// an operand re-read its last rows; they only reach outputs that are not stored.
constexpr int DL_STAGES = 3;

template <int W, int ROWS, int MODE>
struct DlOperand {
  static constexpr int TILE = ROWS * KT;           // floats per stage
  static constexpr int CPW = ROWS / 64;            // 1 KB chunks per wave and tile (4 waves)
  static constexpr bool kInterleaved = MODE == LM_RCONTIG && W == 2;
  const char* sb;                                   // scalar: address of the next tile to request
  long step;                                        // bytes between k-tiles
  unsigned voff[CPW];                               // per-lane byte offset inside the tile, per chunk
  int rd[W][2];                                     // per-lane LDS float offset inside a stage (K mode: per blk)

  __device__ void init(const float* base, long s_r, long s_k, int r0, int R, int wave, int lane, int w0) {
    if (MODE == LM_KCONTIG) {
      sb = reinterpret_cast<const char*>(base);
      step = (long)KT * 4;
#pragma unroll
      for (int j = 0; j < CPW; ++j) {
        const int row = 16 * (wave * CPW + j) + (lane >> 2), p = lane & 3;
        const int kq = p ^ ((row >> 1) & 3);
        const int ra = min(r0 + row, R - 1);
        voff[j] = (unsigned)(((long)ra * s_r + 4 * kq) * 4);
      }
#pragma unroll
      for (int i = 0; i < W; ++i) {
        const int r = w0 + 32 * i + (lane & 31), h = lane >> 5;
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) rd[i][blk] = r * KT + 4 * ((2 * blk + h) ^ ((r >> 1) & 3));
      }
    } else {
      sb = reinterpret_cast<const char*>(base);
      step = (long)KT * s_k * 4;
      constexpr int KPC = 256 / ROWS;  // k-rows per chunk
#pragma unroll
      for (int j = 0; j < CPW; ++j) {
        const int k = (wave * CPW + j) * KPC + (4 * lane) / ROWS, row = (4 * lane) % ROWS;
        const int ra = min(r0 + row, R - 4);
        voff[j] = (unsigned)(((long)k * s_k + ra) * 4);
      }
      // Two tiles per wave: the tiles take every other row of the wave's 64 (tile i: rows 2 r + i), so that a lane's
      // values for both tiles lie side by side in LDS and come with one 8-byte read (kInterleaved; the epilogue maps
      // the rows back).
#pragma unroll
      for (int i = 0; i < W; ++i)
        rd[i][0] = rd[i][1] = (4 * (lane >> 5)) * ROWS + w0 + (kInterleaved ? 2 * (lane & 31) + i : 32 * i + (lane & 31));
    }
  }

  // request the next tile into stage `st` of this operand's LDS area; `more`: a further tile exists.
  // Written as inline assembly on purpose: through the compiler's builtin every later LDS read is
  // made to wait for all outstanding requests (it cannot tell the stages apart), which would undo
  // the prefetch.  M0 carries the wave's LDS destination; nothing else in this kernel uses M0.  The
  // caller orders the requests against the reads with its own waits.
  __device__ __forceinline__ void request(float* lds, int st, int wave, bool more) {
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
      const unsigned dst = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(lds + st * TILE + (wave * CPW + j) * 256);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff[j]), "s"(sb) : "memory");
    }
    sb += more ? step : 0;
  }

  // operand fragments of block blk (4 MFMA steps) of the tile in the stage at float offset `so`;
  // part q of 4 (so that the reads can be spread over four steps)
  __device__ __forceinline__ void fetch(float (&f)[W][4], const float* lds, int so, int blk, int q) const {
    if (MODE == LM_KCONTIG) {
#pragma unroll
      for (int i = 0; i < W; ++i)
        if ((i & 3) == q) {
          const floatx4 x = *reinterpret_cast<const floatx4*>(lds + so + rd[i][blk]);
          f[i][0] = x[0]; f[i][1] = x[1]; f[i][2] = x[2]; f[i][3] = x[3];
        }
    } else if (kInterleaved) {
      const floatx2 x = *reinterpret_cast<const floatx2*>(lds + so + rd[0][0] + (8 * blk + q) * ROWS);
      f[0][q] = x[0];
      f[W - 1][q] = x[1];
    } else {
#pragma unroll
      for (int i = 0; i < W; ++i) f[i][q] = lds[so + rd[i][0] + (8 * blk + q) * ROWS];
    }
  }
  // row (or column) of the output that element rho of the wave's tile i stands for, relative to the wave's first
  static __device__ __forceinline__ int out_index(int i, int rho) { return kInterleaved ? 2 * rho + i : 32 * i + rho; }
};

template <int WM, int WN, int MA, int MB>
__global__ __launch_bounds__(256) void gemm_dl_kernel(const GemmGroupArgs g) {
  constexpr int MT = 64 * WM, NT = 64 * WN;
  using OA = DlOperand<WM, MT, MA>;
  using OB = DlOperand<WN, NT, MB>;
  __shared__ __attribute__((aligned(16))) float As[DL_STAGES * OA::TILE];
  __shared__ __attribute__((aligned(16))) float Bs[DL_STAGES * OB::TILE];

  int pi = 0;
  const int bid = tile_index(g);
  while (pi + 1 < g.nprob && bid >= g.tile_start[pi + 1]) ++pi;
  const GemmProblem& P = g.p[pi];
  const int local = bid - g.tile_start[pi];
  const int tiles_n = (P.N + NT - 1) / NT;
  const int m0 = (local / tiles_n) * MT, n0 = (local % tiles_n) * NT;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  OA oa;
  OB ob;
  oa.init(P.A, P.sAm, P.sAk, m0, P.M, wave, lane, wm * 32 * WM);
  ob.init(P.B, P.sBn, P.sBk, n0, P.N, wave, lane, wn * 32 * WN);
  const int nk = P.K / KT;
  constexpr int NG = OA::CPW + OB::CPW;  // requests per wave and tile
  // s_waitcnt with only the vector-memory counter set: at most NG requests (the newest tile) outstanding
  constexpr int WAIT_NEWEST = (NG & 15) | ((NG >> 4) << 14) | (7 << 4) | (15 << 8);
  constexpr int WAIT_ALL = (7 << 4) | (15 << 8);

  // tiles 0 and 1 (a tile index past the end re-reads the last tile; it is never multiplied)
  oa.request(As, 0, wave, 1 < nk);
  ob.request(Bs, 0, wave, 1 < nk);
  oa.request(As, 1, wave, 2 < nk);
  ob.request(Bs, 1, wave, 2 < nk);
  __builtin_amdgcn_s_waitcnt(WAIT_NEWEST);
  __syncthreads();
  float fa[2][WM][4], fb[2][WN][4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    oa.fetch(fa[0], As, 0, 0, q);
    ob.fetch(fb[0], Bs, 0, 0, q);
  }
  int st = 0;  // stage of the tile being multiplied
  for (int kt = 0; kt < nk; ++kt) {
    const int st1 = st == DL_STAGES - 1 ? 0 : st + 1;   // stage of tile kt + 1
    const int st2 = st1 == DL_STAGES - 1 ? 0 : st1 + 1; // stage of tile kt + 2 (last read for tile kt - 1)
    oa.request(As, st2, wave, kt + 3 < nk);
    ob.request(Bs, st2, wave, kt + 3 < nk);
    // block 0 of this tile; the fragments of block 1 are fetched between its steps
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      oa.fetch(fa[1], As, st * OA::TILE, 1, s4);
      ob.fetch(fb[1], Bs, st * OB::TILE, 1, s4);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[0][i][s4], fb[0][j][s4], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // tile kt + 1 has landed (this wave's share; the barrier collects the others') and every wave has
    // fetched its last fragments of tile kt
    __builtin_amdgcn_s_waitcnt(WAIT_NEWEST);
    __syncthreads();
    // block 1; the fragments of block 0 of the next tile are fetched between its steps
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      oa.fetch(fa[0], As, st1 * OA::TILE, 0, s4);
      ob.fetch(fb[0], Bs, st1 * OB::TILE, 0, s4);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[1][i][s4], fb[1][j][s4], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    st = st1;
  }
  __builtin_amdgcn_s_waitcnt(WAIT_ALL);  // no request may still be writing LDS when the workgroup ends

  // (only the instance that the launcher exchanges roles into carries the transposing epilogue: in the others its
  // registers would cost the kernel a resident workgroup per CU)
  if (MA == LM_RCONTIG && MB == LM_KCONTIG && P.ct) {
    // element (r, c) -> C[c * ldc + r].  With the rows of the wave's two tiles interleaved a lane holds, for each of
    // its columns and each group of four accumulator registers, eight consecutive rows: 32 contiguous bytes of C.
    if constexpr (OA::kInterleaved) {
      const bool vec_ok = (P.ldc & 3) == 0 && (reinterpret_cast<uintptr_t>(P.C) & 15u) == 0;
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        const int c = n0 + wn * 32 * WN + OB::out_index(j, lane & 31);
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int r0 = m0 + wm * 64 + 2 * (8 * gq + 4 * (lane >> 5));
          if (c < P.N && r0 < P.M) {
            float* dst = P.C + (long)c * P.ldc + r0;
            if (vec_ok && r0 + 7 < P.M) {
              floatx4 v0 = {acc[0][j][4 * gq], acc[1][j][4 * gq], acc[0][j][4 * gq + 1], acc[1][j][4 * gq + 1]};
              floatx4 v1 = {acc[0][j][4 * gq + 2], acc[1][j][4 * gq + 2], acc[0][j][4 * gq + 3], acc[1][j][4 * gq + 3]};
              if (P.accumulate) {
                v0 += *reinterpret_cast<const floatx4*>(dst);
                v1 += *reinterpret_cast<const floatx4*>(dst + 4);
              }
              *reinterpret_cast<floatx4*>(dst) = v0;
              *reinterpret_cast<floatx4*>(dst + 4) = v1;
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (r0 + e < P.M) {
                  const float v = acc[e & 1][j][4 * gq + (e >> 1)];
                  dst[e] = P.accumulate ? dst[e] + v : v;
                }
            }
          }
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
          const int col = n0 + wn * 32 * WN + OB::out_index(j, lane & 31);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int row = m0 + wm * 32 * WM + OA::out_index(i, 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3));
            if (row < P.M && col < P.N) {
              float* c = P.C + (long)col * P.ldc + row;
              *c = P.accumulate ? (*c + acc[i][j][r]) : acc[i][j][r];
            }
          }
        }
    }
    return;
  }
  if constexpr (OB::kInterleaved) {
    // a lane holds two neighbouring columns (2 c, 2 c + 1: tiles 0 and 1): one 8-byte store per row where C allows it
    const bool pair_ok = (P.ldc & 1) == 0 && (reinterpret_cast<uintptr_t>(P.C) & 7u) == 0;
    const int col = n0 + wn * 64 + 2 * (lane & 31);
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 32 * WM + OA::out_index(i, 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3));
        if (row < P.M && col < P.N) {
          float* c = P.C + (long)row * P.ldc + col;
          if (pair_ok && col + 1 < P.N) {
            floatx2 v = {acc[i][0][r], acc[i][1][r]};
            if (P.accumulate) v += *reinterpret_cast<const floatx2*>(c);
            *reinterpret_cast<floatx2*>(c) = v;
          } else {
            c[0] = P.accumulate ? (c[0] + acc[i][0][r]) : acc[i][0][r];
            if (col + 1 < P.N) c[1] = P.accumulate ? (c[1] + acc[i][1][r]) : acc[i][1][r];
          }
        }
      }
    return;
  }
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      const int col = n0 + wn * 32 * WN + OB::out_index(j, lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 32 * WM + OA::out_index(i, 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3));
        if (row < P.M && col < P.N) {
          float* c = P.C + (long)row * P.ldc + col;
          *c = P.accumulate ? (*c + acc[i][j][r]) : acc[i][j][r];
        }
      }
    }
}

template <int WM, int WN>
bool launch_tile_dl(int ma, int mb, int grid, const GemmGroupArgs& g, hipStream_t s) {
#define LSTM_GEMM_CASE(A_, B_)                                                                      \
  if (ma == A_ && mb == B_) {                                                                       \
    hipLaunchKernelGGL((gemm_dl_kernel<WM, WN, A_, B_>), dim3(grid), dim3(256), 0, s, g);           \
    return true;                                                                                    \
  }
  LSTM_GEMM_CASE(LM_KCONTIG, LM_KCONTIG)
  LSTM_GEMM_CASE(LM_KCONTIG, LM_RCONTIG)
  LSTM_GEMM_CASE(LM_RCONTIG, LM_RCONTIG)
  LSTM_GEMM_CASE(LM_RCONTIG, LM_KCONTIG)
#undef LSTM_GEMM_CASE
  return false;
}

// Whether the direct-to-LDS kernel can run one operand of a problem.
bool dl_operand_ok(int mode, long s_r, long s_k, int R, int K) {
  if (mode == LM_KCONTIG) return R >= 1 && ((long)R * s_r + K) * 4 < (1L << 31);
  if (mode == LM_RCONTIG) return R >= 4 && ((long)KT * s_k + R) * 4 < (1L << 31);
  return false;
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

// LSTM_GEMM_STAGED=1 keeps every product on the register-staged kernel (for comparison and tests).
static bool gemm_force_staged() { return knobs().gemm_staged; }

namespace {
hipError_t launch_group(const GemmProblem* probs, int nprob, int main_probs, bool split, hipStream_t stream);

// C[r][c] = (accumulate ? C[r][c] : 0) + sum over s of part[s][r][c], s ascending
__global__ void split_reduce_kernel(float* __restrict__ C, long ldc, const float* __restrict__ part, int rows, int cols, int S,
                                    int accumulate) {
  const long n4 = (long)rows * (cols / 4);
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n4; e += (long)gridDim.x * blockDim.x) {
    const int r = (int)(e / (cols / 4)), c = 4 * (int)(e % (cols / 4));
    float* dst = C + (long)r * ldc + c;
    floatx4 v = accumulate ? *reinterpret_cast<const floatx4*>(dst) : floatx4{0.f, 0.f, 0.f, 0.f};
    for (int s2 = 0; s2 < S; ++s2) v += *reinterpret_cast<const floatx4*>(part + ((long)s2 * rows + r) * cols + c);
    *reinterpret_cast<floatx4*>(dst) = v;
  }
}

// Workgroups of the 128 x 128 kernels that the chip holds at once.
int gemm_resident_workgroups() {
  static int cached = 0;
  if (cached) return cached;
  int per_cu = 0, dev = 0, cus = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)gemm_dl_kernel<2, 2, LM_KCONTIG, LM_KCONTIG>, 256, 0) !=
          hipSuccess ||
      per_cu < 1)
    per_cu = 2;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      cus < 1)
    cus = 256;
  cached = per_cu * cus;
  return cached;
}
}  // namespace

// One product whose 128 x 128 tiles do not fill the chip evenly: fewer tiles than the chip holds workgroups, or a
// last partial round of tiles (every tile takes the same time, so a round with a few tiles costs as much as a full
// one: at M = 1600, N = 8192 there are 832 tiles for 768 places, and the last 64 tiles doubled the time).  The
// tile rows of that last round (or all rows, if there is no full round) are cut along K into S slices, as many as fill
// the chip once more; the slices write partial tiles to `part`, a small kernel adds them in fixed order.  Whole tiles
// and slices run in one launch, whole tiles first.  Falls back to the plain launch whenever a condition is not met.
hipError_t launch_gemm_split(const GemmProblem& p, float* part, size_t part_bytes, hipStream_t stream) {
  const int tm = (p.M + 127) / 128, tn = (p.N + 127) / 128, tiles = tm * tn, nk = p.K / KT;
  const bool ok = part && knobs().gemm_split && p.M >= 96 && p.N >= 96 && tiles >= 128 && p.K % KT == 0 && (p.N % 4) == 0 &&
                  (p.ldc % 4) == 0 && (reinterpret_cast<uintptr_t>(p.C) & 15u) == 0 && (reinterpret_cast<uintptr_t>(part) & 15u) == 0;
  if (!ok) return launch_gemm_group(&p, 1, stream);
  const int room = gemm_resident_workgroups();
  int rows_tail;
  if (tiles <= room) {
    rows_tail = tm;
  } else {
    const int tail = tiles % room;
    if (tail == 0) return launch_gemm_group(&p, 1, stream);
    rows_tail = (tail + tn - 1) / tn;
  }
  const int tail_tiles = rows_tail * tn;
  const int row0 = (tm - rows_tail) * 128, mt = p.M - row0;
  // Number of slices: the one with the shortest estimated time for the cut rows.  A CU works off the workgroups it
  // holds at about the same total rate whether it holds two or three (per_cu: what it can hold), and at about two
  // thirds of it when it holds one; the slices are dealt out in rounds of `room`; every slice more costs a little in
  // the addition of the partial tiles.  (208 tiles, 768 places: 6 slices; 64 tiles left over: 8.)
  int cus = 256, dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  const int per_cu = room / cus > 0 ? room / cus : 1;
  auto estimate = [&](int S2) {
    const long items = (long)tail_tiles * S2;
    const long full = items / room, rem = items % room;
    const int last = (int)((rem + cus - 1) / cus);
    const double cost_last = last == 0 ? 0.0 : (last == 1 ? 1.5 : (last == 2 ? 2.2 : (double)last));
    return ((double)full * per_cu + cost_last) / S2 + 0.01 * (S2 - 1);
  };
  int S = 1;
  double best = estimate(1) * 0.95;  // a cut has to promise at least 5 %
  for (int S2 = 2; S2 <= 8; ++S2) {
    if (nk / S2 < 8) break;  // at least eight k-tiles per slice
    if ((size_t)S2 * mt * p.N * sizeof(float) > part_bytes) break;
    const double e = estimate(S2);
    if (e < best) {
      best = e;
      S = S2;
    }
  }
  if (S < 2) return launch_gemm_group(&p, 1, stream);
  GemmProblem g[kMaxGemmGroup];
  int n = 0;
  if (row0 > 0) {
    g[n] = p;
    g[n].M = row0;
    ++n;
  }
  const int main_probs = n;
  for (int s2 = 0; s2 < S; ++s2) {
    const int k0 = (int)((long)nk * s2 / S) * KT, k1 = (int)((long)nk * (s2 + 1) / S) * KT;
    GemmProblem q = p;
    q.A = p.A + (long)row0 * p.sAm + (long)k0 * p.sAk;
    q.B = p.B + (long)k0 * p.sBk;
    q.C = part + (size_t)s2 * mt * p.N;
    q.M = mt;
    q.K = k1 - k0;
    q.ldc = p.N;
    q.accumulate = 0;
    g[n++] = q;
  }
  prof_flops(2.0 * p.M * p.N * p.K, "gemm");
  if (hipError_t e = launch_group(g, n, main_probs, true, stream); e != hipSuccess) return e;
  const long n4 = (long)mt * (p.N / 4);
  const unsigned blocks = (unsigned)std::min<long>((n4 + 255) / 256, 2048);
  hipLaunchKernelGGL(split_reduce_kernel, dim3(blocks), dim3(256), 0, stream, p.C + (long)row0 * p.ldc, p.ldc, part, mt, p.N, S,
                     p.accumulate);
  return hipGetLastError();
}

hipError_t launch_gemm_group(const GemmProblem* probs, int nprob, hipStream_t stream) {
  return launch_group(probs, nprob, nprob, false, stream);
}

namespace {
// split: the group is one product cut up by launch_gemm_split (128 x 128 tiles whatever the parts' heights; its FLOPs
// are counted there)
hipError_t launch_group(const GemmProblem* probs, int nprob, int main_probs, bool split, hipStream_t stream) {
  if (nprob <= 0) return hipSuccess;
  if (nprob > kMaxGemmGroup) return hipErrorInvalidValue;
  GemmGroupArgs g;
  bool big = true;
  long total_big = 0, total_small = 0;
  double area = 0.0;
  // one kernel instance serves the whole group: operands that cannot all take the same vector
  // loader fall back to the scalar one
  int ma = -1, mb = -1;
  for (int i = 0; i < nprob; ++i) {
    g.p[i] = probs[i];
    if (probs[i].M < 96 || probs[i].N < 96) big = false;
    total_big += (long)((probs[i].M + 127) / 128) * ((probs[i].N + 127) / 128);
    total_small += (long)((probs[i].M + 63) / 64) * ((probs[i].N + 63) / 64);
    area += (double)probs[i].M * probs[i].N;
    const int a = pick_mode(probs[i].A, probs[i].sAm, probs[i].sAk, probs[i].M, probs[i].K);
    const int b = pick_mode(probs[i].B, probs[i].sBn, probs[i].sBk, probs[i].N, probs[i].K);
    ma = (i == 0 || ma == a) ? a : LM_SCALAR;
    mb = (i == 0 || mb == b) ? b : LM_SCALAR;
  }
  if (ma == LM_SCALAR || mb == LM_SCALAR) ma = mb = LM_SCALAR;
  bool dl = ma != LM_SCALAR && !gemm_force_staged();
  if (!split) {
    double fl = 0.0;
    for (int i = 0; i < nprob; ++i) fl += 2.0 * probs[i].M * probs[i].N * probs[i].K;
    prof_flops(fl, "gemm");
  }
  for (int i = 0; i < nprob && dl; ++i)
    dl = probs[i].K % KT == 0 && probs[i].K >= KT && dl_operand_ok(ma, probs[i].sAm, probs[i].sAk, probs[i].M, probs[i].K) &&
         dl_operand_ok(mb, probs[i].sBn, probs[i].sBk, probs[i].N, probs[i].K);
  // 128 x 128 or 64 x 64 tiles: whichever the counts of tiles promise more from.  Measured on 256 CUs (forward
  // products of one step, K = 2H = 4096 ... 8192): one 128 x 128 workgroup per CU runs at 128 TFLOP/s, two on a CU
  // take 1.85 times as long as one and three 2.7 times (142 TFLOP/s when every CU has three), so between those counts
  // the rate follows the fullest CU: 288 tiles 80 TFLOP/s, 384 tiles 105.  The 64 x 64 kernel reaches 116 TFLOP/s from
  // two tiles per CU on.  Both are scaled by the part of their tiles that the product really covers.
  if (big && !split) {
    const double cus = (double)std::max(device_cu_count(), 1);
    const double nb = (double)total_big / cus, ns = (double)total_small / cus;
    const double rate_big = nb <= 1.0 ? 128.0 * nb
                          : (nb <= 2.0 ? 128.0 * nb / 1.85 : (nb <= 3.0 ? 128.0 * nb / 2.7 : 138.0));
    const double rate_small = 116.0 * std::min(1.0, ns / 2.0);
    const double use_big = area / ((double)total_big * 128.0 * 128.0), use_small = area / ((double)total_small * 64.0 * 64.0);
    big = rate_big * use_big >= rate_small * use_small;
  }
  if (split) big = true;
  // The 128 x 128 kernel is slower with a K-contiguous A operand than with a K-contiguous B operand (2048 x 2048 x 8192:
  // A K- / B row-contiguous 121 TFLOP/s, both K-contiguous 134, A row- / B K-contiguous 142, both row-contiguous 143;
  // neither the order of the tiles, of the waves, of the requests nor of the matrix instructions changes that).  A
  // product with A K-contiguous and B row-contiguous is therefore computed as its transpose, B^T A^T, whose
  // elements the epilogue writes to where C expects them.
  if (dl && big && ma == LM_KCONTIG && mb == LM_RCONTIG && knobs().gemm_swap) {
    for (int i = 0; i < nprob; ++i) {
      GemmProblem& q = g.p[i];
      std::swap(q.A, q.B);
      std::swap(q.M, q.N);
      std::swap(q.sAm, q.sBn);
      std::swap(q.sAk, q.sBk);
      q.ct = !q.ct;
    }
    std::swap(ma, mb);
  }
  const int mt = big ? 128 : 64;
  int start = 0;
  for (int i = 0; i < nprob; ++i) {
    g.tile_start[i] = start;
    start += ((g.p[i].M + mt - 1) / mt) * ((g.p[i].N + mt - 1) / mt);
  }
  for (int i = nprob; i <= kMaxGemmGroup; ++i) g.tile_start[i] = start;
  g.nprob = nprob;
  g.n_main = main_probs < nprob ? g.tile_start[main_probs] : start;
  if (start == 0) return hipSuccess;
  if (dl) {
    if (big)
      launch_tile_dl<2, 2>(ma, mb, start, g, stream);
    else
      launch_tile_dl<1, 1>(ma, mb, start, g, stream);
  } else if (big) {
    launch_tile<2, 2>(ma, mb, start, g, stream);
  } else {
    launch_tile<1, 1>(ma, mb, start, g, stream);
  }
  return hipGetLastError();
}
}  // namespace

}  // namespace lstm
