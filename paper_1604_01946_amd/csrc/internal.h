// Internal declarations shared by the HIP translation units of the LSTM library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lstm {

typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// ---------------------------------------------------------------- GEMM (gemm.hip)
// One dense product C[M][N] (+)= A*B with arbitrary (unit in one dimension) strides.
struct GemmProblem {
  const float* A;
  const float* B;
  float* C;
  int M, N, K;
  long sAm, sAk, sBk, sBn, ldc;
  int accumulate;
  int ct;  // element (r, c) of the product goes to C[c * ldc + r] (set by the launcher when it exchanges the operands' roles)
};
constexpr int kMaxGemmGroup = 16;
// A group of independent products executed by one launch (Section 2.6: the weight
// update products have no dependencies, so they can all be in flight together).
int device_cu_count();  // compute units of the current device (0 if it cannot be read); persistent.hip
hipError_t launch_gemm_group(const GemmProblem* probs, int nprob, hipStream_t stream);
// One product, with the tiles of its last partial round (or all of them, when they are fewer than the chip holds
// workgroups) cut along K; `part` (16-byte aligned, part_bytes long, free until the stream has passed the call) takes
// the partial tiles.  The same result as launch_gemm_group up to the order of the additions, which is fixed.
hipError_t launch_gemm_split(const GemmProblem& p, float* part, size_t part_bytes, hipStream_t stream);

// ---------------------------------------------------------------- point-wise / layout kernels (pointwise.hip)
enum EwOp : int {
  EW_ADD = 0,       // out = a + b
  EW_ADD_BIAS = 1,  // out[r][c] = a[r][c] + b[c]
  EW_SIGMOID = 2,   // out = sigma(a)
  EW_TANH = 3,      // out = tanh(a)
  EW_MUL = 4,       // out = a * b
  EW_FMA_MUL = 5,   // out = out + a * b
  EW_COPY = 6,
};
// Strided 2-D element-wise op over [rows][cols] (one kernel per operation: the
// Section 2.1 starting point).
hipError_t launch_ew(EwOp op, float* out, long ldo, const float* a, long lda, const float* b, long ldb,
                     int rows, int cols, hipStream_t stream);

// Fused forward point-wise update (Section 2.2.2): gates from pre-activations, cell and hidden update.
// pre1 (+ pre2 if non-null) [B][4H], bias [4H], c_prev [B][H] (may be null = zeros).
hipError_t launch_pointwise_fwd(const float* pre1, const float* pre2, const float* bias, const float* c_prev,
                                float* h_out, float* c_out, float* gates_out, float* h_out2, float* c_out2,
                                int B, int H, hipStream_t stream);
// Fused backward point-wise: gate pre-activation gradients dA [B][4H] and dc_{t-1}.
// dh = dh_a + dh_b (either may be null), dc_in may be null.
hipError_t launch_pointwise_bwd(const float* gates, const float* c_t, const float* c_prev, const float* dh_a,
                                const float* dh_b, const float* dc_in, float* dA, float* dc_out, int B, int H,
                                hipStream_t stream);
// out[c][r] = in[r][c] for `batch` matrices laid one after the other.
hipError_t launch_transpose(const float* in, float* out, int rows, int cols, int batch, hipStream_t stream);
// out[n] = sum_r in[r][n]; partial must hold 64*cols floats.
hipError_t launch_colsum(const float* in, int rows, int cols, float* partial, float* out, hipStream_t stream);
hipError_t launch_colsum_batched(const float* in, int rows, int cols, int count, float* partial, float* out,
                                 hipStream_t stream);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream);

// ---------------------------------------------------------------- fused step kernels (step.hip)
struct StepFwdArgs {
  const float* Rp;      // recurrent matrix of this layer, packed by launch_pack_fwd
  const float* h_prev;  // [B][H] or null (zeros)
  const float* c_prev;  // [B][H] or null (zeros)
  const float* P;       // [B][4H] input projection of this step
  const float* bias;    // [4H]
  float* h_out;         // [B][H]
  float* c_out;         // [B][H]
  float* gates_out;     // [B][4H]
  float* h_out2;        // optional second copy of h (y / hT), may be null
  float* c_out2;        // optional second copy of c (cT), may be null
  int B, H;
};
hipError_t launch_step_fwd(const StepFwdArgs& a, hipStream_t stream);

struct StepBwdArgs {
  const float* RTp;      // recurrent matrix of this layer, packed by launch_pack_bwd
  const float* dA_next;  // [B][4H] gate gradients of step t+1, null at the last step
  const float* dh_extra; // [B][H] added to dh (dhT at the last step), may be null
  const float* dout;     // [B][H] gradient from above (dy or the upper layer's input gradient); null when !pointwise
  const float* gates;    // [B][4H] of step t
  const float* c_t;      // [B][H]
  const float* c_prev;   // [B][H] c_{t-1} (c0 at t=0), null = zeros
  const float* dc_in;    // [B][H] carried cell gradient, null = zeros
  float* dA;             // [B][4H] out
  float* dc_out;         // [B][H] out
  float* dh_out;         // [B][H] out when !pointwise (dh0)
  int pointwise;         // 0: only dh_out = dA_next * R (+dh_extra)
  int B, H;
  int units_per_wg;      // set by the launcher
};
hipError_t launch_step_bwd(const StepBwdArgs& a, hipStream_t stream);

// Per-pass weight re-layout for the step kernels (Section 2.3): R [L][4H][H] -> the order in which
// the forward / backward step kernels stream it.  per_layer_floats = step_pack_floats(H).
size_t step_pack_floats(int H);
hipError_t launch_pack_fwd(const float* R, float* Rp, int L, int H, int B, size_t per_layer_floats, hipStream_t s);
hipError_t launch_pack_bwd(const float* R, float* RTp, int L, int H, int B, size_t per_layer_floats, hipStream_t s);

// ---------------------------------------------------------------- split-K step kernels (step_splitk.hip)
struct SplitK {
  float* partial;  // partial sums of this layer
  int* counters;   // arrival counters of this (layer, step), zeroed once per pass
  int KS;          // K slices
  int per;         // k-steps (of 16) per K slice
};
bool splitk_supported(int H);
size_t splitk_pack_floats(int H);
size_t splitk_partial_floats(int H, int B);
size_t splitk_counter_ints(int H, int B);
hipError_t launch_pack_bwd_sk(const float* R, float* RTp, int L, int H, int B, size_t per_layer_floats, hipStream_t s);
hipError_t launch_step_bwd_sk(const StepBwdArgs& a, float* partial, int* counters, hipStream_t s);

// ---------------------------------------------------------------- measurement hook (api.hip)
// Adds the algorithmic FLOPs of a matrix product that is being launched to the innermost open timing interval
// and, when `kernel` is given, names the kernel that carries that phase (no-ops unless lstm_profile_enable(1)).
void prof_flops(double flops, const char* kernel = nullptr);

// ---------------------------------------------------------------- device math
// sigma and tanh on the hardware's exp2 and reciprocal instructions (about 1 ulp each): absolute error of
// a few 1e-7 over the whole range, exact limits at +-infinity (exp2 overflows to inf, 1/inf = 0).  The
// library versions cost four to eight times as many instructions, which the per-step epilogues of the
// recurrent kernels pay on their critical path.
__device__ __forceinline__ float exp_dev(float z) { return __builtin_amdgcn_exp2f(z * 1.44269504088896341f); }
__device__ __forceinline__ float sigmoidf_dev(float z) { return __builtin_amdgcn_rcpf(1.0f + exp_dev(-z)); }
__device__ __forceinline__ float tanhf_dev(float z) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + exp_dev(2.0f * z)); }

}  // namespace lstm
