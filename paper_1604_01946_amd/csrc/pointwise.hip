// Point-wise, layout and reduction kernels of the LSTM library (gfx950).
//
//  * one-operation kernels: the "one kernel per operation" starting point of Section 2.1
//    of arXiv 1604.01946 (used only by the naive / grouped baseline paths);
//  * fused forward / backward point-wise kernels: Section 2.2.2 (all point-wise work of a
//    cell in one kernel, no round trips through memory between the operations);
//  * matrix transpose: Section 2.3 (weights re-laid out once per pass; the backward pass
//    needs the other orientation);
//  * column sum: the bias gradient of Section 2.6.
#include "internal.h"

namespace lstm {
namespace {

__global__ void ew_kernel(int op, float* __restrict__ out, long ldo, const float* __restrict__ a, long lda,
                          const float* __restrict__ b, long ldb, int rows, int cols) {
  const long n = (long)rows * cols;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long)gridDim.x * blockDim.x) {
    const int r = (int)(e / cols), c = (int)(e % cols);
    const float av = a[r * lda + c];
    float v;
    switch (op) {
      case EW_ADD: v = av + b[r * ldb + c]; break;
      case EW_ADD_BIAS: v = av + b[c]; break;
      case EW_SIGMOID: v = sigmoidf_dev(av); break;
      case EW_TANH: v = tanhf_dev(av); break;
      case EW_MUL: v = av * b[r * ldb + c]; break;
      case EW_FMA_MUL: v = out[r * ldo + c] + av * b[r * ldb + c]; break;
      default: v = av; break;
    }
    out[r * ldo + c] = v;
  }
}

// Thread per (batch row, hidden unit); consecutive threads take consecutive units so every
// access to the [B][4H] and [B][H] arrays is a contiguous run.
__global__ void pointwise_fwd_kernel(const float* __restrict__ pre1, const float* __restrict__ pre2,
                                     const float* __restrict__ bias, const float* __restrict__ c_prev,
                                     float* __restrict__ h_out, float* __restrict__ c_out,
                                     float* __restrict__ gates_out, float* __restrict__ h_out2,
                                     float* __restrict__ c_out2, int B, int H) {
  const long n = (long)B * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long)gridDim.x * blockDim.x) {
    const int bb = (int)(e / H), j = (int)(e % H);
    const long g0 = (long)bb * 4 * H + j;
    float a[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      a[q] = pre1[g0 + (long)q * H] + bias[q * H + j];
      if (pre2) a[q] += pre2[g0 + (long)q * H];
    }
    const float ig = sigmoidf_dev(a[0]), fg = sigmoidf_dev(a[1]), og = sigmoidf_dev(a[2]), gg = tanhf_dev(a[3]);
    const float cp = c_prev ? c_prev[e] : 0.f;
    const float c = fg * cp + ig * gg;
    const float h = og * tanhf_dev(c);
    gates_out[g0] = ig; gates_out[g0 + H] = fg; gates_out[g0 + 2L * H] = og; gates_out[g0 + 3L * H] = gg;
    c_out[e] = c; h_out[e] = h;
    if (h_out2) h_out2[e] = h;
    if (c_out2) c_out2[e] = c;
  }
}

__global__ void pointwise_bwd_kernel(const float* __restrict__ gates, const float* __restrict__ c_t,
                                     const float* __restrict__ c_prev, const float* __restrict__ dh_a,
                                     const float* __restrict__ dh_b, const float* __restrict__ dc_in,
                                     float* __restrict__ dA, float* __restrict__ dc_out, int B, int H) {
  const long n = (long)B * H;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long)gridDim.x * blockDim.x) {
    const int bb = (int)(e / H), j = (int)(e % H);
    const long g0 = (long)bb * 4 * H + j;
    const float ig = gates[g0], fg = gates[g0 + H], og = gates[g0 + 2L * H], gg = gates[g0 + 3L * H];
    const float tc = tanhf_dev(c_t[e]);
    float dh = 0.f;
    if (dh_a) dh += dh_a[e];
    if (dh_b) dh += dh_b[e];
    const float dc = (dc_in ? dc_in[e] : 0.f) + dh * og * (1.f - tc * tc);
    const float cp = c_prev ? c_prev[e] : 0.f;
    dA[g0] = dc * gg * ig * (1.f - ig);
    dA[g0 + H] = dc * cp * fg * (1.f - fg);
    dA[g0 + 2L * H] = dh * tc * og * (1.f - og);
    dA[g0 + 3L * H] = dc * ig * (1.f - gg * gg);
    dc_out[e] = dc * fg;
  }
}

__global__ void transpose_kernel(const float* __restrict__ in, float* __restrict__ out, int rows, int cols) {
  __shared__ float tile[32][33];
  const long off = (long)blockIdx.z * rows * cols;
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    const int r = r0 + i, c = c0 + tx;
    tile[i][tx] = (r < rows && c < cols) ? in[off + (long)r * cols + c] : 0.f;
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int c = c0 + i, r = r0 + tx;
    if (r < rows && c < cols) out[off + (long)c * rows + r] = tile[tx][i];
  }
}

constexpr int kColsumChunks = 64;
// grid (ceil(cols/64), kColsumChunks, matrices); 256 threads = 64 columns x 4 row lanes.  Matrix z is in + z*rows*cols,
// its partial sums partial + z*kColsumChunks*cols.
__global__ void colsum_partial_kernel(const float* __restrict__ in, int rows, int cols, float* __restrict__ partial) {
  __shared__ float red[4][64];
  in += (size_t)blockIdx.z * rows * cols;
  partial += (size_t)blockIdx.z * kColsumChunks * cols;
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + cx;
  const int per = (rows + kColsumChunks - 1) / kColsumChunks;
  const int rbeg = blockIdx.y * per, rend = min(rows, rbeg + per);
  float s = 0.f;
  if (col < cols)
    for (int r = rbeg + ry; r < rend; r += 4) s += in[(long)r * cols + col];
  red[ry][cx] = s;
  __syncthreads();
  if (ry == 0 && col < cols) partial[(long)blockIdx.y * cols + col] = (red[0][cx] + red[1][cx]) + (red[2][cx] + red[3][cx]);
}
// The same for cols % 4 == 0 and a 16-byte aligned matrix: grid (ceil(cols/256), kColsumChunks, matrices); a wave reads 1 KB
// of a row per request (four columns per lane), the four waves take every fourth row, four requests in flight each.
__global__ void colsum_partial4_kernel(const float* __restrict__ in, int rows, int cols, float* __restrict__ partial) {
  __shared__ floatx4 red[4][64];
  in += (size_t)blockIdx.z * rows * cols;
  partial += (size_t)blockIdx.z * kColsumChunks * cols;
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int col = blockIdx.x * 256 + 4 * cx;
  const int per = (rows + kColsumChunks - 1) / kColsumChunks;
  const int rbeg = blockIdx.y * per, rend = min(rows, rbeg + per);
  floatx4 s[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) s[u] = floatx4{0.f, 0.f, 0.f, 0.f};
  if (col < cols) {
    const float* const base = in + col;
    int r = rbeg + ry;
    for (; r + 12 < rend; r += 16) {
      floatx4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const floatx4*>(base + (long)(r + 4 * u) * cols);
#pragma unroll
      for (int u = 0; u < 4; ++u) s[u] += v[u];
    }
    for (; r < rend; r += 4) s[0] += *reinterpret_cast<const floatx4*>(base + (long)r * cols);
  }
  red[ry][cx] = (s[0] + s[1]) + (s[2] + s[3]);
  __syncthreads();
  if (ry == 0 && col < cols)
    *reinterpret_cast<floatx4*>(partial + (long)blockIdx.y * cols + col) = (red[0][cx] + red[1][cx]) + (red[2][cx] + red[3][cx]);
}
__global__ void colsum_final_kernel(const float* __restrict__ partial, int cols, float* __restrict__ out) {
  const int col = blockIdx.x * blockDim.x + threadIdx.x;
  if (col >= cols) return;
  partial += (size_t)blockIdx.y * kColsumChunks * cols;
  out += (size_t)blockIdx.y * cols;
  float s = 0.f;
  for (int k = 0; k < kColsumChunks; ++k) s += partial[(long)k * cols + col];
  out[col] = s;
}

__global__ void fill_zero_kernel(uint32_t* p, size_t n) {
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) p[e] = 0u;
}

inline int grid_for(long n, int block = 256, int cap = 4096) {
  long g = (n + block - 1) / block;
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return (int)g;
}

}  // namespace

hipError_t launch_ew(EwOp op, float* out, long ldo, const float* a, long lda, const float* b, long ldb, int rows,
                     int cols, hipStream_t stream) {
  hipLaunchKernelGGL(ew_kernel, dim3(grid_for((long)rows * cols)), dim3(256), 0, stream, (int)op, out, ldo, a, lda, b,
                     ldb, rows, cols);
  return hipGetLastError();
}

hipError_t launch_pointwise_fwd(const float* pre1, const float* pre2, const float* bias, const float* c_prev,
                                float* h_out, float* c_out, float* gates_out, float* h_out2, float* c_out2, int B,
                                int H, hipStream_t stream) {
  hipLaunchKernelGGL(pointwise_fwd_kernel, dim3(grid_for((long)B * H)), dim3(256), 0, stream, pre1, pre2, bias,
                     c_prev, h_out, c_out, gates_out, h_out2, c_out2, B, H);
  return hipGetLastError();
}

hipError_t launch_pointwise_bwd(const float* gates, const float* c_t, const float* c_prev, const float* dh_a,
                                const float* dh_b, const float* dc_in, float* dA, float* dc_out, int B, int H,
                                hipStream_t stream) {
  hipLaunchKernelGGL(pointwise_bwd_kernel, dim3(grid_for((long)B * H)), dim3(256), 0, stream, gates, c_t, c_prev,
                     dh_a, dh_b, dc_in, dA, dc_out, B, H);
  return hipGetLastError();
}

hipError_t launch_transpose(const float* in, float* out, int rows, int cols, int batch, hipStream_t stream) {
  hipLaunchKernelGGL(transpose_kernel, dim3((cols + 31) / 32, (rows + 31) / 32, batch), dim3(256), 0, stream, in, out,
                     rows, cols);
  return hipGetLastError();
}

hipError_t launch_colsum(const float* in, int rows, int cols, float* partial, float* out, hipStream_t stream) {
  return launch_colsum_batched(in, rows, cols, 1, partial, out, stream);
}

// `count` matrices [rows][cols] one after the other -> out [count][cols]; partial: count * 64 * cols floats.
hipError_t launch_colsum_batched(const float* in, int rows, int cols, int count, float* partial, float* out,
                                 hipStream_t stream) {
  const bool vec = cols % 4 == 0 && ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(partial)) & 15u) == 0;
  if (vec)
    hipLaunchKernelGGL(colsum_partial4_kernel, dim3((cols + 255) / 256, kColsumChunks, count), dim3(256), 0, stream, in,
                       rows, cols, partial);
  else
    hipLaunchKernelGGL(colsum_partial_kernel, dim3((cols + 63) / 64, kColsumChunks, count), dim3(256), 0, stream, in, rows,
                       cols, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colsum_final_kernel, dim3((cols + 255) / 256, count), dim3(256), 0, stream, partial, cols, out);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for((long)n, 256, 2048)), dim3(256), 0, stream,
                     reinterpret_cast<uint32_t*>(p), n);
  return hipGetLastError();
}

}  // namespace lstm
