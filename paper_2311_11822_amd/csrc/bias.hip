// Bias gradients (appendix A.1 of the paper, last paragraph): the per-sample bias gradient is
// 1^T dL/ds_i, the sum of sample i's T output-gradient rows; its norm is taken by
// instantiation.  The B x d_out matrix of these sums is tiny, so it is kept (book-keeping): the
// clipped bias gradient sum_i C_i 1^T g_i is then formed from it without reading g again.
// Both kernels are streams over memory (HBM-bound); sums run in a fixed order.
#include "dp_internal.h"

namespace dpbk {

namespace {

constexpr int kRowGroups = 16, kColThreads = 32;

// One workgroup: sample blockIdx.y, a strip of 32 * VEC columns.  Thread (rg, ct) adds rows
// rg, rg + 16, ... of its VEC columns; the 16 row groups are then added in order through LDS.
template <int DT>                       // dp_dtype of g
__global__ void __launch_bounds__(kRowGroups * kColThreads)
bias_colsum_kernel(const void* __restrict__ g_all, int T, int p, float* __restrict__ colsum) {
  constexpr bool HALF = DT != DP_F32;   // 16-bit storage: 8 columns per thread
  constexpr int VEC = HALF ? 8 : 1;
  __shared__ float red[kRowGroups][kColThreads * VEC + 1];
  const int ct = threadIdx.x % kColThreads, rg = threadIdx.x / kColThreads;
  const int i = blockIdx.y;
  const int col = (blockIdx.x * kColThreads + ct) * VEC;
  float acc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
  if (col < p) {
    if (HALF) {
      const uint16_t* g = static_cast<const uint16_t*>(g_all) + (size_t)i * T * p + col;
      auto add = [&](const uint4& w) {
        const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (DT == DP_BF16) {
            acc[2 * q] += __uint_as_float(u[q] << 16);             // bf16 -> fp32 is a shift
            acc[2 * q + 1] += __uint_as_float(u[q] & 0xFFFF0000u);
          } else {
            acc[2 * q] += (float)__builtin_bit_cast(_Float16, (uint16_t)(u[q] & 0xFFFFu));
            acc[2 * q + 1] += (float)__builtin_bit_cast(_Float16, (uint16_t)(u[q] >> 16));
          }
        }
      };
      // four rows in flight per thread; they are added in row order, so the sum does not depend
      // on the unrolling
      int t = rg;
      for (; t + 3 * kRowGroups < T; t += 4 * kRowGroups) {
        uint4 w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w[u] = *reinterpret_cast<const uint4*>(g + (size_t)(t + u * kRowGroups) * p);
#pragma unroll
        for (int u = 0; u < 4; ++u) add(w[u]);
      }
      for (; t < T; t += kRowGroups) add(*reinterpret_cast<const uint4*>(g + (size_t)t * p));
    } else {
      const float* g = static_cast<const float*>(g_all) + (size_t)i * T * p + col;
      for (int t = rg; t < T; t += kRowGroups) acc[0] += g[(size_t)t * p];
    }
  }
#pragma unroll
  for (int v = 0; v < VEC; ++v) red[rg][ct * VEC + v] = acc[v];
  __syncthreads();
  for (int c = threadIdx.x; c < kColThreads * VEC; c += kRowGroups * kColThreads) {
    const int out_col = blockIdx.x * kColThreads * VEC + c;
    if (out_col < p) {
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < kRowGroups; ++r) s += red[r][c];
      colsum[(size_t)i * p + out_col] = s;
    }
  }
}

// sqnorm[i] = sum_k colsum[i,k]^2; one workgroup per sample, fixed-order reduction.
__global__ void __launch_bounds__(256)
bias_sqnorm_kernel(const float* __restrict__ colsum, int p, float* __restrict__ sqnorm) {
  __shared__ float red[256];
  const float* row = colsum + (size_t)blockIdx.x * p;
  float s = 0.f;
  for (int k = threadIdx.x; k < p; k += 256) s = fmaf(row[k], row[k], s);
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) sqnorm[blockIdx.x] = red[0];
}

// grad_b[k] (+)= sum_i C_i colsum[i,k]
__global__ void __launch_bounds__(256)
clipped_bias_kernel(const float* __restrict__ colsum, int B, int p, const float* __restrict__ C,
                    float* __restrict__ grad_b, int accumulate) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= p) return;
  float s = 0.f;
  for (int i = 0; i < B; ++i) s = fmaf(C[i], colsum[(size_t)i * p + k], s);
  grad_b[k] = accumulate ? grad_b[k] + s : s;
}

}  // namespace

dp_status launch_bias_norm(const void* g, dp_dtype dt, int B, int T, int p, float* colsum,
                           float* sqnorm_out, hipStream_t s) {
  const int cols_per_block = kColThreads * (dt == DP_F32 ? 1 : 8);
  const dim3 grid((p + cols_per_block - 1) / cols_per_block, B), block(kRowGroups * kColThreads);
  if (dt == DP_BF16)
    hipLaunchKernelGGL(bias_colsum_kernel<DP_BF16>, grid, block, 0, s, g, T, p, colsum);
  else if (dt == DP_F16)
    hipLaunchKernelGGL(bias_colsum_kernel<DP_F16>, grid, block, 0, s, g, T, p, colsum);
  else
    hipLaunchKernelGGL(bias_colsum_kernel<DP_F32>, grid, block, 0, s, g, T, p, colsum);
  if (hipGetLastError() != hipSuccess) return DP_ERR_HIP;
  hipLaunchKernelGGL(bias_sqnorm_kernel, dim3(B), dim3(256), 0, s, colsum, p, sqnorm_out);
  return hip_status(hipGetLastError());
}

dp_status launch_clipped_bias_grad(const float* colsum, int B, int p, const float* C, float* grad_b,
                                   int accumulate, hipStream_t s) {
  hipLaunchKernelGGL(clipped_bias_kernel, dim3((p + 255) / 256), dim3(256), 0, s, colsum, B, p, C, grad_b,
                     accumulate);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
