// fp32-input forms of the three contractions, for small layers (the tiny all-fp32
// configuration).  Plain vector-ALU code: these shapes are launch-latency bound, so there
// is nothing for the matrix cores to win.  Reductions run in a fixed order (no atomics).
// The norm kernels run one workgroup per sample, so they are meant for layers of a few
// thousand elements; the host side refuses fp32 layers beyond kF32MaxWork multiply-adds per
// sample (DP_ERR_UNSUPPORTED) rather than run for seconds.
#include "dp_internal.h"

namespace dpbk {

namespace {

constexpr int kThreads = 256;

// Sum over the workgroup in a fixed order; result valid in thread 0.
__device__ float block_sum(float v) {
  __shared__ float red[kThreads];
  red[threadIdx.x] = v;
  __syncthreads();
  for (int w = kThreads / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  return red[0];
}

// Ghost norm (appendix A.1): sum over token pairs of (a_t . a_t')(g_t . g_t'); one workgroup per sample.
__global__ void __launch_bounds__(kThreads)
ghost_f32_kernel(const float* __restrict__ a, const float* __restrict__ g, int T, int d, int p,
                 float* __restrict__ out) {
  const int i = blockIdx.x;
  const float* ai = a + (size_t)i * T * d;
  const float* gi = g + (size_t)i * T * p;
  float acc = 0.f;
  const long pairs = (long)T * T;
  for (long q = threadIdx.x; q < pairs; q += kThreads) {
    const int t = (int)(q / T), u = (int)(q % T);
    if (u < t) continue;                       // Gram matrices are symmetric
    float da = 0.f, dg = 0.f;
    for (int k = 0; k < d; ++k) da = fmaf(ai[(size_t)t * d + k], ai[(size_t)u * d + k], da);
    for (int k = 0; k < p; ++k) dg = fmaf(gi[(size_t)t * p + k], gi[(size_t)u * p + k], dg);
    acc += (u == t ? 1.f : 2.f) * da * dg;
  }
  const float total = block_sum(acc);
  if (threadIdx.x == 0) out[i] = total;
}

// Instantiated norm (appendix A.1): || a_i^T g_i ||_F^2; one workgroup per sample.
__global__ void __launch_bounds__(kThreads)
perex_f32_kernel(const float* __restrict__ a, const float* __restrict__ g, int T, int d, int p,
                 float* __restrict__ out) {
  const int i = blockIdx.x;
  const float* ai = a + (size_t)i * T * d;
  const float* gi = g + (size_t)i * T * p;
  float acc = 0.f;
  const long cells = (long)d * p;
  for (long q = threadIdx.x; q < cells; q += kThreads) {
    const int j = (int)(q / p), k = (int)(q % p);
    float s = 0.f;
    for (int t = 0; t < T; ++t) s = fmaf(ai[(size_t)t * d + j], gi[(size_t)t * p + k], s);
    acc = fmaf(s, s, acc);
  }
  const float total = block_sum(acc);
  if (threadIdx.x == 0) out[i] = total;
}

// Clip-weighted gradient (section 3): grad[j,k] = sum_i C_i sum_t a[i,t,j] g[i,t,k].
__global__ void __launch_bounds__(kThreads)
clipped_grad_f32_kernel(const float* __restrict__ a, const float* __restrict__ g, int B, int T,
                        int d, int p, const float* __restrict__ C, float* __restrict__ grad,
                        int accumulate) {
  const long q = (long)blockIdx.x * kThreads + threadIdx.x;
  if (q >= (long)d * p) return;
  const int j = (int)(q / p), k = (int)(q % p);
  float total = 0.f;
  for (int i = 0; i < B; ++i) {
    if (C[i] == 0.f) continue;                 // a masked sample is not read, as in the 16-bit kernels
    const float* ai = a + (size_t)i * T * d;
    const float* gi = g + (size_t)i * T * p;
    float s = 0.f;
    for (int t = 0; t < T; ++t) s = fmaf(ai[(size_t)t * d + j], gi[(size_t)t * p + k], s);
    total = fmaf(C[i], s, total);
  }
  grad[q] = accumulate ? grad[q] + total : total;
}

}  // namespace

dp_status launch_ghost_f32(const float* a, const float* g, int B, int T, int d, int p, float* out,
                           hipStream_t s) {
  hipLaunchKernelGGL(ghost_f32_kernel, dim3(B), dim3(kThreads), 0, s, a, g, T, d, p, out);
  return hip_status(hipGetLastError());
}

dp_status launch_perex_f32(const float* a, const float* g, int B, int T, int d, int p, float* out,
                           hipStream_t s) {
  hipLaunchKernelGGL(perex_f32_kernel, dim3(B), dim3(kThreads), 0, s, a, g, T, d, p, out);
  return hip_status(hipGetLastError());
}

dp_status launch_clipped_grad_f32(const float* a, const float* g, int B, int T, int d, int p,
                                  const float* C, float* grad, int accumulate, hipStream_t s) {
  const long cells = (long)d * p;
  hipLaunchKernelGGL(clipped_grad_f32_kernel, dim3((unsigned)((cells + kThreads - 1) / kThreads)),
                     dim3(kThreads), 0, s, a, g, B, T, d, p, C, grad, accumulate);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
