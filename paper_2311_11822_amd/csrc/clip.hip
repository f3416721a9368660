// Cross-layer norm accumulation and clip factors (section 2.1 of the paper; all-layer
// clipping = one group, eq. (1) with M = 1).  A few hundred floats: one tiny launch.
#include "dp_internal.h"

namespace dpbk {

namespace {

// Sum of rows [l0, l1) of sqnorm at column i, by one wave: each lane adds a strided subset in
// order, then a fixed butterfly, so the result is deterministic; the rows are loaded in
// parallel (a serial loop would pay one memory latency per layer).
__device__ __forceinline__ float column_sum(const float* __restrict__ sqnorm, int B, int i, int l0, int l1) {
  float total = 0.f;
  for (int l = l0 + (int)threadIdx.x; l < l1; l += 64) total += sqnorm[(size_t)l * B + i];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) total += __shfl_xor(total, off);
  return total;
}

// Clip factor of one (sample, group) from its norm (section 2.1).  A NaN norm gives a NaN
// factor, so a sample whose gradient is not a number shows in the result instead of passing
// unclipped (fminf would drop the NaN).  Automatic clipping with norm + stability == 0 (a zero
// gradient and no stability constant) gives 0 rather than R/0: the sample adds nothing under any
// weight, and an infinite weight would turn its zero gradient into NaN.
__device__ __forceinline__ float clip_factor(float norm, int mode, float R, float stability) {
  if (norm != norm) return norm;
  if (mode == DP_CLIP_STANDARD) return fminf(R / norm, 1.f);     // norm == 0: R/0 = +inf -> 1
  const float den = norm + stability;
  return den > 0.f ? R / den : 0.f;
}

__global__ void __launch_bounds__(64)
clip_factor_kernel(const float* __restrict__ sqnorm, int L, int B, int mode, float R,
                   float stability, float* __restrict__ C_out, float* __restrict__ norm_out) {
  const int i = blockIdx.x;                                  // one wave per sample
  const float total = column_sum(sqnorm, B, i, 0, L);
  if (threadIdx.x != 0) return;
  const float norm = total != total ? total : __builtin_sqrtf(fmaxf(total, 0.f));   // fmaxf drops a NaN
  C_out[i] = clip_factor(norm, mode, R, stability);
  if (norm_out) norm_out[i] = norm;
}

// Group-wise clipping (eq. (1) with M groups): group m owns the rows
// [begin[m], begin[m+1]) of sqnorm and has threshold R[m].  Up to kGroupsPerLaunch groups
// travel in the kernel arguments.
constexpr int kGroupsPerLaunch = 256;
struct GroupedClipArgs {
  int n_groups;
  int first_group;
  int begin[kGroupsPerLaunch + 1];
  float R[kGroupsPerLaunch];
};

__global__ void __launch_bounds__(64)
clip_factor_grouped_kernel(const float* __restrict__ sqnorm, int B, int mode, float stability,
                           float* __restrict__ C_out, float* __restrict__ norm_out,
                           const GroupedClipArgs ga) {
  const int i = blockIdx.x, m = blockIdx.y;                  // one wave per (sample, group)
  const float total = column_sum(sqnorm, B, i, ga.begin[m], ga.begin[m + 1]);
  if (threadIdx.x != 0) return;
  const float norm = total != total ? total : __builtin_sqrtf(fmaxf(total, 0.f));   // fmaxf drops a NaN
  const float c = clip_factor(norm, mode, ga.R[m], stability);
  const size_t o = (size_t)(ga.first_group + m) * B + i;
  C_out[o] = c;
  if (norm_out) norm_out[o] = norm;
}

}  // namespace

dp_status launch_clip_factors_grouped(const float* sqnorm, int B, const int32_t* group_begin, int M,
                                      const float* R, int mode, float stability, float* C_out,
                                      float* norm_out, hipStream_t s) {
  for (int first = 0; first < M; first += kGroupsPerLaunch) {
    GroupedClipArgs ga;
    ga.n_groups = M - first < kGroupsPerLaunch ? M - first : kGroupsPerLaunch;
    ga.first_group = first;
    for (int m = 0; m <= ga.n_groups; ++m) ga.begin[m] = group_begin[first + m];
    for (int m = 0; m < ga.n_groups; ++m) ga.R[m] = R[first + m];
    hipLaunchKernelGGL(clip_factor_grouped_kernel, dim3(B, ga.n_groups), dim3(64), 0, s,
                       sqnorm, B, mode, stability, C_out, norm_out, ga);
    if (hipGetLastError() != hipSuccess) return DP_ERR_HIP;
  }
  return DP_OK;
}

dp_status launch_clip_factors(const float* sqnorm, int L, int B, int mode, float R, float stability,
                              float* C_out, float* norm_out, hipStream_t s) {
  hipLaunchKernelGGL(clip_factor_kernel, dim3(B), dim3(64), 0, s, sqnorm, L, B, mode,
                     R, stability, C_out, norm_out);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
