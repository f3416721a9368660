// Cross-layer norm accumulation and clip factors (section 2.1 of the paper; all-layer
// clipping = one group, eq. (1) with M = 1).  A few hundred floats: one tiny launch.
#include "dp_internal.h"

namespace dpbk {

namespace {

__global__ void __launch_bounds__(256)
clip_factor_kernel(const float* __restrict__ sqnorm, int L, int B, int mode, float R,
                   float stability, float* __restrict__ C_out, float* __restrict__ norm_out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B) return;
  float total = 0.f;
  for (int l = 0; l < L; ++l) total += sqnorm[(size_t)l * B + i];   // fixed order: deterministic
  const float norm = __builtin_sqrtf(fmaxf(total, 0.f));
  float c;
  if (mode == DP_CLIP_STANDARD)
    c = fminf(R / norm, 1.f);          // norm == 0: R/0 = +inf -> 1
  else
    c = R / (norm + stability);
  C_out[i] = c;
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

__global__ void __launch_bounds__(256)
clip_factor_grouped_kernel(const float* __restrict__ sqnorm, int B, int mode, float stability,
                           float* __restrict__ C_out, float* __restrict__ norm_out,
                           const GroupedClipArgs ga) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int m = blockIdx.y;
  if (i >= B) return;
  float total = 0.f;
  for (int l = ga.begin[m]; l < ga.begin[m + 1]; ++l) total += sqnorm[(size_t)l * B + i];
  const float norm = __builtin_sqrtf(fmaxf(total, 0.f));
  const float R = ga.R[m];
  const float c = mode == DP_CLIP_STANDARD ? fminf(R / norm, 1.f) : R / (norm + stability);
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
    hipLaunchKernelGGL(clip_factor_grouped_kernel, dim3((B + 255) / 256, ga.n_groups), dim3(256), 0, s,
                       sqnorm, B, mode, stability, C_out, norm_out, ga);
    if (hipGetLastError() != hipSuccess) return DP_ERR_HIP;
  }
  return DP_OK;
}

dp_status launch_clip_factors(const float* sqnorm, int L, int B, int mode, float R, float stability,
                              float* C_out, float* norm_out, hipStream_t s) {
  hipLaunchKernelGGL(clip_factor_kernel, dim3((B + 255) / 256), dim3(256), 0, s, sqnorm, L, B, mode,
                     R, stability, C_out, norm_out);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
