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

}  // namespace

dp_status launch_clip_factors(const float* sqnorm, int L, int B, int mode, float R, float stability,
                              float* C_out, float* norm_out, hipStream_t s) {
  hipLaunchKernelGGL(clip_factor_kernel, dim3((B + 255) / 256), dim3(256), 0, s, sqnorm, L, B, mode,
                     R, stability, C_out, norm_out);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
