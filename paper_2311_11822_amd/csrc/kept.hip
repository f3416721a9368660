// Clip-weighted gradient of layers whose per-sample gradients were kept by the instantiated-norm
// kernel (section 3 of the paper, "DP gradient", for layers on the left side of appendix A.1's
// eq. "mixed ghost norm"):
//     grad[e] (+)= sum_i C_i G_i[e]  (+ sigma R z_e, eq. (1)),     G_i = a_i^T g_i as kept, [B, d_in * d_out] fp32.
// A stream over B + 1 arrays of d_in * d_out floats (HBM-bound) in place of a second contraction over
// the T tokens of a and g.  Samples are added in index order; samples with C_i == 0 are not read.
#include "dp_internal.h"

namespace dpbk {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4v;
constexpr int kPerBlock = 1024;                 // elements per workgroup: 256 threads x one float4

// GroupLayer fields as used here: a = kept gradients [B, n], out = grad [n], d_in * d_out = n (a
// multiple of 4), tile_begin = first workgroup of the layer, c_off = the layer's row of C.
// na.layer_off[l] == ~0: no noise for that layer in this kernel.
__global__ void __launch_bounds__(256)
kept_weighted_sum_kernel(const GroupArgs ga, const float* __restrict__ C_all, const NoiseArgs na) {
  const int l = layer_of(ga, blockIdx.x);
  const GroupLayer& ly = ga.layer[l];
  const int n = ly.d_in * ly.d_out;
  const int e = ((blockIdx.x - ly.tile_begin) * 256 + threadIdx.x) * 4;
  if (e >= n) return;
  const float* __restrict__ C = C_all + ly.c_off;
  const float* src = static_cast<const float*>(ly.a) + e;
  f32x4v v = {0.f, 0.f, 0.f, 0.f};
  for (int i = 0; i < ga.B; ++i) {
    const float c = C[i];
    if (c == 0.f) continue;
    const f32x4v x = *reinterpret_cast<const f32x4v*>(src + (size_t)i * n);
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = fmaf(c, x[k], v[k]);
  }
  f32x4v* dst = reinterpret_cast<f32x4v*>(ly.out + e);
  if (ga.accumulate) {
    const f32x4v old = *dst;
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] += old[k];
  }
  const uint64_t off = na.layer_off[l];
  if (na.stddev != 0.f && off != ~(uint64_t)0) {
    const uint64_t idx = off + (uint64_t)e;                // a multiple of 4: one generator block
    if (idx + 4 > na.lo && idx < na.hi) {
      float z[4];
      normal_block(idx >> 2, na.step_lo, na.step_hi, na.rk, z);
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (idx + k >= na.lo && idx + k < na.hi) v[k] = fmaf(na.stddev, z[k], v[k]);
    }
  }
  *dst = v;
}

}  // namespace

int kept_blocks(int d, int p) { return (int)(((int64_t)d * p + kPerBlock - 1) / kPerBlock); }

dp_status launch_kept_weighted_sum(const GroupArgs& ga, const float* C, const NoiseArgs& na, hipStream_t s) {
  hipLaunchKernelGGL(kept_weighted_sum_kernel, dim3(ga.total_blocks), dim3(256), 0, s, ga, C, na);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
