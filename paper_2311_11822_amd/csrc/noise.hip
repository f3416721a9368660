// Gaussian mechanism on a contiguous gradient shard (eq. (1) of the paper, one group):
// grad[e] += sigma*R * z_e with z_e from Philox4x32-10 (Salmon et al., SC'11) + Box-Muller.
//
// The pass is a stream over fp32 memory (4 B read + 4 B written per element), so the
// kernel is built to stay under the HBM time: one thread owns one 128-bit Philox block
// = one float4 of gradient, the round keys are wave-uniform (kernel arguments, scalar
// registers), each 32x32->64 multiply is a single 64-bit multiply, and log2 / sin / cos
// use the hardware units (sin and cos take their argument in revolutions, which is
// exactly the uniform variate; measured absolute error 1.3e-7, log2 relative 1.2e-7).
#include "dp_internal.h"
#include "philox.h"

namespace dpbk {

namespace {

// Blocks [first_block, first_block + n_blocks) of the element stream.  `base` points at the
// element 4*first_block (it may lie before the caller's slice; lanes outside [lo, hi) neither
// load nor store).  VEC: base is 16-byte aligned, so whole blocks move as float4.
template <bool VEC>
__global__ void __launch_bounds__(256)
noise_kernel(float* __restrict__ base, uint64_t first_block, uint64_t n_blocks, uint64_t lo,
             uint64_t hi, float stddev, uint32_t step_lo, uint32_t step_hi, RoundKeys rk) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; j < n_blocks; j += stride) {
    uint32_t x[4];
    philox_block(first_block + j, step_lo, step_hi, rk, x);
    float z[4];
    box_muller(x[0], x[1], z[0], z[1]);
    box_muller(x[2], x[3], z[2], z[3]);
    const uint64_t e0 = 4 * j;   // element index relative to base
    float* p = base + e0;
    if (VEC && e0 >= lo && e0 + 4 <= hi) {
      float4 v = *reinterpret_cast<float4*>(p);
      v.x = fmaf(stddev, z[0], v.x);
      v.y = fmaf(stddev, z[1], v.y);
      v.z = fmaf(stddev, z[2], v.z);
      v.w = fmaf(stddev, z[3], v.w);
      *reinterpret_cast<float4*>(p) = v;
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (e0 + q >= lo && e0 + q < hi) p[q] = fmaf(stddev, z[q], p[q]);
    }
  }
}

// Whole, 16-byte aligned blocks [j0, j1) of the stream starting at `base`: the bulk of a shard.
// Four independent blocks per thread and iteration, loaded before any arithmetic, and
// streaming (non-temporal) accesses: the gradient is touched once, so it should not displace
// anything in the caches.  Measured on a 2.8 GB buffer: 5.2-5.5 TB/s for a bare read-modify-
// write pass with this access pattern against 4.6-4.8 TB/s for one block per iteration.
typedef __attribute__((ext_vector_type(4))) float f32x4v;
__global__ void __launch_bounds__(256)
noise_bulk_kernel(float* __restrict__ base, uint64_t first_block, uint64_t j0, uint64_t j1,
                  float stddev, uint32_t step_lo, uint32_t step_hi, RoundKeys rk) {
  constexpr int U = 4;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  f32x4v* p = reinterpret_cast<f32x4v*>(base);
  uint64_t j = j0 + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; j + (U - 1) * stride < j1; j += U * stride) {
    f32x4v v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(p + j + u * stride);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      uint32_t x[4];
      philox_block(first_block + j + u * stride, step_lo, step_hi, rk, x);
      float z[4];
      box_muller(x[0], x[1], z[0], z[1]);
      box_muller(x[2], x[3], z[2], z[3]);
#pragma unroll
      for (int q = 0; q < 4; ++q) v[u][q] = fmaf(stddev, z[q], v[u][q]);
      __builtin_nontemporal_store(v[u], p + j + u * stride);
    }
  }
  for (; j < j1; j += stride) {
    uint32_t x[4];
    philox_block(first_block + j, step_lo, step_hi, rk, x);
    float z[4];
    box_muller(x[0], x[1], z[0], z[1]);
    box_muller(x[2], x[3], z[2], z[3]);
    f32x4v v = p[j];
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = fmaf(stddev, z[q], v[q]);
    p[j] = v;
  }
}

__global__ void __launch_bounds__(256)
philox_dump_kernel(uint4* __restrict__ out, uint64_t first_block, uint64_t n_blocks,
                   uint32_t step_lo, uint32_t step_hi, RoundKeys rk) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; j < n_blocks; j += stride) {
    uint32_t x[4];
    philox_block(first_block + j, step_lo, step_hi, rk, x);
    out[j] = make_uint4(x[0], x[1], x[2], x[3]);
  }
}

int stream_grid(uint64_t n_blocks) {
  // 256 compute units x 8 resident workgroups; fewer when the slice is small.
  uint64_t want = (n_blocks + 255) / 256;
  if (want > 2048 * 4) want = 2048 * 4;
  return want < 1 ? 1 : (int)want;
}

}  // namespace

dp_status launch_noise(float* grad, uint64_t global_offset, uint64_t count, float stddev,
                       uint64_t seed, uint64_t step, hipStream_t s) {
  const uint64_t first_block = global_offset >> 2;
  const uint64_t last_block = (global_offset + count - 1) >> 2;
  const uint64_t n_blocks = last_block - first_block + 1;
  const uint64_t lead = global_offset - 4 * first_block;   // elements of the first block before the slice
  float* base = grad - lead;                               // never dereferenced below index `lead`
  const bool vec = (reinterpret_cast<uintptr_t>(base) & 15u) == 0;
  const RoundKeys rk = make_round_keys(seed);
  const dim3 grid(stream_grid(n_blocks)), block(256);
  const uint32_t step_lo = (uint32_t)step, step_hi = (uint32_t)(step >> 32);
  if (vec) {
    // whole blocks [j0, j1) in bulk; the partial first / last block through the general kernel
    const uint64_t j0 = lead ? 1 : 0, j1 = (lead + count) >> 2;
    if (j1 > j0) {
      // One workgroup per 1024 blocks, so that a thread makes a single pass of four blocks: measured
      // on 2.8 GB, 5.9 TB/s against 5.45 TB/s for a grid capped at 16384 workgroups whose threads
      // loop (0.9 GB: 6.3 against 5.9 TB/s; two or eight blocks per thread were slower).  Beyond
      // 2^22 workgroups (16 G elements) the threads loop.
      uint64_t want = (j1 - j0 + 1023) / 1024;
      const dim3 bulk_grid((unsigned)(want > (1u << 22) ? (1u << 22) : want));
      hipLaunchKernelGGL(noise_bulk_kernel, bulk_grid, block, 0, s, base, first_block, j0, j1, stddev,
                         step_lo, step_hi, rk);
      if (hipGetLastError() != hipSuccess) return DP_ERR_HIP;
    }
    if (j0 == 1)
      hipLaunchKernelGGL(noise_kernel<false>, dim3(1), dim3(64), 0, s, base, first_block, (uint64_t)1, lead,
                         lead + count, stddev, step_lo, step_hi, rk);
    if (j1 < n_blocks && !(j0 == 1 && n_blocks == 1))
      hipLaunchKernelGGL(noise_kernel<false>, dim3(1), dim3(64), 0, s, base + 4 * j1, first_block + j1,
                         n_blocks - j1, (uint64_t)0, lead + count - 4 * j1, stddev, step_lo, step_hi, rk);
  } else
    hipLaunchKernelGGL(noise_kernel<false>, grid, block, 0, s, base, first_block, n_blocks, lead,
                       lead + count, stddev, (uint32_t)step, (uint32_t)(step >> 32), rk);
  return hip_status(hipGetLastError());
}

dp_status launch_philox_blocks(uint32_t* out, uint64_t first_block, uint64_t n_blocks,
                               uint64_t seed, uint64_t step, hipStream_t s) {
  const RoundKeys rk = make_round_keys(seed);
  hipLaunchKernelGGL(philox_dump_kernel, dim3(stream_grid(n_blocks)), dim3(256), 0, s,
                     reinterpret_cast<uint4*>(out), first_block, n_blocks, (uint32_t)step,
                     (uint32_t)(step >> 32), rk);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
