// Counter-based Gaussian generator shared by the noise pass and by the gradient kernels that
// add the noise in their epilogue: Philox4x32-10 (Salmon et al., SC'11) + Box-Muller.
// Block k of the element stream (elements 4k .. 4k+3) has counter (k_lo, k_hi, step_lo,
// step_hi) and key (seed_lo, seed_hi); u = ((x >> 9) + 1/2) 2^-23;
// (z_4k, z_4k+1) = sqrt(-2 ln u(x0)) (cos, sin)(2 pi u(x1)), (z_4k+2, z_4k+3) likewise from
// (x2, x3).  log2 / sin / cos use the hardware units (sin and cos take their argument in
// revolutions, which is exactly the uniform variate; measured absolute error 1.3e-7, log2
// relative 1.2e-7).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dpbk {

constexpr uint32_t kMulA = 0xD2511F53u;
constexpr uint32_t kMulB = 0xCD9E8D57u;
constexpr uint32_t kWeylA = 0x9E3779B9u;
constexpr uint32_t kWeylB = 0xBB67AE85u;

struct RoundKeys {
  uint32_t k[10][2];
};

inline RoundKeys make_round_keys(uint64_t seed) {
  RoundKeys rk;
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  for (int r = 0; r < 10; ++r) {
    rk.k[r][0] = k0;
    rk.k[r][1] = k1;
    k0 += kWeylA;
    k1 += kWeylB;
  }
  return rk;
}

__device__ __forceinline__ void philox_block(uint64_t block, uint32_t step_lo, uint32_t step_hi,
                                             const RoundKeys& rk, uint32_t x[4]) {
  uint32_t c0 = (uint32_t)block, c1 = (uint32_t)(block >> 32), c2 = step_lo, c3 = step_hi;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t pa = (uint64_t)kMulA * c0;
    const uint64_t pb = (uint64_t)kMulB * c2;
    const uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ rk.k[r][0];
    const uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ rk.k[r][1];
    c1 = (uint32_t)pb;
    c3 = (uint32_t)pa;
    c0 = n0;
    c2 = n2;
  }
  x[0] = c0;
  x[1] = c1;
  x[2] = c2;
  x[3] = c3;
}

// u = ((x >> 9) + 1/2) * 2^-23: every step is exact in fp32.
__device__ __forceinline__ float to_uniform(uint32_t x) {
  return ((float)(x >> 9) + 0.5f) * 1.1920928955078125e-07f;
}

__device__ __forceinline__ void box_muller(uint32_t xa, uint32_t xb, float& z0, float& z1) {
  const float ua = to_uniform(xa), ub = to_uniform(xb);
  // -2 ln u = (-2 ln 2) log2 u
  const float r = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(ua));
  z0 = r * __builtin_amdgcn_cosf(ub);
  z1 = r * __builtin_amdgcn_sinf(ub);
}

// The four normals of one block.
__device__ __forceinline__ void normal_block(uint64_t block, uint32_t step_lo, uint32_t step_hi,
                                             const RoundKeys& rk, float z[4]) {
  uint32_t x[4];
  philox_block(block, step_lo, step_hi, rk, x);
  box_muller(x[0], x[1], z[0], z[1]);
  box_muller(x[2], x[3], z[2], z[3]);
}

}  // namespace dpbk
