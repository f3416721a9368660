// bf16 matrix-core kernels for the two contractions over the token axis:
//
//   clip-weighted gradient (section 3 of the paper, "DP gradient"):
//       grad[j,k] = sum_i C_i sum_t a[i,t,j] g[i,t,k]
//   instantiated per-sample norm (appendix A.1, left side of eq. "mixed ghost norm"):
//       sqnorm[i] = sum_{j,k} ( sum_t a[i,t,j] g[i,t,k] )^2
//
// Both are "TN" products: the contraction runs over the slow (token) axis of two
// row-major operands.  The MFMA wants each lane to hold 8 consecutive k of one row, so
// tiles are staged in LDS as [k][m] exactly as they lie in memory and fetched with the
// gfx950 transposing LDS read (tile machinery in tn_tile.h).
//
// The gradient keeps one accumulator set re-expressed at sample boundaries (tn_tile.h): the
// register file cannot hold two at these tile sizes, and the re-expression adds only B fp32
// roundings per output.
#include "dp_internal.h"
#include "tile_order.h"
#include "tn_tile.h"

namespace dpbk {

namespace {

__device__ __forceinline__ int find_layer(const GroupArgs& ga, int block) { return layer_of(ga, block); }

// ---------------------------------------------------------------------------------
// Clip-weighted gradient, grouped over layers.
// ---------------------------------------------------------------------------------
template <class S, bool F16>
__global__ void __launch_bounds__(S::NT)
clipped_grad_kernel(const GroupArgs ga, const float* __restrict__ C_all) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const int l = find_layer(ga, blockIdx.x);
  const GroupLayer& ly = ga.layer[l];
  const int local = blockIdx.x - ly.tile_begin;
  const int tiles_n = (ly.d_out + S::BN - 1) / S::BN;
  const float* __restrict__ C = C_all + ly.c_off;      // the layer's clipping group
  clipped_grad_tile<S, F16>(ly, ga.B, ga.accumulate, (local / tiles_n) * S::BM, (local % tiles_n) * S::BN, C,
                       lds);
}

// ---------------------------------------------------------------------------------
// Instantiated per-sample norm, grouped over layers: one workgroup per (sample, tile).
// ---------------------------------------------------------------------------------
template <class S, bool F16>
__global__ void __launch_bounds__(S::NT)
perex_norm_kernel(const GroupArgs ga, float* __restrict__ partials) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  // The tiles of one (layer, sample) read the same panels of a_i and g_i: numbered consecutively
  // and dealt to the XCDs in contiguous eighths, they share them through one L2.
  const int item = contiguous_eighth(blockIdx.x, ga.total_blocks);
  const int l = find_layer(ga, item);
  const GroupLayer& ly = ga.layer[l];
  const int local = item - ly.tile_begin;
  const int sample = local / ly.tiles_per_sample;
  const int tile = local % ly.tiles_per_sample;
  const int tiles_n = (ly.d_out + S::BN - 1) / S::BN;

  TnTile<S> t;
  t.a = static_cast<const uint16_t*>(ly.a);
  t.g = static_cast<const uint16_t*>(ly.g);
  t.T = ly.T;
  t.d = ly.d_in;
  t.p = ly.d_out;
  t.m0 = (tile / tiles_n) * S::BM;
  t.n0 = (tile % tiles_n) * S::BN;
  const int nkb = (ly.T + S::BK - 1) / S::BK;

  f32x16 acc[S::TM][S::TN];
  zero_acc<S>(acc);
  t.gload(sample, 0);
  t.lds_store(lds);
  __syncthreads();
  for (int kb = 0, stage = 0; kb < nkb; ++kb, stage ^= 1) {
    const bool more = kb + 1 < nkb;
    if (more) t.gload(sample, kb + 1);
    t.template compute<F16>(lds + stage * S::STAGE, acc);
    if (more) t.lds_store(lds + (stage ^ 1) * S::STAGE);
    __syncthreads();
  }

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Book-keeping of the instantiated gradient (appendix A.2 applied to this path): when the
  // caller provides room, the tile of a_i^T g_i is kept, and the clip-weighted gradient is later
  // formed as sum_i C_i G_i from these copies instead of a second pass over a and g.
  if (ly.out) {
    float* dst = ly.out + (size_t)sample * ly.d_in * ly.d_out;
    const int wm = (wave / S::WN) * S::WTM, wn = (wave % S::WN) * S::WTN;
#pragma unroll
    for (int im = 0; im < S::TM; ++im)
#pragma unroll
      for (int jn = 0; jn < S::TN; ++jn) {
        const int col = t.n0 + wn + jn * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = t.m0 + wm + im * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (row < t.d && col < t.p) dst[(size_t)row * t.p + col] = acc[im][jn][r];
        }
      }
  }

  // Rows/columns past the layer's edge were loaded as zeros, so they add nothing.
  float s = 0.f;
#pragma unroll
  for (int im = 0; im < S::TM; ++im)
#pragma unroll
    for (int jn = 0; jn < S::TN; ++jn)
#pragma unroll
      for (int r = 0; r < 16; ++r) s = fmaf(acc[im][jn][r], acc[im][jn][r], s);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  float* red = reinterpret_cast<float*>(lds);    // all LDS reads finished at the last barrier
  if (lane == 0) red[wave] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float total = 0.f;
    for (int w = 0; w < S::WM * S::WN; ++w) total += red[w];
    partials[ly.part_begin + local] = total;
  }
}

// sqnorm[l, i] = sum of the layer's per-tile partials of sample i, in tile order.
__global__ void __launch_bounds__(64)
norm_reduce_kernel(const GroupArgs ga, const float* __restrict__ partials, float* __restrict__ sqnorm) {
  const int l = blockIdx.x / ga.B, i = blockIdx.x % ga.B;
  const GroupLayer& ly = ga.layer[l];
  const float* src = partials + ly.part_begin + (size_t)i * ly.tiles_per_sample;
  // 64 lanes each add a strided subset in order, then a fixed butterfly: deterministic.
  float s = 0.f;
  for (int q = threadIdx.x; q < ly.tiles_per_sample; q += 64) s += src[q];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  if (threadIdx.x == 0) sqnorm[(size_t)ly.sq_index * ga.B + i] = s;
}

// Tile shapes.  Gradient: 256x256 output tile, 8 waves of 128x64, k-step 32.
// Per-sample norm: long-sequence layers are small in d x p, so use 128x128 tiles / 4 waves; k-step 64
// (one barrier per 16 MFMAs of a wave: measured 15 % faster than k-step 32 on T = 4096 layers).
#ifndef DP_GRAD_SHAPE
#define DP_GRAD_SHAPE 256, 256, 32, 2, 4
#endif
using GradShape = TnShape<DP_GRAD_SHAPE>;
using PerexShape = TnShape<128, 128, 64, 2, 2>;

}  // namespace

int perex_tiles_per_sample(int d, int p) {
  return ((d + PerexShape::BM - 1) / PerexShape::BM) * ((p + PerexShape::BN - 1) / PerexShape::BN);
}

int clipped_grad_tiles(int d, int p) {
  return ((d + GradShape::BM - 1) / GradShape::BM) * ((p + GradShape::BN - 1) / GradShape::BN);
}

template <bool F16>
dp_status launch_clipped_grad_group_t(const GroupArgs& ga, const float* C, hipStream_t s) {
  auto kernel = clipped_grad_kernel<GradShape, F16>;
  static ReadyTable ready;
  dp_status st = allow_big_lds(kernel, (int)GradShape::LDS_BYTES, ready);
  if (st != DP_OK) return st;
  hipLaunchKernelGGL(kernel, dim3(ga.total_blocks), dim3(GradShape::NT), GradShape::LDS_BYTES, s, ga, C);
  return hip_status(hipGetLastError());
}

template <bool F16>
dp_status launch_perex_group_t(const GroupArgs& ga, float* partials, hipStream_t s) {
  auto kernel = perex_norm_kernel<PerexShape, F16>;
  static ReadyTable ready;
  dp_status st = allow_big_lds(kernel, (int)PerexShape::LDS_BYTES, ready);
  if (st != DP_OK) return st;
  hipLaunchKernelGGL(kernel, dim3(ga.total_blocks), dim3(PerexShape::NT), PerexShape::LDS_BYTES, s, ga,
                     partials);
  return hip_status(hipGetLastError());
}

dp_status launch_clipped_grad_group(const GroupArgs& ga, const float* C, hipStream_t s) {
  return ga.f16 ? launch_clipped_grad_group_t<true>(ga, C, s) : launch_clipped_grad_group_t<false>(ga, C, s);
}

dp_status launch_perex_group(const GroupArgs& ga, float* partials, hipStream_t s) {
  return ga.f16 ? launch_perex_group_t<true>(ga, partials, s) : launch_perex_group_t<false>(ga, partials, s);
}

dp_status launch_norm_reduce_group(const GroupArgs& ga, const float* partials, float* sqnorm_out,
                                   hipStream_t s) {
  hipLaunchKernelGGL(norm_reduce_kernel, dim3(ga.n_layers * ga.B), dim3(64), 0, s, ga, partials,
                     sqnorm_out);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
