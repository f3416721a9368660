// Layer-wise clipping in one pass over a layer's a and g (section 3.3 (II) of the paper and the
// formula of its appendix on the hook-free implementation): with one clipping group per layer
// the factor C_{l,i} depends on layer l alone, so for a layer whose whole d_in x d_out gradient
// fits one workgroup tile the same kernel can instantiate G_i = a_i^T g_i (appendix A.1, left
// side of eq. "mixed ghost norm"), take its norm, turn it into C_i (section 2.1) and add
// C_i G_i to the running sum (section 3, "DP gradient") -- nothing is book-kept and a, g are read
// once.
//
// One workgroup owns (layer, chunk of consecutive samples).  Per sample it runs the token
// contraction of the instantiated-norm kernel (tn_tile.h machinery) into one accumulator set,
// reduces the sum of squares over the workgroup in a fixed order, and adds C_i times the
// accumulators to a second set.  The chunk's weighted sum goes to a workspace; a second small
// kernel adds the chunks in order, adds the noise of eq. (1) and writes the gradient.  No
// atomics: the result is deterministic.
#include "dp_internal.h"
#include "tn_tile.h"

namespace dpbk {

namespace {

// As in clip.hip: NaN norm -> NaN factor; automatic clipping with norm + stability == 0 -> 0.
__device__ __forceinline__ float clip_factor_of(float norm, int mode, float R, float stability) {
  if (norm != norm) return norm;
  if (mode == DP_CLIP_STANDARD) return fminf(R / norm, 1.f);
  const float den = norm + stability;
  return den > 0.f ? R / den : 0.f;
}

struct FusedArgs {
  int mode;
  float stability;
  float R[kMaxGroup];            // threshold of each layer of the launch
};

// GroupLayer fields as used here: tile_begin = first workgroup of the layer, tiles_per_sample =
// number of sample chunks, part_begin = float offset of the layer's [chunks][d_in * d_out]
// partial sums in the workspace, sq_index = row of sqnorm / C.
template <class S, bool F16>
__global__ void __launch_bounds__(S::NT)
layerwise_fused_kernel(const GroupArgs ga, const FusedArgs fa, float* __restrict__ partial,
                       float* __restrict__ sqnorm, float* __restrict__ C_out) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const int l = layer_of(ga, blockIdx.x);
  const GroupLayer& ly = ga.layer[l];
  const int chunk = blockIdx.x - ly.tile_begin;
  const int per = (ga.B + ly.tiles_per_sample - 1) / ly.tiles_per_sample;
  const int i0 = chunk * per, i1 = min(ga.B, i0 + per);

  TnTile<S> t;
  t.a = static_cast<const uint16_t*>(ly.a);
  t.g = static_cast<const uint16_t*>(ly.g);
  t.T = ly.T;
  t.d = ly.d_in;
  t.p = ly.d_out;
  t.m0 = 0;
  t.n0 = 0;
  const int nkb = (ly.T + S::BK - 1) / S::BK;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int NW = S::WM * S::WN;
  float* red = reinterpret_cast<float*>(lds);

  f32x16 total[S::TM][S::TN];
  zero_acc<S>(total);
  for (int i = i0; i < i1; ++i) {
    f32x16 acc[S::TM][S::TN];
    zero_acc<S>(acc);
    t.gload(i, 0);
    t.lds_store(lds);
    __syncthreads();
    for (int kb = 0, stage = 0; kb < nkb; ++kb, stage ^= 1) {
      const bool more = kb + 1 < nkb;
      if (more) t.gload(i, kb + 1);
      t.template compute<F16>(lds + stage * S::STAGE, acc);
      if (more) t.lds_store(lds + (stage ^ 1) * S::STAGE);
      __syncthreads();
    }
    // ||G_i||_F^2: rows and columns past the layer's edge were loaded as zeros and add nothing
    float s = 0.f;
#pragma unroll
    for (int im = 0; im < S::TM; ++im)
#pragma unroll
      for (int jn = 0; jn < S::TN; ++jn)
#pragma unroll
        for (int r = 0; r < 16; ++r) s = fmaf(acc[im][jn][r], acc[im][jn][r], s);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (lane == 0) red[wave] = s;                  // every LDS read of the loop is behind a barrier
    __syncthreads();
    float sq = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sq += red[w];     // same order in every thread
    __syncthreads();                               // red is overwritten by the next sample's tiles
    const float norm = sq != sq ? sq : __builtin_sqrtf(fmaxf(sq, 0.f));
    const float c = clip_factor_of(norm, fa.mode, fa.R[l], fa.stability);
    if (threadIdx.x == 0) {
      sqnorm[(size_t)ly.sq_index * ga.B + i] = sq;
      C_out[(size_t)ly.sq_index * ga.B + i] = c;
    }
    if (c != 0.f) {
#pragma unroll
      for (int im = 0; im < S::TM; ++im)
#pragma unroll
        for (int jn = 0; jn < S::TN; ++jn)
#pragma unroll
          for (int r = 0; r < 16; ++r) total[im][jn][r] = fmaf(c, acc[im][jn][r], total[im][jn][r]);
    }
  }

  // the chunk's weighted sum, [d_in, d_out] row-major
  const int wm = (wave / S::WN) * S::WTM, wn = (wave % S::WN) * S::WTN;
  float* out = partial + ly.part_begin + (size_t)chunk * ly.d_in * ly.d_out;
#pragma unroll
  for (int im = 0; im < S::TM; ++im)
#pragma unroll
    for (int jn = 0; jn < S::TN; ++jn) {
      const int col = wn + jn * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = wm + im * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < ly.d_in && col < ly.d_out) out[(size_t)row * ly.d_out + col] = total[im][jn][r];
      }
    }
}

// grad[e] (+)= sum over the layer's chunks, in chunk order, (+ noise of eq. (1) at the element's
// global index, the same values dp_add_noise draws).  blockIdx.y = layer of the launch.
__global__ void __launch_bounds__(256)
layerwise_reduce_kernel(const GroupArgs ga, const float* __restrict__ partial, const NoiseArgs na) {
  const GroupLayer& ly = ga.layer[blockIdx.y];
  const int n = ly.d_in * ly.d_out;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= n) return;
  const float* src = partial + ly.part_begin + e;
  float v = 0.f;
  for (int c = 0; c < ly.tiles_per_sample; ++c) v += src[(size_t)c * n];
  if (ga.accumulate) v += ly.out[e];
  if (na.stddev != 0.f) {
    const uint64_t idx = na.layer_off[blockIdx.y] + (uint64_t)e;
    if (idx >= na.lo && idx < na.hi) {
      float z[4];
      normal_block(idx >> 2, na.step_lo, na.step_hi, na.rk, z);
      const int k = (int)(idx & 3);
      v = fmaf(na.stddev, k == 0 ? z[0] : k == 1 ? z[1] : k == 2 ? z[2] : z[3], v);
    }
  }
  ly.out[e] = v;
}

// One workgroup tile holds the whole layer: 128 x 128, or a strip 512 x 32 / 32 x 512 (the
// shapes of low-rank adapter factors).
using FusedSquare = TnShape<128, 128, 64, 2, 2>;
using FusedTall = TnShape<512, 32, 64, 4, 1>;
using FusedWide = TnShape<32, 512, 64, 1, 4>;

template <class S, bool F16>
dp_status launch_fused_t(const GroupArgs& ga, const FusedArgs& fa, float* partial, float* sqnorm, float* C_out,
                         hipStream_t s) {
  auto kernel = layerwise_fused_kernel<S, F16>;
  static ReadyTable ready;
  dp_status st = allow_big_lds(kernel, (int)S::LDS_BYTES, ready);
  if (st != DP_OK) return st;
  hipLaunchKernelGGL(kernel, dim3(ga.total_blocks), dim3(S::NT), S::LDS_BYTES, s, ga, fa, partial, sqnorm, C_out);
  return hip_status(hipGetLastError());
}

}  // namespace

int layerwise_fused_shape(int d, int p) {
  if (d <= 128 && p <= 128) return 0;
  if (d <= 512 && p <= 32) return 1;
  if (d <= 32 && p <= 512) return 2;
  return -1;
}

dp_status launch_layerwise_fused(int shape, const GroupArgs& ga, const float* R, int mode, float stability,
                                 float* partial, float* sqnorm, float* C_out, hipStream_t s) {
  FusedArgs fa;
  fa.mode = mode;
  fa.stability = stability;
  for (int j = 0; j < ga.n_layers; ++j) fa.R[j] = R[j];
  for (int j = ga.n_layers; j < kMaxGroup; ++j) fa.R[j] = 1.f;
  switch (shape * 2 + (ga.f16 ? 1 : 0)) {
    case 0: return launch_fused_t<FusedSquare, false>(ga, fa, partial, sqnorm, C_out, s);
    case 1: return launch_fused_t<FusedSquare, true>(ga, fa, partial, sqnorm, C_out, s);
    case 2: return launch_fused_t<FusedTall, false>(ga, fa, partial, sqnorm, C_out, s);
    case 3: return launch_fused_t<FusedTall, true>(ga, fa, partial, sqnorm, C_out, s);
    case 4: return launch_fused_t<FusedWide, false>(ga, fa, partial, sqnorm, C_out, s);
    case 5: return launch_fused_t<FusedWide, true>(ga, fa, partial, sqnorm, C_out, s);
  }
  return DP_ERR_INVALID_ARG;
}

dp_status launch_layerwise_reduce(const GroupArgs& ga, const float* partial, const NoiseArgs& na, hipStream_t s) {
  int widest = 0;
  for (int j = 0; j < ga.n_layers; ++j) widest = std::max(widest, ga.layer[j].d_in * ga.layer[j].d_out);
  hipLaunchKernelGGL(layerwise_reduce_kernel, dim3((widest + 255) / 256, ga.n_layers), dim3(256), 0, s, ga,
                     partial, na);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
