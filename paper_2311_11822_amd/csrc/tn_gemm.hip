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
// gfx950 transposing LDS read (ds_read_b64_tr_b16): within 16 lanes, lanes 4e..4e+3 supply
// row k0+e (16 consecutive m), and lane L receives column m0+L for k0..k0+3.
//
// Per-sample weights never touch the bf16 operands.  The accumulator holds
// sum_{j<=i} (C_j / C_i) G_j while sample i is being added; crossing to the next sample
// multiplies it by C_i / C_{i+1} and the epilogue by the last C.  Samples with C == 0 are
// skipped.  This keeps one accumulator set (the register file cannot hold two at these
// tile sizes) and adds only B fp32 roundings per output.
#include "dp_internal.h"

namespace dpbk {

namespace {

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct TnShape {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
  static constexpr int NT = 64 * WM * WN;
  static constexpr int WTM = BM / WM, WTN = BN / WN;        // wave tile
  static constexpr int TM = WTM / 32, TN = WTN / 32;        // 32x32 MFMA tiles per wave
  // Row strides in elements: +32 (64 B) makes 4 consecutive k rows hit 4 different bank
  // groups for the transposing read.
  static constexpr int SA = BM + 32, SB = BN + 32;
  static constexpr int A_PER_T = BK * BM / 8 / NT, B_PER_T = BK * BN / 8 / NT;
  static constexpr int STAGE = BK * (SA + SB);              // elements per pipeline stage
  static constexpr size_t LDS_BYTES = 2 * STAGE * sizeof(uint16_t);
  static_assert(BK % 16 == 0 && WTM % 32 == 0 && WTN % 32 == 0, "tile shape");
  static_assert((BK * BM / 8) % NT == 0 && (BK * BN / 8) % NT == 0, "load split");
};

// 8 consecutive-k bf16 of column `col` starting at k row `row0` (see file header).
__device__ __forceinline__ bf16x8 read_frag_tr(const uint16_t* tile, int stride, int row0, int col0,
                                               int lane) {
  const int b = lane >> 4, s = lane & 15;
  const uint16_t* p = tile + (row0 + 8 * (b >> 1) + (s >> 2)) * stride + col0 + 16 * (b & 1) + 4 * (s & 3);
  union {
    s16x4 h[2];
    bf16x8 v;
  } u;
  u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(DP_LDS(s16x4, p));
  u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(DP_LDS(s16x4, p + 4 * stride));
  return u.v;
}

template <class S>
struct TnTile {
  const uint16_t* a;   // sample 0, row 0 of the layer's activation
  const uint16_t* g;
  int T, d, p;
  int m0, n0;          // tile origin in [d, p]

  uint4 ra[S::A_PER_T], rb[S::B_PER_T];

  __device__ __forceinline__ void gload(int sample, int kb) {
    const int tid = threadIdx.x;
    const size_t row_base = (size_t)sample * T;
#pragma unroll
    for (int j = 0; j < S::A_PER_T; ++j) {
      const int c = tid + j * S::NT;
      const int row = c / (S::BM / 8), col = (c % (S::BM / 8)) * 8;
      const int k = kb * S::BK + row;
      ra[j] = make_uint4(0, 0, 0, 0);
      if (k < T && m0 + col < d)
        ra[j] = *reinterpret_cast<const uint4*>(a + (row_base + k) * d + m0 + col);
    }
#pragma unroll
    for (int j = 0; j < S::B_PER_T; ++j) {
      const int c = tid + j * S::NT;
      const int row = c / (S::BN / 8), col = (c % (S::BN / 8)) * 8;
      const int k = kb * S::BK + row;
      rb[j] = make_uint4(0, 0, 0, 0);
      if (k < T && n0 + col < p)
        rb[j] = *reinterpret_cast<const uint4*>(g + (row_base + k) * p + n0 + col);
    }
  }

  __device__ __forceinline__ void lds_store(uint16_t* stage) const {
    const int tid = threadIdx.x;
    uint16_t* sa = stage;
    uint16_t* sb = stage + S::BK * S::SA;
#pragma unroll
    for (int j = 0; j < S::A_PER_T; ++j) {
      const int c = tid + j * S::NT;
      const int row = c / (S::BM / 8), col = (c % (S::BM / 8)) * 8;
      *reinterpret_cast<uint4*>(sa + row * S::SA + col) = ra[j];
    }
#pragma unroll
    for (int j = 0; j < S::B_PER_T; ++j) {
      const int c = tid + j * S::NT;
      const int row = c / (S::BN / 8), col = (c % (S::BN / 8)) * 8;
      *reinterpret_cast<uint4*>(sb + row * S::SB + col) = rb[j];
    }
  }

  __device__ __forceinline__ void compute(const uint16_t* stage, f32x16 (&acc)[S::TM][S::TN]) const {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave / S::WN) * S::WTM, wn = (wave % S::WN) * S::WTN;
    const uint16_t* sa = stage;
    const uint16_t* sb = stage + S::BK * S::SA;
#pragma unroll
    for (int ks = 0; ks < S::BK / 16; ++ks) {
      bf16x8 fa[S::TM], fb[S::TN];
#pragma unroll
      for (int i = 0; i < S::TM; ++i) fa[i] = read_frag_tr(sa, S::SA, ks * 16, wm + i * 32, lane);
#pragma unroll
      for (int j = 0; j < S::TN; ++j) fb[j] = read_frag_tr(sb, S::SB, ks * 16, wn + j * 32, lane);
#pragma unroll
      for (int i = 0; i < S::TM; ++i)
#pragma unroll
        for (int j = 0; j < S::TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }
};

template <class S>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[S::TM][S::TN]) {
#pragma unroll
  for (int i = 0; i < S::TM; ++i)
#pragma unroll
    for (int j = 0; j < S::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
}

template <class S>
__device__ __forceinline__ void scale_acc(f32x16 (&acc)[S::TM][S::TN], float f) {
#pragma unroll
  for (int i = 0; i < S::TM; ++i)
#pragma unroll
    for (int j = 0; j < S::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] *= f;
}

__device__ __forceinline__ int find_layer(const GroupArgs& ga, int block) {
  int l = 0;
  while (l + 1 < ga.n_layers && block >= ga.layer[l + 1].tile_begin) ++l;
  return l;
}

// ---------------------------------------------------------------------------------
// Clip-weighted gradient, grouped over layers.
// ---------------------------------------------------------------------------------
template <class S>
__global__ void __launch_bounds__(S::NT)
clipped_grad_kernel(const GroupArgs ga, const float* __restrict__ C_all) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const int l = find_layer(ga, blockIdx.x);
  const GroupLayer& ly = ga.layer[l];
  const int local = blockIdx.x - ly.tile_begin;
  const int tiles_n = (ly.d_out + S::BN - 1) / S::BN;
  const int B = ga.B;
  const float* __restrict__ C = C_all + ly.c_off;      // the layer's clipping group

  TnTile<S> t;
  t.a = static_cast<const uint16_t*>(ly.a);
  t.g = static_cast<const uint16_t*>(ly.g);
  t.T = ly.T;
  t.d = ly.d_in;
  t.p = ly.d_out;
  t.m0 = (local / tiles_n) * S::BM;
  t.n0 = (local % tiles_n) * S::BN;
  const int nkb = (ly.T + S::BK - 1) / S::BK;

  f32x16 acc[S::TM][S::TN];
  zero_acc<S>(acc);

  int i = 0;
  while (i < B && C[i] == 0.f) ++i;
  float held = 0.f;                       // weight the accumulator is currently expressed in
  if (i < B) {
    int kb = 0, stage = 0;
    held = C[i];
    t.gload(i, 0);
    t.lds_store(lds);
    __syncthreads();
    while (true) {
      int ni = i, nkb_next = kb + 1;
      if (nkb_next == nkb) {
        nkb_next = 0;
        ++ni;
        while (ni < B && C[ni] == 0.f) ++ni;
      }
      const bool more = ni < B;
      if (more) t.gload(ni, nkb_next);
      t.compute(lds + stage * S::STAGE, acc);
      if (more) t.lds_store(lds + (stage ^ 1) * S::STAGE);
      __syncthreads();
      if (!more) break;
      if (ni != i) {                      // next block starts another sample: re-express acc
        const float c = C[ni];
        scale_acc<S>(acc, held / c);
        held = c;
      }
      i = ni;
      kb = nkb_next;
      stage ^= 1;
    }
  }

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave / S::WN) * S::WTM, wn = (wave % S::WN) * S::WTN;
  float* out = ly.out;
#pragma unroll
  for (int im = 0; im < S::TM; ++im)
#pragma unroll
    for (int jn = 0; jn < S::TN; ++jn) {
      const int col = t.n0 + wn + jn * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = t.m0 + wm + im * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < t.d && col < t.p) {
          float* dst = out + (size_t)row * t.p + col;
          const float v = acc[im][jn][r] * held;
          *dst = ga.accumulate ? *dst + v : v;
        }
      }
    }
}

// ---------------------------------------------------------------------------------
// Instantiated per-sample norm, grouped over layers: one workgroup per (sample, tile).
// ---------------------------------------------------------------------------------
template <class S>
__global__ void __launch_bounds__(S::NT)
perex_norm_kernel(const GroupArgs ga, float* __restrict__ partials) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const int l = find_layer(ga, blockIdx.x);
  const GroupLayer& ly = ga.layer[l];
  const int local = blockIdx.x - ly.tile_begin;
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
    t.compute(lds + stage * S::STAGE, acc);
    if (more) t.lds_store(lds + (stage ^ 1) * S::STAGE);
    __syncthreads();
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
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
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
// Per-sample norm: long-sequence layers are small in d x p, so use 128x128 tiles / 4 waves.
#ifndef DP_GRAD_SHAPE
#define DP_GRAD_SHAPE 256, 256, 32, 2, 4
#endif
using GradShape = TnShape<DP_GRAD_SHAPE>;
using PerexShape = TnShape<128, 128, 32, 2, 2>;

template <class K>
dp_status allow_lds(K kernel, size_t bytes) {
  return hip_status(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
}

}  // namespace

int perex_tiles_per_sample(int d, int p) {
  return ((d + PerexShape::BM - 1) / PerexShape::BM) * ((p + PerexShape::BN - 1) / PerexShape::BN);
}

int clipped_grad_tiles(int d, int p) {
  return ((d + GradShape::BM - 1) / GradShape::BM) * ((p + GradShape::BN - 1) / GradShape::BN);
}

dp_status launch_clipped_grad_group(const GroupArgs& ga, const float* C, hipStream_t s) {
  auto kernel = clipped_grad_kernel<GradShape>;
  dp_status st = allow_lds(kernel, GradShape::LDS_BYTES);
  if (st != DP_OK) return st;
  hipLaunchKernelGGL(kernel, dim3(ga.total_blocks), dim3(GradShape::NT), GradShape::LDS_BYTES, s, ga, C);
  return hip_status(hipGetLastError());
}

dp_status launch_perex_group(const GroupArgs& ga, float* partials, hipStream_t s) {
  auto kernel = perex_norm_kernel<PerexShape>;
  dp_status st = allow_lds(kernel, PerexShape::LDS_BYTES);
  if (st != DP_OK) return st;
  hipLaunchKernelGGL(kernel, dim3(ga.total_blocks), dim3(PerexShape::NT), PerexShape::LDS_BYTES, s, ga,
                     partials);
  return hip_status(hipGetLastError());
}

dp_status launch_norm_reduce_group(const GroupArgs& ga, const float* partials, float* sqnorm_out,
                                   hipStream_t s) {
  hipLaunchKernelGGL(norm_reduce_kernel, dim3(ga.n_layers * ga.B), dim3(64), 0, s, ga, partials,
                     sqnorm_out);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
