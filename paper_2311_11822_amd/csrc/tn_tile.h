// Register-staged bf16 tile machinery for products that contract over the token axis of two
// row-major operands (used by the kernels in tn_gemm.hip and by the tail kernel in
// grad_gemm.hip).  Tiles are staged in LDS as [k][m], exactly as they lie in memory, and
// fetched with the gfx950 transposing LDS read (ds_read_b64_tr_b16): within 16 lanes, lanes
// 4e..4e+3 supply row k0+e (16 consecutive m), and lane L receives column m0+L for k0..k0+3.
#pragma once

#include "dp_internal.h"

namespace dpbk {

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

  template <bool F16>
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
          acc[i][j] = mfma16<F16>(fa[i], fb[j], acc[i][j]);
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

// Clip-weighted gradient of one BM x BN output tile at (m0, n0) of layer `ly` (section 3 of the
// paper, "DP gradient"): out[j,k] (+)= sum_i C_i sum_t a[i,t,j] g[i,t,k].
//
// Per-sample weights never touch the bf16 operands.  The accumulator holds
// sum_{j<=i} (C_j / C_i) G_j while sample i is being added; crossing to the next sample
// multiplies it by C_i / C_{i+1} and the epilogue by the last C.  Samples with C == 0 are
// skipped.
template <class S, bool F16>
__device__ __forceinline__ void clipped_grad_tile(const GroupLayer& ly, int B, int accumulate, int m0,
                                                  int n0, const float* __restrict__ C, uint16_t* lds) {
  TnTile<S> t;
  t.a = static_cast<const uint16_t*>(ly.a);
  t.g = static_cast<const uint16_t*>(ly.g);
  t.T = ly.T;
  t.d = ly.d_in;
  t.p = ly.d_out;
  t.m0 = m0;
  t.n0 = n0;
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
      t.template compute<F16>(lds + stage * S::STAGE, acc);
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
          *dst = accumulate ? *dst + v : v;
        }
      }
    }
}

}  // namespace dpbk
