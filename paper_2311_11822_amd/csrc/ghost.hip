// Ghost norm on the matrix cores (appendix A.1 of the paper, right side of eq. "mixed ghost
// norm"):   sqnorm[i] = sum_{t,t'} (a_t . a_t') (g_t . g_t')   for sample i.
//
// One workgroup owns a BT x BT tile (I, J), J >= I, of both T x T Gram matrices of one
// sample.  It forms the tile of a a^T (contraction over d_in) and then the tile of g g^T
// (contraction over d_out) in two accumulator sets, multiplies them element by element,
// and reduces to one number; off-diagonal tiles count twice (both Gram matrices are
// symmetric).  No T x T matrix is ever written to memory.  Both products are "NT": rows
// are k-contiguous in memory, in LDS and in the MFMA operand, so tiles are staged as they
// lie and read back with plain 128-bit LDS reads.
#include "dp_internal.h"

namespace dpbk {

namespace {

template <int BT_, int BK_, int WM_, int WN_>
struct GramShape {
  static constexpr int BT = BT_, BK = BK_, WM = WM_, WN = WN_;
  static constexpr int NT = 64 * WM * WN;
  static constexpr int WTM = BT / WM, WTN = BT / WN;
  static constexpr int TM = WTM / 32, TN = WTN / 32;
  static constexpr int SK = BK + 8;                         // +16 B: 16 consecutive rows, 16 distinct banks groups
  static constexpr int PER_T = BT * BK / 8 / NT;            // 16-byte chunks per thread per tile
  static constexpr int TILE = BT * SK;
  static constexpr int STAGE = 2 * TILE;
  static constexpr size_t LDS_BYTES = 2 * STAGE * sizeof(uint16_t);
  static_assert(BK % 16 == 0 && (BT * BK / 8) % NT == 0, "tile shape");
};

template <class S, bool F16>
struct GramTile {
  const uint16_t* x;     // current operand of this sample: a_i or g_i, [T, width]
  int T, width;
  int r0, c0;            // first token of the row block I and of the column block J
  bool diag;
  uint4 ri[S::PER_T], rj[S::PER_T];

  __device__ __forceinline__ void gload(int kb) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < S::PER_T; ++j) {
      const int c = tid + j * S::NT;
      const int row = c / (S::BK / 8), k = kb * S::BK + (c % (S::BK / 8)) * 8;
      ri[j] = make_uint4(0, 0, 0, 0);
      rj[j] = make_uint4(0, 0, 0, 0);
      if (k < width) {
        if (r0 + row < T) ri[j] = *reinterpret_cast<const uint4*>(x + (size_t)(r0 + row) * width + k);
        if (!diag && c0 + row < T)
          rj[j] = *reinterpret_cast<const uint4*>(x + (size_t)(c0 + row) * width + k);
      }
    }
  }

  __device__ __forceinline__ void lds_store(uint16_t* stage) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < S::PER_T; ++j) {
      const int c = tid + j * S::NT;
      const int row = c / (S::BK / 8), k = (c % (S::BK / 8)) * 8;
      *reinterpret_cast<uint4*>(stage + row * S::SK + k) = ri[j];
      if (!diag) *reinterpret_cast<uint4*>(stage + S::TILE + row * S::SK + k) = rj[j];
    }
  }

  __device__ __forceinline__ void compute(const uint16_t* stage, f32x16 (&acc)[S::TM][S::TN]) const {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave / S::WN) * S::WTM, wn = (wave % S::WN) * S::WTN;
    const uint16_t* ti = stage;
    const uint16_t* tj = diag ? stage : stage + S::TILE;
#pragma unroll
    for (int ks = 0; ks < S::BK / 16; ++ks) {
      const int k = ks * 16 + 8 * (lane >> 5);
      bf16x8 fa[S::TM], fb[S::TN];
#pragma unroll
      for (int i = 0; i < S::TM; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(ti + (wm + i * 32 + (lane & 31)) * S::SK + k);
#pragma unroll
      for (int j = 0; j < S::TN; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(tj + (wn + j * 32 + (lane & 31)) * S::SK + k);
#pragma unroll
      for (int i = 0; i < S::TM; ++i)
#pragma unroll
        for (int j = 0; j < S::TN; ++j)
          acc[i][j] = mfma16<F16>(fa[i], fb[j], acc[i][j]);
    }
  }

  // Pipelined contraction over the operand's width into acc.  On return every LDS read has
  // been followed by a barrier.
  __device__ __forceinline__ void gram(uint16_t* lds, f32x16 (&acc)[S::TM][S::TN]) {
    const int nkb = (width + S::BK - 1) / S::BK;
    gload(0);
    lds_store(lds);
    __syncthreads();
    for (int kb = 0, stage = 0; kb < nkb; ++kb, stage ^= 1) {
      const bool more = kb + 1 < nkb;
      if (more) gload(kb + 1);
      compute(lds + stage * S::STAGE, acc);
      if (more) lds_store(lds + (stage ^ 1) * S::STAGE);
      __syncthreads();
    }
  }
};

__device__ __forceinline__ int find_layer_g(const GroupArgs& ga, int block) { return layer_of(ga, block); }

template <class S, bool F16>
__global__ void __launch_bounds__(S::NT)
ghost_norm_kernel(const GroupArgs ga, float* __restrict__ partials) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const int l = find_layer_g(ga, blockIdx.x);
  const GroupLayer& ly = ga.layer[l];
  const int local = blockIdx.x - ly.tile_begin;
  const int sample = local / ly.tiles_per_sample;
  int q = local % ly.tiles_per_sample;
  // q enumerates the upper triangle row by row: (0,0) (0,1) .. (0,nt-1) (1,1) ..
  const int nt = (ly.T + S::BT - 1) / S::BT;
  int I = 0;
  while (q >= nt - I) {
    q -= nt - I;
    ++I;
  }
  const int J = I + q;

  GramTile<S, F16> t;
  t.T = ly.T;
  t.r0 = I * S::BT;
  t.c0 = J * S::BT;
  t.diag = (I == J);

  f32x16 ga_acc[S::TM][S::TN], gg_acc[S::TM][S::TN];
#pragma unroll
  for (int i = 0; i < S::TM; ++i)
#pragma unroll
    for (int j = 0; j < S::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        ga_acc[i][j][r] = 0.f;
        gg_acc[i][j][r] = 0.f;
      }

  t.x = static_cast<const uint16_t*>(ly.a) + (size_t)sample * ly.T * ly.d_in;
  t.width = ly.d_in;
  t.gram(lds, ga_acc);
  t.x = static_cast<const uint16_t*>(ly.g) + (size_t)sample * ly.T * ly.d_out;
  t.width = ly.d_out;
  t.gram(lds, gg_acc);

  // Token rows past T were loaded as zeros: their Gram entries are zero.
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < S::TM; ++i)
#pragma unroll
    for (int j = 0; j < S::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s = fmaf(ga_acc[i][j][r], gg_acc[i][j][r], s);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  float* red = reinterpret_cast<float*>(lds);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) red[wave] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float total = 0.f;
    for (int w = 0; w < S::WM * S::WN; ++w) total += red[w];
    partials[ly.part_begin + local] = t.diag ? total : 2.f * total;
  }
}

using GhostShape = GramShape<128, 64, 2, 2>;

}  // namespace

int ghost_tiles_per_sample(int T) {
  const int nt = (T + GhostShape::BT - 1) / GhostShape::BT;
  return nt * (nt + 1) / 2;
}

template <bool F16>
dp_status launch_ghost_group_t(const GroupArgs& ga, float* partials, hipStream_t s) {
  auto kernel = ghost_norm_kernel<GhostShape, F16>;
  dp_status st = hip_status(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                                (int)GhostShape::LDS_BYTES));
  if (st != DP_OK) return st;
  hipLaunchKernelGGL(kernel, dim3(ga.total_blocks), dim3(GhostShape::NT), GhostShape::LDS_BYTES, s, ga,
                     partials);
  return hip_status(hipGetLastError());
}

dp_status launch_ghost_group(const GroupArgs& ga, float* partials, hipStream_t s) {
  return ga.f16 ? launch_ghost_group_t<true>(ga, partials, s) : launch_ghost_group_t<false>(ga, partials, s);
}

}  // namespace dpbk
