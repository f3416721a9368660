// Instantiated per-sample norm on the matrix cores with a deep load pipeline (appendix A.1 of the
// paper, left side of eq. "mixed ghost norm"):  sqnorm[i] = || a_i^T g_i ||_F^2.
//
// One workgroup owns (sample, 128 x 128 tile of the d_in x d_out gradient): it contracts over the
// sample's T token rows, squares and adds (and, on request, keeps the tile of G_i: appendix A.2
// applied to this path).  The register-staged kernel of tn_gemm.hip has one k-block in flight
// between memory and LDS, so each of its iterations lasts one memory latency (measured: 0.8 us
// per 64-token block, 50 us for T = 4096 with 16 us of matrix instructions).  Here the operand
// rows go from global memory to LDS without passing through registers (buffer_load ... lds),
// five stages of 32 token rows (80 KiB, so that two workgroups share a compute unit and cover
// each other's barriers), three blocks ahead of the one being computed (measured: 29 us for the
// same workgroup; seven or ten stages change nothing - what is left is LDS traffic: a 64 x 64
// wave tile reads one fragment per MFMA):
// in iteration i a wave waits for its own loads of k-block i+1, meets the others at one barrier
// (block i+1 is then whole in LDS and block i-1 no longer read), issues the loads of block i+4
// into the stage block i-1 used, and computes block i while it fetches the next fragments.
//
// Rows are d-contiguous in memory and in LDS (256 bytes per tile row); the MFMA wants 8
// consecutive k per lane, so fragments come through the transposing LDS read.  A wave's load
// lands as four consecutive 256-byte rows, so rows cannot be padded: the 16-byte chunks of row k
// are XOR-swizzled by (k & 3) << 2, which spreads the four consecutive k rows one transposing
// read touches over four 64-byte bank groups.  Token rows past T and tile columns past the
// layer's edge are fetched with an offset past the buffer descriptor's size and arrive as zeros.
#include <type_traits>

#include "dp_internal.h"
#include "lds_dma.h"
#include "tile_order.h"

namespace dpbk {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4v;

constexpr int BM = 128, BN = 128, BK = 32, NSTAGE = 5;
constexpr int NT = 256;
constexpr int ROW_BYTES = 256;                         // 128 16-bit values
constexpr int TILE_BYTES = BK * ROW_BYTES;             // one operand, one stage (8 KiB)
constexpr int STAGE_BYTES = 2 * TILE_BYTES;            // 16 KiB
constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;        // 80 KiB: two workgroups per compute unit
constexpr int LOADS = 2;                               // per operand per thread per k-block
constexpr int LOADS_ALL = 2 * LOADS;

__device__ __forceinline__ s16x4 lds_read_tr(unsigned addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(uintptr_t)addr);
}

struct Frag {
  union {
    s16x4 h[2];
    bf16x8 v;
  };
};

template <bool F16>
__global__ void __launch_bounds__(NT)
perex_dma_kernel(const GroupArgs ga, float* __restrict__ partials) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  const unsigned lds0 = (unsigned)(uintptr_t)lds_raw;

  // The tiles of one (layer, sample) read the same panels of a_i and g_i: numbered consecutively
  // and dealt to the XCDs in contiguous eighths, they meet in one L2.
  const int item = contiguous_eighth(blockIdx.x, ga.total_blocks);
  const int l = layer_of(ga, item);
  const GroupLayer& ly = ga.layer[l];
  const int local = item - ly.tile_begin;
  const int sample = local / ly.tiles_per_sample;
  const int tile = local - sample * ly.tiles_per_sample;
  const int T = ly.T, d = ly.d_in, p = ly.d_out;
  const int tiles_n = (p + BN - 1) / BN;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const int nkb = (T + BK - 1) / BK;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- global -> LDS ------------------------------------------------------------------
  // Load j (0, 1) of a wave covers token rows j*16 + wave*4 + (lane >> 4) of the 32-row k-block,
  // 16 chunks of 16 bytes per row; the lane's LDS chunk c holds logical chunk c ^ ((row & 3) << 2).
  // The whole byte offset (row and column) is per lane, so that the descriptor's range check
  // zero-fills the rows past T.
  const int lrow = wave * 4 + (lane >> 4);
  const int chunk = (lane & 15) ^ ((lrow & 3) << 2);
  const unsigned a_slab = (unsigned)T * d * 2u, b_slab = (unsigned)T * p * 2u;
  const i32x4 ra = make_rsrc(static_cast<const unsigned char*>(ly.a) + (size_t)sample * a_slab, a_slab);
  const i32x4 rb = make_rsrc(static_cast<const unsigned char*>(ly.g) + (size_t)sample * b_slab, b_slab);
  unsigned va = m0 + chunk * 8 < d ? (unsigned)(lrow * d + m0 + chunk * 8) * 2u : OOB;
  unsigned vb = n0 + chunk * 8 < p ? (unsigned)(lrow * p + n0 + chunk * 8) * 2u : OOB;
  const unsigned a_half = 16u * d * 2u, b_half = 16u * p * 2u;       // bytes per 16 token rows
  const unsigned lds_ld = lds0 + wave * 4 * ROW_BYTES;
  int p_stage = 0;
  auto prefetch_issue = [&](int x) {                  // x = 0, 1: a; x = 2, 3: g
    const int j = x & 1;
    if (x < 2)
      load_to_lds(ra, va + j * a_half, 0, lds_ld + p_stage * STAGE_BYTES + j * 16 * ROW_BYTES);
    else
      load_to_lds(rb, vb + j * b_half, 0, lds_ld + p_stage * STAGE_BYTES + TILE_BYTES + j * 16 * ROW_BYTES);
  };
  auto prefetch_advance = [&]() {                     // blocks past the last one lie past the slab: zeros
    va += 2u * a_half;
    vb += 2u * b_half;
    p_stage = p_stage + 1 == NSTAGE ? 0 : p_stage + 1;
  };

  // ---- LDS -> MFMA operands -------------------------------------------------------------
  // 16-lane block b = lane >> 4, s = lane & 15 of the transposing read: k row 8*(b>>1) + (s>>2)
  // (+4 for the second half), element column 16*(b&1) + 4*(s&3) inside a 32-wide MFMA tile.
  const int blk = lane >> 4, s = lane & 15;
  const int rrow = 8 * (blk >> 1) + (s >> 2);
  const int sw = (rrow & 3) << 2;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  unsigned a_rd[2], b_rd[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int ca = (wm + i * 32 + 16 * (blk & 1) + 4 * (s & 3)) >> 3;
    const int cb = (wn + i * 32 + 16 * (blk & 1) + 4 * (s & 3)) >> 3;
    a_rd[i] = lds0 + rrow * ROW_BYTES + ((ca ^ sw) << 4) + (s & 1) * 8;
    b_rd[i] = lds0 + TILE_BYTES + rrow * ROW_BYTES + ((cb ^ sw) << 4) + (s & 1) * 8;
  }

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Fragments of a whole k-block (two k-steps) are fetched one block ahead, into the buffer set
  // of the other parity: a k-step of this tile is only 4 MFMAs per wave, too short to cover the
  // latency of the transposing reads of the next one.
  Frag fa[2][2][2], fb[2][2][2];                       // [block parity][k-step][tile]
  // item q of a k-step's fragments: g fragments (q = 0, 1), then a fragments (q = 2, 3)
  auto read_frag = [&](int par, int ks, int q, int stage) {
    const unsigned o = stage * STAGE_BYTES + ks * 16 * ROW_BYTES;
    if (q < 2) {
      fb[par][ks][q].h[0] = lds_read_tr(b_rd[q] + o);
      fb[par][ks][q].h[1] = lds_read_tr(b_rd[q] + o + 4 * ROW_BYTES);
    } else {
      fa[par][ks][q - 2].h[0] = lds_read_tr(a_rd[q - 2] + o);
      fa[par][ks][q - 2].h[1] = lds_read_tr(a_rd[q - 2] + o + 4 * ROW_BYTES);
    }
  };

  // prologue: blocks 0 .. NSTAGE-2 in flight, block 0 complete in LDS
  for (int q = 0; q < NSTAGE - 1; ++q) {
#pragma unroll
    for (int x = 0; x < LOADS_ALL; ++x) prefetch_issue(x);
    prefetch_advance();
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * LOADS_ALL) : "memory");
  __syncthreads();
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int q = 0; q < 4; ++q) read_frag(0, ks, q, 0);

  int c_stage = 0;
  // One k-block out of buffer set `par`: 8 MFMAs, the next block's fragments into the other set
  // (after the last block: a stage of zeros or of old rows, never used), 4 loads.
  auto block = [&](auto par_tag) {
    constexpr int par = decltype(par_tag)::value;
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 3) * LOADS_ALL) : "memory");
    __builtin_amdgcn_s_barrier();
    const int n_stage = c_stage + 1 == NSTAGE ? 0 : c_stage + 1;
    DP_PIN();
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
          acc[g][y] = mfma16<F16>(fb[par][ks][y].v, fa[par][ks][g].v, acc[g][y]);
          DP_PIN();
          read_frag(par ^ 1, ks, 2 * g + y, n_stage);
          DP_PIN();
          if (y == 1) prefetch_issue(ks * 2 + g);
          DP_PIN();
        }
    prefetch_advance();
    c_stage = n_stage;
  };
  for (int kb = 0; kb < nkb; kb += 2) {
    block(std::integral_constant<int, 0>{});
    if (kb + 1 < nkb) block(std::integral_constant<int, 1>{});
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // zero-fill loads past the end
  __syncthreads();                                      // LDS is reused below

  // The MFMAs take the g fragment as first operand and the a fragment as second, so a wave holds
  // the transposed product: lane l has gradient row (l & 31) of a 32 x 32 tile and the columns
  // 8 q + 4 (l >> 5) + e (q, e = 0 .. 3) in register 4 q + e.
  if (ly.out) {
    float* dst = ly.out + (size_t)sample * d * p;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        const int row = m0 + wm + x * 32 + (lane & 31);
        const int col0 = n0 + wn + y * 32 + 4 * (lane >> 5);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (row < d && col0 + 8 * q < p) {
            const f32x4v w = {acc[x][y][4 * q], acc[x][y][4 * q + 1], acc[x][y][4 * q + 2], acc[x][y][4 * q + 3]};
            *reinterpret_cast<f32x4v*>(dst + (size_t)row * p + col0 + 8 * q) = w;
          }
      }
  }

  // Rows/columns past the layer's edge were loaded as zeros, so they add nothing.
  float sum = 0.f;
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum = fmaf(acc[x][y][r], acc[x][y][r], sum);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  float* red = reinterpret_cast<float*>(lds_raw);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  if (threadIdx.x == 0) partials[ly.part_begin + local] = (red[0] + red[1]) + (red[2] + red[3]);
}

template <bool F16>
dp_status launch_perex_dma_t(const GroupArgs& ga, float* partials, hipStream_t s) {
  auto kernel = perex_dma_kernel<F16>;
  static ReadyTable ready;
  dp_status st = allow_big_lds(kernel, LDS_BYTES, ready);
  if (st != DP_OK) return st;
  hipLaunchKernelGGL(kernel, dim3(ga.total_blocks), dim3(NT), LDS_BYTES, s, ga, partials);
  return hip_status(hipGetLastError());
}

}  // namespace

// 32-bit byte offsets inside a sample's slab, bit 31 as the "fetch zeros" marker, and the
// prefetch runs up to NSTAGE blocks past the last token row without wrapping.
bool perex_dma_supports(int T, int d, int p) {
  const int64_t rows = (int64_t)T + (NSTAGE + 1) * BK;
  return rows * d * 2 < (int64_t)1 << 31 && rows * p * 2 < (int64_t)1 << 31;
}

dp_status launch_perex_dma_group(const GroupArgs& ga, float* partials, hipStream_t s) {
  return ga.f16 ? launch_perex_dma_t<true>(ga, partials, s) : launch_perex_dma_t<false>(ga, partials, s);
}

}  // namespace dpbk
