// Clip-weighted gradient on the matrix cores, large-tile kernel (section 3 of the paper,
// "DP gradient"):   grad[j,k] = sum_i C_i sum_t a[i,t,j] g[i,t,k].
//
// Design for gfx950 (measured on the device: dense bf16 MFMA sustains 2.2 PFLOP/s; the
// transposing 64-bit LDS read sustains ~130-150 B/clk/CU, half the rate of 128-bit reads):
//  * 256x256 output tile per workgroup, 4 waves of 128x128: LDS read traffic per MFMA is the
//    lowest the register file allows (256 accumulator registers per lane), so the transposing
//    reads use about half of their bandwidth.
//  * global -> LDS without passing through registers (buffer_load ... lds, 16 B per lane).
//    A wave's load lands as 1 KiB of consecutive LDS = two 512-byte k rows, so rows cannot be
//    padded; instead the 16-byte chunks of row k are XOR-swizzled by (k & 3) << 2, which
//    spreads four consecutive k rows over the four 64-byte bank groups the transposing read
//    touches at once.  Out-of-range chunks (tile edge, ragged T, past the last k-block) are
//    fetched with an offset past the buffer descriptor's size and arrive as zeros.
//  * five LDS stages of 32 k rows (all 160 KiB of the CU).  In iteration i a wave waits for its
//    own loads of k-block i+1, meets the others at one barrier (which certifies block i+1 in
//    LDS and block i-1 no longer read), issues the loads of block i+4 into the stage block i-1
//    used, and computes block i.  A load has three iterations (about 3000 clocks) to land.
//    Operand fragments of the next k-step are fetched from LDS during the MFMAs of the current
//    one, across the barrier too, so the matrix pipe never waits for LDS latency.
//    The loads are issued from inline assembly because the compiler otherwise waits for every
//    outstanding LDS-DMA load before any LDS read; MFMAs, LDS reads and loads are interleaved
//    by hand (one wave per SIMD: there is no second wave to hide issue gaps).
//  * per-sample weights: see tn_gemm.hip (single accumulator set, re-expressed at sample
//    boundaries).
#include <type_traits>

#include "dp_internal.h"
#include "lds_dma.h"
#include "tile_order.h"
#include "tn_tile.h"

namespace dpbk {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4v;

#ifndef DP_GRAD_NSTAGE
#define DP_GRAD_NSTAGE 5
#endif
constexpr int BM = 256, BN = 256, BK = 32, NSTAGE = DP_GRAD_NSTAGE;
constexpr int NT = 256;
constexpr int ROW_BYTES = 512;                         // 256 bf16
constexpr int TILE_BYTES = BK * ROW_BYTES;             // one operand, one stage (16 KiB)
constexpr int STAGE_BYTES = 2 * TILE_BYTES;            // 32 KiB
constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;        // 160 KiB with 5 stages: all of the CU's LDS
constexpr int LOADS = BK / 8;                          // per operand per thread per k-block

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

// Tile t of the launch -> layer and tile origin (order inside a layer: tile_order.h).
__device__ __forceinline__ void locate_tile(const GroupArgs& ga, int t, int& layer, int& m0, int& n0) {
  const int l = layer_of(ga, t);
  layer = l;
  const GroupLayer& ly = ga.layer[l];
  int tm, tn;
  grad_tile_of((ly.d_in + BM - 1) / BM, (ly.d_out + BN - 1) / BN, t - ly.tile_begin, tm, tn);
  m0 = tm * BM;
  n0 = tn * BN;
}

// 16-bit gradient output (mixed-precision training keeps gradients in the storage type of the
// activations: section 2.3 of the paper): the fp32 value - weighted sum, old value when
// accumulating, noise - is rounded once, to nearest even, to bf16 or IEEE binary16.
template <bool F16>
__device__ __forceinline__ uint16_t to_half_bits(float x) {
  if constexpr (F16) {
    return __builtin_bit_cast(uint16_t, (_Float16)x);
  } else {
    const uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;                    // NaN stays NaN
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
  }
}
template <bool F16>
__device__ __forceinline__ float from_half_bits(uint16_t h) {
  if constexpr (F16)
    return (float)__builtin_bit_cast(_Float16, h);
  else
    return __uint_as_float((uint32_t)h << 16);
}

// Four consecutive outputs of one row: (+)= and store, fp32 (16 bytes) or 16-bit (8 bytes).
template <bool F16, bool OUT16, bool ACCUMULATE>
__device__ __forceinline__ void load_old4(const float* out32, size_t index, float (&old)[4]) {
  if constexpr (!ACCUMULATE) {
    old[0] = old[1] = old[2] = old[3] = 0.f;
  } else if constexpr (OUT16) {
    const uint2 w = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(out32) + index);
    old[0] = from_half_bits<F16>((uint16_t)(w.x & 0xFFFFu));
    old[1] = from_half_bits<F16>((uint16_t)(w.x >> 16));
    old[2] = from_half_bits<F16>((uint16_t)(w.y & 0xFFFFu));
    old[3] = from_half_bits<F16>((uint16_t)(w.y >> 16));
  } else {
    const f32x4v w = *reinterpret_cast<const f32x4v*>(out32 + index);
    old[0] = w[0]; old[1] = w[1]; old[2] = w[2]; old[3] = w[3];
  }
}
template <bool F16, bool OUT16>
__device__ __forceinline__ void store4(float* out32, size_t index, const float* v) {
  if constexpr (OUT16) {
    uint2 w;
    w.x = (uint32_t)to_half_bits<F16>(v[0]) | ((uint32_t)to_half_bits<F16>(v[1]) << 16);
    w.y = (uint32_t)to_half_bits<F16>(v[2]) | ((uint32_t)to_half_bits<F16>(v[3]) << 16);
    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out32) + index) = w;
  } else {
    const f32x4v w = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4v*>(out32 + index) = w;
  }
}

// The kernel's copy of what tile_noise needs, read once from the kernel arguments into registers.
struct TileNoise {
  float stddev;
  uint32_t step_lo, step_hi;
  uint64_t lo, hi, layer_off;
  RoundKeys rk;
};

__device__ __forceinline__ TileNoise load_tile_noise(const NoiseArgs& na, int layer) {
  TileNoise t;
  t.stddev = na.stddev;
  t.step_lo = na.step_lo;
  t.step_hi = na.step_hi;
  t.lo = na.lo;
  t.hi = na.hi;
  t.layer_off = na.layer_off[layer];
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    t.rk.k[r][0] = na.rk.k[r][0];
    t.rk.k[r][1] = na.rk.k[r][1];
  }
  return t;
}

// Output layout.  The MFMAs take the g fragment as first operand and the a fragment as second,
// so a wave holds the transposed product: lane l has row (l & 31) of a 32 x 32 output tile and
// the columns 8 q + 4 (l >> 5) + e (q, e = 0 .. 3) in register 4 q + e: four runs of four
// consecutive columns, which are stored as 16-byte vectors (a quarter of the store
// instructions of the untransposed layout, whose lanes hold single columns) and each of which
// is exactly one block of the noise generator.
//
// Adds the noise of eq. (1) to the lane's 16 values of the tile at (tile_row0, tile_col0): same
// values as the separate noise pass, which indexes the generator by global element too.
// Requires layer_off and d_out to be multiples of 4.
__device__ __forceinline__ void tile_noise(float (&v)[16], const TileNoise& na, int tile_row0, int tile_col0,
                                           int d, int p, int lane) {
  const int rows = min(32, d - tile_row0), cols = min(32, p - tile_col0);
  if (rows <= 0 || cols <= 0) return;
  const uint64_t e_first = na.layer_off + (uint64_t)tile_row0 * p + tile_col0;
  const uint64_t e_last = na.layer_off + (uint64_t)(tile_row0 + rows - 1) * p + (tile_col0 + cols - 1);
  if (e_last < na.lo || e_first >= na.hi) return;               // wave-uniform: tile outside the shard
  const bool whole = e_first >= na.lo && e_last < na.hi;
  const int row = tile_row0 + (lane & 31);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int col = tile_col0 + 8 * q + 4 * (lane >> 5);
    if (row < d && col < p) {
      const uint64_t e = na.layer_off + (uint64_t)row * p + col;
      float z[4];
      normal_block(e >> 2, na.step_lo, na.step_hi, na.rk, z);
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (whole || (e + k >= na.lo && e + k < na.hi)) v[4 * q + k] = fmaf(na.stddev, z[k], v[4 * q + k]);
    }
  }
}

template <bool F16, bool NOISE, bool OUT16>
__global__ void __launch_bounds__(NT)
clipped_grad_big_kernel(const GroupArgs ga, const float* __restrict__ C_global, const NoiseArgs na) {
  // The weights do not change during the kernel: read them through the constant address space
  // so that they come by scalar loads (a vector load here would make the compiler wait for
  // every outstanding prefetch load at each sample boundary).
  const __attribute__((address_space(4))) float* C =
      (const __attribute__((address_space(4))) float*)(uintptr_t)C_global;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  const unsigned lds0 = (unsigned)(uintptr_t)lds_raw;

  const int logical = grad_logical_tile(blockIdx.x, ga.total_blocks);     // XCD-aware: tile_order.h
  int l, m0, n0;
  locate_tile(ga, logical, l, m0, n0);
  const GroupLayer& ly = ga.layer[l];
  const int T = ly.T, d = ly.d_in, p = ly.d_out;
  const int B = ga.B;
  const int nkb = (T + BK - 1) / BK;
  C += ly.c_off;                                  // the layer's clipping group

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: keeps LDS bases scalar

  // ---- global -> LDS addressing -------------------------------------------------------
  // Load j of a wave covers rows j*8 + wave*2 + (lane >> 5) of the 32-row k-block; the lane's
  // LDS chunk (lane & 31) holds logical chunk (lane & 31) ^ ((row & 3) << 2).
  const int lrow = wave * 2 + (lane >> 5);
  const int chunk = (lane & 31) ^ ((lrow & 3) << 2);
  const bool a_in = m0 + chunk * 8 < d, b_in = n0 + chunk * 8 < p;
  const unsigned a_off0 = (unsigned)(lrow * d + m0 + chunk * 8) * 2u;
  const unsigned b_off0 = (unsigned)(lrow * p + n0 + chunk * 8) * 2u;
  const unsigned a_step = 8u * d * 2u, b_step = 8u * p * 2u;          // bytes per 8 rows
  const unsigned a_slab = (unsigned)T * d * 2u, b_slab = (unsigned)T * p * 2u;
  const unsigned char* a_base = static_cast<const unsigned char*>(ly.a);
  const unsigned char* b_base = static_cast<const unsigned char*>(ly.g);
  const unsigned lds_ld = lds0 + wave * 2 * ROW_BYTES;

  // Prefetch stream: (p_i, p_kb) is the next k-block to fetch.  Once p_i >= B ("past the
  // end") every lane fetches zeros, so each iteration issues the same number of loads.
  // T is a multiple of BK here (checked on the host), so rows never run past a sample.
  int p_i = 0, p_kb = 0, p_stage = 0;
  while (p_i < B && C[p_i] == 0.f) ++p_i;
  i32x4 ra, rb;
  unsigned va, vb;                 // per-lane byte offset inside the sample's slab, or OOB
  unsigned sa = 0, sb = 0;         // scalar byte offset of the k-block inside the slab
  auto prefetch_sample = [&]() {
    const bool valid = p_i < B;
    const int smp = valid ? p_i : 0;
    ra = make_rsrc(a_base + (size_t)smp * a_slab, a_slab);
    rb = make_rsrc(b_base + (size_t)smp * b_slab, b_slab);
    va = (valid && a_in) ? a_off0 : OOB;
    vb = (valid && b_in) ? b_off0 : OOB;
    sa = 0;
    sb = 0;
  };
  prefetch_sample();
  // One of the LOADS load pairs of the current prefetch block.
  auto prefetch_issue_a = [&](int j) {
    load_to_lds(ra, va, sa + j * a_step, lds_ld + p_stage * STAGE_BYTES + j * 8 * ROW_BYTES);
  };
  auto prefetch_issue_b = [&](int j) {
    load_to_lds(rb, vb, sb + j * b_step, lds_ld + p_stage * STAGE_BYTES + j * 8 * ROW_BYTES + TILE_BYTES);
  };
  auto prefetch_advance = [&]() {
    sa += BK * d * 2u;
    sb += BK * p * 2u;
    if (p_i < B && ++p_kb == nkb) {
      p_kb = 0;
      ++p_i;
      while (p_i < B && C[p_i] == 0.f) ++p_i;
      prefetch_sample();
    }
    p_stage = p_stage + 1 == NSTAGE ? 0 : p_stage + 1;
  };

  // ---- LDS -> MFMA operand addressing ---------------------------------------------------
  // 16-lane block b = lane >> 4, s = lane & 15: row = 8*(b>>1) + (s>>2) (+4 for the second
  // half), element column = 16*(b&1) + 4*(s&3) inside a 32-wide MFMA tile.
  const int blk = lane >> 4, s = lane & 15;
  const int rrow = 8 * (blk >> 1) + (s >> 2);
  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
  unsigned a_rd[4], b_rd[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ca = (wm + i * 32 + 16 * (blk & 1) + 4 * (s & 3)) >> 3;
    const int cb = (wn + i * 32 + 16 * (blk & 1) + 4 * (s & 3)) >> 3;
    const int sw = (rrow & 3) << 2;
    a_rd[i] = lds0 + rrow * ROW_BYTES + ((ca ^ sw) << 4) + (s & 1) * 8;
    b_rd[i] = lds0 + TILE_BYTES + rrow * ROW_BYTES + ((cb ^ sw) << 4) + (s & 1) * 8;
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  Frag fa[2][4], fb[2][4];
  // Fragment reads of k-step `ks` of the block in `stage`: item q in 0..7 reads fb[q] (q < 4)
  // or fa[q - 4].  The first MFMA row of the next k-step needs every fb but only fa[0], so the
  // B fragments go first and the last-issued read (fa[3]) is needed last.
  auto read_frag = [&](int buf, int q, int stage, int ks) {
    const unsigned o = stage * STAGE_BYTES + ks * 16 * ROW_BYTES;
    if (q < 4) {
      fb[buf][q].h[0] = lds_read_tr(b_rd[q] + o);
      fb[buf][q].h[1] = lds_read_tr(b_rd[q] + o + 4 * ROW_BYTES);
    } else {
      fa[buf][q - 4].h[0] = lds_read_tr(a_rd[q - 4] + o);
      fa[buf][q - 4].h[1] = lds_read_tr(a_rd[q - 4] + o + 4 * ROW_BYTES);
    }
  };

  // Compute stream: outer loop over samples with a non-zero weight, inner loop over the
  // sample's k-blocks.  The global->LDS prefetch runs ahead across sample boundaries; the
  // fragment pipeline restarts at each sample (one exposed LDS latency per sample).
  int c_i = p_i;
  float held = 0.f;
  if (c_i < B) {
    held = C[c_i];
    // prologue: blocks 0 .. NSTAGE-2 in flight; block 0 complete in LDS
    for (int q = 0; q < NSTAGE - 1; ++q) {
#pragma unroll
      for (int j = 0; j < LOADS; ++j) {
        prefetch_issue_a(j);
        prefetch_issue_b(j);
      }
      prefetch_advance();
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * 2 * LOADS) : "memory");
    __syncthreads();

    int c_stage = 0;
    // One k-block: wait for block +1, barrier, issue block +(NSTAGE-1), 32 MFMAs.  `last` = last block
    // of the sample: the fragments of the following block are not fetched here.
    auto block = [&](auto last_tag) {
      constexpr bool last = decltype(last_tag)::value;
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 3) * 2 * LOADS) : "memory");
      __builtin_amdgcn_s_barrier();
      const int n_stage = c_stage + 1 == NSTAGE ? 0 : c_stage + 1;
      DP_PIN();
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const int cb = ks, nb = ks ^ 1;
        const bool fetch = ks == 0 || !last;
        const int r_stage = ks == 0 ? c_stage : n_stage, r_ks = ks == 0 ? 1 : 0;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          acc[g][0] = mfma16<F16>(fb[cb][0].v, fa[cb][g].v, acc[g][0]);
          DP_PIN();
          if (fetch) read_frag(nb, 2 * g, r_stage, r_ks);
          DP_PIN();
          acc[g][1] = mfma16<F16>(fb[cb][1].v, fa[cb][g].v, acc[g][1]);
          DP_PIN();
          if (fetch) read_frag(nb, 2 * g + 1, r_stage, r_ks);
          DP_PIN();
          acc[g][2] = mfma16<F16>(fb[cb][2].v, fa[cb][g].v, acc[g][2]);
          DP_PIN();
          if (g & 1)
            prefetch_issue_b(ks * 2 + (g >> 1));
          else
            prefetch_issue_a(ks * 2 + (g >> 1));
          DP_PIN();
          acc[g][3] = mfma16<F16>(fb[cb][3].v, fa[cb][g].v, acc[g][3]);
          DP_PIN();
        }
      }
      prefetch_advance();
      c_stage = n_stage;
    };

    bool first = true;
    while (c_i < B) {
      const float c = C[c_i];
      if (!first) {
        // re-express the accumulator in this sample's weight
        // In place on the accumulator registers, four at a time, from assembly: left to the
        // compiler this block wants every accumulator in a VGPR at once and spills the loop's
        // operands.  The s_nop pairs cover the MFMA-result -> VALU-read and the
        // accumulator-write -> MFMA-read wait states, which the compiler does not track
        // through inline assembly.
        const float f = held / c;
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        if (f != 1.f)                       // equal weights (e.g. nothing clipped): nothing to do
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
          for (int y = 0; y < 4; ++y)
#pragma unroll
            for (int h = 0; h < 4; ++h) {
              float e0 = acc[x][y][4 * h], e1 = acc[x][y][4 * h + 1], e2 = acc[x][y][4 * h + 2],
                    e3 = acc[x][y][4 * h + 3];
              float t0, t1, t2, t3;
              asm volatile(
                  "v_accvgpr_read_b32 %4, %0\n\tv_accvgpr_read_b32 %5, %1\n\t"
                  "v_accvgpr_read_b32 %6, %2\n\tv_accvgpr_read_b32 %7, %3\n\t"
                  "v_mul_f32 %4, %8, %4\n\tv_mul_f32 %5, %8, %5\n\t"
                  "v_mul_f32 %6, %8, %6\n\tv_mul_f32 %7, %8, %7\n\t"
                  "v_accvgpr_write_b32 %0, %4\n\tv_accvgpr_write_b32 %1, %5\n\t"
                  "v_accvgpr_write_b32 %2, %6\n\tv_accvgpr_write_b32 %3, %7"
                  : "+a"(e0), "+a"(e1), "+a"(e2), "+a"(e3), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
                  : "v"(f));
              acc[x][y][4 * h] = e0;
              acc[x][y][4 * h + 1] = e1;
              acc[x][y][4 * h + 2] = e2;
              acc[x][y][4 * h + 3] = e3;
            }
        asm volatile("s_nop 7" ::: "memory");
      }
      first = false;
      held = c;
#pragma unroll
      for (int q = 0; q < 8; ++q) read_frag(0, q, c_stage, 0);
      for (int kb = 0; kb + 1 < nkb; ++kb) block(std::false_type{});
      block(std::true_type{});
      ++c_i;
      while (c_i < B && C[c_i] == 0.f) ++c_i;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // zero-fill loads past the end
  }

  // epilogue: grad (+)= held * acc (+ noise), in the transposed layout described at tile_noise.
  // With no active sample the accumulator is zero.
  float* out = ly.out;
  TileNoise tn = {};
  if (NOISE) tn = load_tile_noise(na, l);
  auto store_tile = [&](auto acc_tag) {
    constexpr bool accumulate = decltype(acc_tag)::value;
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        const int row = m0 + wm + x * 32 + (lane & 31);
        const int col0 = n0 + wn + y * 32 + 4 * (lane >> 5);
        const size_t base = (size_t)row * p + col0;                  // + 8 q: columns col0 + 8 q ..
        float v[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float old[4] = {0.f, 0.f, 0.f, 0.f};
          if (accumulate && row < d && col0 + 8 * q < p) load_old4<F16, OUT16, accumulate>(out, base + 8 * q, old);
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const float t = acc[x][y][4 * q + k] * held;
            v[4 * q + k] = accumulate ? old[k] + t : t;
          }
        }
        if (NOISE) tile_noise(v, tn, m0 + wm + x * 32, n0 + wn + y * 32, d, p, lane);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (row < d && col0 + 8 * q < p) store4<F16, OUT16>(out, base + 8 * q, v + 4 * q);
        __builtin_amdgcn_sched_barrier(0);
      }
  };
  if (ga.accumulate)
    store_tile(std::true_type{});
  else
    store_tile(std::false_type{});
}

// ---------------------------------------------------------------------------------
// Tail of a launch.  All tiles of a launch take the same time and one workgroup fills a compute
// unit, so n tiles run in ceil(n / 256) rounds; when the last round would hold only a few tiles
// (n mod 256 small), those tiles are cut into TAIL x TAIL sub-tiles instead, one small
// workgroup each (register-staged tile code of tn_tile.h), which spreads them over the whole
// chip.  Sub-tile b of the launch belongs to tile first_tile + b / SUBS of locate_tile's order.
// ---------------------------------------------------------------------------------
#ifndef DP_TAIL_SHAPE
#define DP_TAIL_SHAPE 64, 64, 64, 2, 2
#endif
#ifndef DP_TAIL_DEPTH
#define DP_TAIL_DEPTH 4
#endif

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// One small output tile with D k-blocks in flight between memory and LDS (register slots used
// in rotation, the loop unrolled D times so that every slot index is a constant).  A small
// tile's k-block holds too little arithmetic to cover the latency of the next one's loads,
// and with one wave per SIMD every instruction of the loop counts: the loads are buffer loads
// whose range check zero-fills what lies outside the sample's slab (rows past T, columns past
// the layer's edge through the OOB offset, blocks past the last sample through an empty
// descriptor), so a k-block costs one add and one load per 16 bytes and nothing is
// conditional: the number of loads in flight is a compile-time constant and a thread waits only
// for the slot it is about to store.  Two LDS stages, one barrier per k-block.  The k-steps of an output element are added in
// the same order as in the large kernel.
template <class S, int D, bool F16, bool NOISE, bool OUT16>
__device__ __forceinline__ void clipped_grad_tile_deep(const GroupLayer& ly, int B, int accumulate,
                                                       const NoiseArgs& na, int layer, int m0, int n0,
                                                       const __attribute__((address_space(4))) float* C,
                                                       uint16_t* lds) {
  static_assert(D % 2 == 0, "the LDS stage of slot q is q & 1");
  const int tid = threadIdx.x;
  const int T = ly.T, d = ly.d_in, p = ly.d_out;
  const int nkb = (T + S::BK - 1) / S::BK;
  const unsigned a_slab = (unsigned)T * d * 2u, b_slab = (unsigned)T * p * 2u;
  const unsigned a_step = (unsigned)S::BK * d * 2u, b_step = (unsigned)S::BK * p * 2u;
  const unsigned char* a_base = static_cast<const unsigned char*>(ly.a);
  const unsigned char* b_base = static_cast<const unsigned char*>(ly.g);

  // Per-thread geometry of the loads of one k-block: byte offset inside the slab (k-block 0)
  // and element offset inside the LDS stage.
  unsigned va[S::A_PER_T], vb[S::B_PER_T];
  int sta[S::A_PER_T], stb[S::B_PER_T];
#pragma unroll
  for (int j = 0; j < S::A_PER_T; ++j) {
    const int c = tid + j * S::NT, row = c / (S::BM / 8), col = (c % (S::BM / 8)) * 8;
    va[j] = m0 + col < d ? (unsigned)(row * d + m0 + col) * 2u : OOB;
    sta[j] = row * S::SA + col;
  }
#pragma unroll
  for (int j = 0; j < S::B_PER_T; ++j) {
    const int c = tid + j * S::NT, row = c / (S::BN / 8), col = (c % (S::BN / 8)) * 8;
    vb[j] = n0 + col < p ? (unsigned)(row * p + n0 + col) * 2u : OOB;
    stb[j] = S::BK * S::SA + row * S::SB + col;
  }

  // All operand fragments of a k-block are requested from LDS before its first MFMA, so one LDS
  // latency is exposed per k-block instead of one per MFMA (a wave has nothing else to run).
  static_assert(S::TM == 1 && S::TN == 1, "one 32 x 32 MFMA tile per wave");
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave / S::WN) * S::WTM, wn = (wave % S::WN) * S::WTN;
  auto compute = [&](const uint16_t* stage, f32x16& c) {
    constexpr int KS = S::BK / 16;
    bf16x8 fa[KS], fb[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      fa[ks] = read_frag_tr(stage, S::SA, ks * 16, wm, lane);
      fb[ks] = read_frag_tr(stage + S::BK * S::SA, S::SB, ks * 16, wn, lane);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) c = mfma16<F16>(fb[ks], fa[ks], c);
  };
  u32x4 sa[D][S::A_PER_T], sb[D][S::B_PER_T];
  f32x16 acc[S::TM][S::TN];
  zero_acc<S>(acc);

  // (sample, k-block) cursors over the samples with a non-zero weight: ld = next block to
  // request from memory, cp = next block to compute.
  int ld_i = 0, ld_kb = 0, cp_i, cp_kb = 0, active = 0;
  for (int i = 0; i < B; ++i) active += C[i] != 0.f;
  while (ld_i < B && C[ld_i] == 0.f) ++ld_i;
  cp_i = ld_i;
  float held = cp_i < B ? C[cp_i] : 0.f;   // weight the accumulator is currently expressed in
  __amdgpu_buffer_rsrc_t ra, rb;
  unsigned koff_a = 0, koff_b = 0;         // byte offset of the load cursor's k-block in the slab
  auto open_sample = [&]() {
    const bool valid = ld_i < B;
    const int smp = valid ? ld_i : 0;
    ra = __builtin_amdgcn_make_buffer_rsrc((void*)(a_base + (size_t)smp * a_slab), 0,
                                           valid ? (int)a_slab : 0, 0x00020000);
    rb = __builtin_amdgcn_make_buffer_rsrc((void*)(b_base + (size_t)smp * b_slab), 0,
                                           valid ? (int)b_slab : 0, 0x00020000);
    koff_a = 0;
    koff_b = 0;
  };
  open_sample();
  auto fetch = [&](u32x4 (&xa)[S::A_PER_T], u32x4 (&xb)[S::B_PER_T]) {
#pragma unroll
    for (int j = 0; j < S::A_PER_T; ++j)
      xa[j] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(ra, va[j] + koff_a, 0, 0));
#pragma unroll
    for (int j = 0; j < S::B_PER_T; ++j)
      xb[j] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, vb[j] + koff_b, 0, 0));
    koff_a += a_step;
    koff_b += b_step;
    if (ld_i < B && ++ld_kb == nkb) {
      ld_kb = 0;
      ++ld_i;
      while (ld_i < B && C[ld_i] == 0.f) ++ld_i;
      open_sample();
    }
  };
#pragma unroll
  for (int q = 0; q < D; ++q) fetch(sa[q], sb[q]);
  auto store = [&](uint16_t* stage, const u32x4 (&xa)[S::A_PER_T], const u32x4 (&xb)[S::B_PER_T]) {
#pragma unroll
    for (int j = 0; j < S::A_PER_T; ++j) *reinterpret_cast<u32x4*>(stage + sta[j]) = xa[j];
#pragma unroll
    for (int j = 0; j < S::B_PER_T; ++j) *reinterpret_cast<u32x4*>(stage + stb[j]) = xb[j];
  };
  // Block n is computed from stage n & 1 while block n + 1 is being written to the other stage;
  // the barrier at the end of an iteration certifies both that write and that nobody still
  // reads the stage the next iteration overwrites.
  const int blocks = active * nkb;
  store(lds, sa[0], sb[0]);
  fetch(sa[0], sb[0]);
  __syncthreads();
  for (int n = 0; n < blocks; n += D) {
#pragma unroll
    for (int q = 0; q < D; ++q) {
      const int nq = (q + 1) % D;
      store(lds + ((q + 1) & 1) * S::STAGE, sa[nq], sb[nq]);
      fetch(sa[nq], sb[nq]);
      compute(lds + (q & 1) * S::STAGE, acc[0][0]);
      __syncthreads();
      if (cp_i < B && ++cp_kb == nkb) {
        cp_kb = 0;
        ++cp_i;
        while (cp_i < B && C[cp_i] == 0.f) ++cp_i;
        if (cp_i < B) {                   // next block starts another sample: re-express acc
          const float c = C[cp_i];
          scale_acc<S>(acc, held / c);
          held = c;
        }
      }
    }
  }

  // epilogue in the transposed layout described at tile_noise
  float* out = ly.out;
  const int row = m0 + wm + (lane & 31), col0 = n0 + wn + 4 * (lane >> 5);
  const size_t base = (size_t)row * p + col0;
  float v[16];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float old[4] = {0.f, 0.f, 0.f, 0.f};
    if (accumulate && row < d && col0 + 8 * q < p) load_old4<F16, OUT16, true>(out, base + 8 * q, old);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float t = acc[0][0][4 * q + k] * held;
      v[4 * q + k] = accumulate ? old[k] + t : t;
    }
  }
  if (NOISE) tile_noise(v, load_tile_noise(na, layer), m0 + wm, n0 + wn, d, p, lane);
#pragma unroll
  for (int q = 0; q < 4; ++q)
    if (row < d && col0 + 8 * q < p) store4<F16, OUT16>(out, base + 8 * q, v + 4 * q);
}

// Sub-tiles are 64 x 64 (16 per tile), k-blocks of 64 rows, four k-blocks in flight: three
// workgroups fit in a compute unit's LDS.
using TailShape = TnShape<DP_TAIL_SHAPE>;
constexpr int TAIL = 64, SUBS_N = BN / TAIL, SUBS = (BM / TAIL) * SUBS_N;
static_assert(TailShape::BM == TAIL && TailShape::BN == TAIL, "sub-tile shape");

template <bool F16, bool NOISE, bool OUT16>
__global__ void __launch_bounds__(TailShape::NT)
clipped_grad_tail_kernel(const GroupArgs ga, const float* __restrict__ C_all, int first_tile,
                         const NoiseArgs na) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_tail[];
  // Workgroup b runs on XCD b % 8: give each XCD a contiguous eighth of the sub-tiles (the grid
  // is a multiple of 16), so that the 16 sub-tiles of a tile, which share its operand panels,
  // meet in one L2.
  const int logical = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  int l, m0, n0;
  locate_tile(ga, first_tile + logical / SUBS, l, m0, n0);
  const GroupLayer& ly = ga.layer[l];
  const int sub = logical % SUBS;
  m0 += (sub / SUBS_N) * TAIL;
  n0 += (sub % SUBS_N) * TAIL;
  if (m0 >= ly.d_in || n0 >= ly.d_out) return;       // sub-tile past the layer's edge (whole workgroup)
  const __attribute__((address_space(4))) float* C =
      (const __attribute__((address_space(4))) float*)(uintptr_t)(C_all + ly.c_off);
  clipped_grad_tile_deep<TailShape, DP_TAIL_DEPTH, F16, NOISE, OUT16>(ly, ga.B, ga.accumulate, na, l, m0,
                                                               n0, C, lds_tail);
}

}  // namespace

int clipped_grad_big_tiles(int d, int p) { return ((d + BM - 1) / BM) * ((p + BN - 1) / BN); }

// The kernel addresses each sample's slab of a layer with 32-bit byte offsets and uses
// bit 31 as the "fetch zeros" marker, so a slab must be smaller than 2 GiB; k-blocks must
// not straddle samples, so T must be a multiple of the k-block.
bool clipped_grad_big_supports(int T, int d, int p) {
  return T % BK == 0 && (int64_t)T * d * 2 < (int64_t)1 << 31 && (int64_t)T * p * 2 < (int64_t)1 << 31;
}

// Tiles left for the tail kernel: the last n mod 256 tiles of the launch when they are few.
// Sub-tiles fetch four times the operand bytes per flop of a large tile and the tail kernel runs
// at the rate the L2 delivers them (measured: 16 tiles with K = 4096 take 30-50 us, a round of
// large tiles 150 us; 36 tiles about 0.7 of a round), so beyond kTailMax tiles a short last
// round of large tiles is as fast.
#ifndef DP_TAIL_MAX
#define DP_TAIL_MAX 40
#endif
constexpr int kRound = 256;           // compute units = large-tile workgroups resident at a time

int clipped_grad_big_tail_tiles(int n) {
  const int n_tail = n % kRound;
  return n_tail > DP_TAIL_MAX ? 0 : n_tail;
}

template <bool F16, bool NOISE, bool OUT16>
dp_status launch_clipped_grad_big_group_t(const GroupArgs& ga, const float* C, const NoiseArgs& na,
                                          hipStream_t s) {
  auto big = clipped_grad_big_kernel<F16, NOISE, OUT16>;
  auto tail = clipped_grad_tail_kernel<F16, NOISE, OUT16>;
  static ReadyTable ready_big, ready_tail;
  dp_status st0 = allow_big_lds(big, LDS_BYTES, ready_big);
  if (st0 != DP_OK) return st0;
  st0 = allow_big_lds(tail, (int)TailShape::LDS_BYTES, ready_tail);
  if (st0 != DP_OK) return st0;
  const int n = ga.total_blocks;
  const int n_tail = clipped_grad_big_tail_tiles(n);
  if (n > n_tail) {
    GroupArgs main_args = ga;
    main_args.total_blocks = n - n_tail;
    hipLaunchKernelGGL(big, dim3(n - n_tail), dim3(NT), LDS_BYTES, s, main_args, C, na);
    dp_status st = hip_status(hipGetLastError());
    if (st != DP_OK) return st;
  }
  if (n_tail == 0) return DP_OK;
  hipLaunchKernelGGL(tail, dim3(n_tail * SUBS), dim3(TailShape::NT), TailShape::LDS_BYTES, s, ga, C,
                     n - n_tail, na);
  return hip_status(hipGetLastError());
}

// out16: the layers' `out` pointers address 16-bit arrays of the operands' storage type.
dp_status launch_clipped_grad_big_group(const GroupArgs& ga, const float* C, const NoiseArgs* noise,
                                        hipStream_t s, bool out16) {
  static const NoiseArgs none = {};
  const NoiseArgs& na = noise ? *noise : none;
  switch ((ga.f16 ? 4 : 0) + (noise ? 2 : 0) + (out16 ? 1 : 0)) {
    case 0: return launch_clipped_grad_big_group_t<false, false, false>(ga, C, na, s);
    case 1: return launch_clipped_grad_big_group_t<false, false, true>(ga, C, na, s);
    case 2: return launch_clipped_grad_big_group_t<false, true, false>(ga, C, na, s);
    case 3: return launch_clipped_grad_big_group_t<false, true, true>(ga, C, na, s);
    case 4: return launch_clipped_grad_big_group_t<true, false, false>(ga, C, na, s);
    case 5: return launch_clipped_grad_big_group_t<true, false, true>(ga, C, na, s);
    case 6: return launch_clipped_grad_big_group_t<true, true, false>(ga, C, na, s);
    default: return launch_clipped_grad_big_group_t<true, true, true>(ga, C, na, s);
  }
}

}  // namespace dpbk
