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

namespace dpbk {

namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;

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
constexpr unsigned OOB = 0x80000000u;

__device__ __forceinline__ i32x4 make_rsrc(const void* base, unsigned bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  i32x4 r;
  r[0] = (int)(uint32_t)p;
  r[1] = (int)(uint32_t)(p >> 32) & 0xFFFF;            // stride 0: raw buffer
  r[2] = (int)bytes;
  r[3] = 0x00020000;
  return r;
}

// 16 bytes per lane from buffer `rsrc` at byte `voff` to LDS at lds_base + 16*lane.
// The lane's byte address is voff + soff; the range check sees voff, so a lane whose voff has
// bit 31 set (>= any slab size) fetches zeros whatever soff is.
__device__ __forceinline__ void load_to_lds(i32x4 rsrc, unsigned voff, unsigned soff, unsigned lds_base) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "buffer_load_dwordx4 %1, %2, %3 offen lds"
      :
      : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff)
      : "memory", "m0");
}

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

#define DP_PIN() __builtin_amdgcn_sched_barrier(0)

// Tile t of the launch -> layer and tile origin.  Inside a layer, tiles are numbered so that
// 32 consecutive numbers form a patch of 4 tile rows x 8 tile columns and 8 consecutive
// patches form a 16 x 16 super-patch (clamped at the layer's edges): 32 compute units of one
// XCD then pull 12 operand panels per 32 tiles through that XCD's L2, and the 8 XCDs 32 panels
// per 256 tiles through the memory-side cache.
__device__ __forceinline__ void locate_tile(const GroupArgs& ga, int t, int& layer, int& m0, int& n0) {
  int l = 0;
  while (l + 1 < ga.n_layers && t >= ga.layer[l + 1].tile_begin) ++l;
  layer = l;
  const GroupLayer& ly = ga.layer[l];
  int rem = t - ly.tile_begin;
  const int tiles_m = (ly.d_in + BM - 1) / BM, tiles_n = (ly.d_out + BN - 1) / BN;
  const int sr = min(rem / (16 * tiles_n), (tiles_m - 1) / 16);      // super-patch row
  rem -= sr * 16 * tiles_n;
  const int hm = min(16, tiles_m - 16 * sr);
  const int sc = min(rem / (hm * 16), (tiles_n - 1) / 16);           // super-patch column
  rem -= sc * hm * 16;
  const int wn = min(16, tiles_n - 16 * sc);
  const int pr = min(rem / (4 * wn), (hm - 1) / 4);                  // patch row inside it
  rem -= pr * 4 * wn;
  const int ph = min(4, hm - 4 * pr);
  const int pc = min(rem / (ph * 8), (wn - 1) / 8);                  // patch column
  rem -= pc * ph * 8;
  m0 = (16 * sr + 4 * pr + rem % ph) * BM;
  n0 = (16 * sc + 8 * pc + rem / ph) * BN;
}

__global__ void __launch_bounds__(NT)
clipped_grad_big_kernel(const GroupArgs ga, const float* __restrict__ C_global) {
  // The weights do not change during the kernel: read them through the constant address space
  // so that they come by scalar loads (a vector load here would make the compiler wait for
  // every outstanding prefetch load at each sample boundary).
  const __attribute__((address_space(4))) float* C =
      (const __attribute__((address_space(4))) float*)(uintptr_t)C_global;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  const unsigned lds0 = (unsigned)(uintptr_t)lds_raw;

  // XCD-aware order.  Workgroup b runs on XCD b % 8 (round-robin dispatch) and about 256
  // consecutive ids are resident at a time.  Within each run of 256 ids, XCD x gets the x-th
  // group of 32 consecutive tile numbers, i.e. one 4 x 8 patch of locate_tile's numbering, and
  // the eight XCDs together one 16 x 16 super-patch.
  int logical;
  {
    constexpr int ROUND = 256;
    const int base = (blockIdx.x / ROUND) * ROUND, q = blockIdx.x - base;
    const int n = min(ROUND, ga.total_blocks - base);
    const int per = n >> 3, rest = n & 7, xcd = q & 7, idx = q >> 3;
    logical = base + (xcd < rest ? xcd * (per + 1) + idx : rest * (per + 1) + (xcd - rest) * per + idx);
  }
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
          acc[g][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cb][g].v, fb[cb][0].v, acc[g][0], 0, 0, 0);
          DP_PIN();
          if (fetch) read_frag(nb, 2 * g, r_stage, r_ks);
          DP_PIN();
          acc[g][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cb][g].v, fb[cb][1].v, acc[g][1], 0, 0, 0);
          DP_PIN();
          if (fetch) read_frag(nb, 2 * g + 1, r_stage, r_ks);
          DP_PIN();
          acc[g][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cb][g].v, fb[cb][2].v, acc[g][2], 0, 0, 0);
          DP_PIN();
          if (g & 1)
            prefetch_issue_b(ks * 2 + (g >> 1));
          else
            prefetch_issue_a(ks * 2 + (g >> 1));
          DP_PIN();
          acc[g][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cb][g].v, fb[cb][3].v, acc[g][3], 0, 0, 0);
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

  // epilogue: grad (+)= held * acc.  With no active sample the accumulator is zero.
  float* out = ly.out;
  auto store_tile = [&](auto acc_tag) {
    constexpr bool accumulate = decltype(acc_tag)::value;
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        const int col = n0 + wn + y * 32 + (lane & 31);
        float* base = out + (size_t)(m0 + wm + x * 32 + 4 * (lane >> 5)) * p + col;
        float old[16];
        if (accumulate) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int row = m0 + wm + x * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            old[r] = (row < d && col < p) ? base[(size_t)(8 * (r >> 2) + (r & 3)) * p] : 0.f;
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm + x * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const float v = acc[x][y][r] * held;
          if (row < d && col < p) base[(size_t)(8 * (r >> 2) + (r & 3)) * p] = accumulate ? old[r] + v : v;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
  };
  if (ga.accumulate)
    store_tile(std::true_type{});
  else
    store_tile(std::false_type{});
}

}  // namespace

int clipped_grad_big_tiles(int d, int p) { return ((d + BM - 1) / BM) * ((p + BN - 1) / BN); }

// The kernel addresses each sample's slab of a layer with 32-bit byte offsets and uses
// bit 31 as the "fetch zeros" marker, so a slab must be smaller than 2 GiB; k-blocks must
// not straddle samples, so T must be a multiple of the k-block.
bool clipped_grad_big_supports(int T, int d, int p) {
  return T % BK == 0 && (int64_t)T * d * 2 < (int64_t)1 << 31 && (int64_t)T * p * 2 < (int64_t)1 << 31;
}

dp_status launch_clipped_grad_big_group(const GroupArgs& ga, const float* C, hipStream_t s) {
  static bool ready = false;
  if (!ready) {
    dp_status st = hip_status(hipFuncSetAttribute(reinterpret_cast<const void*>(clipped_grad_big_kernel),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize,
                                                  LDS_BYTES));
    if (st != DP_OK) return st;
    ready = true;
  }
  hipLaunchKernelGGL(clipped_grad_big_kernel, dim3(ga.total_blocks), dim3(NT), LDS_BYTES, s, ga, C);
  return hip_status(hipGetLastError());
}

}  // namespace dpbk
