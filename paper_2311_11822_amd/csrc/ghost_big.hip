// Ghost norm on the matrix cores, large-tile kernel (appendix A.1 of the paper, right side of
// eq. "mixed ghost norm"):  sqnorm[i] = sum_{t,t'} (a_t . a_t') (g_t . g_t')  for sample i.
//
// One workgroup owns a 256 x 128 tile (token rows [256 I, +256), token columns [128 J, +128),
// J >= 2 I) of both T x T Gram matrices of one sample: it accumulates the tile of a a^T over
// d_in, then the tile of g g^T over d_out, in two accumulator sets (4 waves x 128 x 64 x 2 sets
// = all 256 accumulator registers per lane), multiplies them element by element and reduces to
// one partial sum.  Both Gram matrices are symmetric, so 128 x 128 sub-blocks above the
// diagonal count twice and diagonal ones once.  The first tile of a tile row (J = 2I) holds one
// diagonal sub-block and one below the diagonal, which is not needed: that tile runs in
// "diagonal mode", the four waves sharing its one 128 x 128 sub-block (64 x 64 each), with half
// the loads and half the MFMAs of a full tile.  No T x T matrix is written to memory.
//
// Data path (same machinery as the gradient kernel in grad_gemm.hip): operand rows go from
// global memory to LDS without passing through registers (buffer_load ... lds), three stages
// of 64 k each, issued two k-blocks ahead across the a -> g switch; rows are k-contiguous
// in memory, in LDS and in the MFMA operand, so fragments come back with plain 128-bit LDS
// reads.  A wave's load lands as eight consecutive 128-byte rows, so rows cannot be padded;
// the 16-byte chunks of row r are XOR-swizzled by (r >> 1) & 7, which makes 16 consecutive
// rows of one k-chunk hit 16 different bank groups.  Token rows past T are fetched past the
// end of the sample's buffer descriptor and arrive as zeros.  When the column block lies
// inside the row block (J = 2I or 2I+1, always the case for T <= 256) it is not loaded again.
#include <type_traits>

#include "dp_internal.h"
#include "lds_dma.h"
#include "tile_order.h"

namespace dpbk {

namespace {

constexpr int TI = 256, TJ = 128, BK = 64;
constexpr int NT = 256;
constexpr int ROW_BYTES = 128;                       // 64 bf16
constexpr int I_BYTES = TI * ROW_BYTES;              // 32 KiB
constexpr int J_BYTES = TJ * ROW_BYTES;              // 16 KiB
// Two LDS plans.  General: 3 stages of row block + column block (144 KiB).  Compact, for
// launches whose layers all have T <= 256 (every column block lies inside its row block):
// 5 stages of the row block alone (160 KiB), which buys a deeper prefetch and lets the
// fragment reads run across the barrier.
template <bool COMPACT>
struct Plan {
  static constexpr int STAGE_BYTES = COMPACT ? I_BYTES : I_BYTES + J_BYTES;
  static constexpr int NSTAGE = COMPACT ? 5 : 3;
  static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
};
constexpr int LOADS_I = 8, LOADS_J = 4;              // per wave per k-block (a wave-load = 8 rows)

__device__ __forceinline__ bf16x8 lds_read16(unsigned addr) {
  return *(__attribute__((address_space(3))) bf16x8*)(uintptr_t)addr;
}

// After which MFMA of a k-step (2 MI MFMAs) load x of its per_ks global->LDS loads is issued.
constexpr int load_slot(int mi, int per_ks, int x) {
  if (mi == 2) return 2;                                       // 4 MFMAs, one load
  if (per_ks == 3) return x == 0 ? 3 : (x == 1 ? 5 : 6);       // 8 MFMAs, three loads
  return x == 0 ? 3 : 6;                                       // 8 MFMAs, two loads
}

template <bool COMPACT, bool F16>
__global__ void __launch_bounds__(NT)
ghost_big_kernel(const GroupArgs ga, float* __restrict__ partials) {
  constexpr int STAGE_BYTES = Plan<COMPACT>::STAGE_BYTES, NSTAGE = Plan<COMPACT>::NSTAGE;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  const unsigned lds0 = (unsigned)(uintptr_t)lds_raw;

  // XCD-aware order of the launch's tiles and of a layer's tiles: see tile_order.h.
  const int logical = ghost_logical_tile(blockIdx.x, ga.total_blocks);
  const int l = layer_of(ga, logical);
  const GroupLayer& ly = ga.layer[l];
  const int T = ly.T;
  const GhostTile gt = ghost_tile_of(T, ly.tiles_per_sample, logical - ly.tile_begin);
  const int sample = gt.sample, I = gt.I, J = gt.J;
  const int q = J - 2 * I;                        // position in the tile row: 0 holds the diagonal
  const int r0 = I * TI, c0 = J * TJ;
  const bool inside = q < 2;                      // column block is one half of the row block

  const bool diag = q == 0;                       // only the sub-block (2I, 2I) is needed

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // full tile: waves 2 x 2 of 128 x 64; diagonal mode: 2 x 2 of 64 x 64 on rows [r0, r0 + 128)
  const int wm = (wave >> 1) * (diag ? 64 : 128), wn = (wave & 1) * 64;
  // weight of this wave's sub-block: above the diagonal twice, on it once (a full tile has
  // J >= 2I + 1, so none of its two sub-block rows 2I, 2I + 1 lies below the diagonal)
  const float weight = (!diag && J > 2 * I + (wave >> 1)) ? 2.f : 1.f;
  const int li = diag ? LOADS_I / 2 : LOADS_I;    // wave-loads of the row block per wave and k-block

  // ---- prefetch stream ---------------------------------------------------------------
  // Wave-load j of the row block covers rows (wave*8 + j)*8 + (lane >> 3); the lane's LDS chunk
  // (lane & 7) holds logical chunk (lane & 7) ^ ((row >> 1) & 7).  Same for the column block
  // with wave*4 + j.
  const int nka = ly.d_in / BK, nkg = ly.d_out / BK, nblocks = nka + nkg;
  unsigned vi[LOADS_I], vj[LOADS_J];
  i32x4 rs;
  auto set_operand = [&](const void* base, int width) {
    const unsigned slab = (unsigned)T * width * 2u;
    rs = make_rsrc(static_cast<const unsigned char*>(base) + (size_t)sample * slab, slab);
#pragma unroll
    for (int j = 0; j < LOADS_I; ++j) {
      const int row = (wave * li + j) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      vi[j] = (unsigned)(r0 + row) * width * 2u + chunk * 16u;     // rows >= T: past the slab -> zeros
    }
#pragma unroll
    for (int j = 0; j < LOADS_J; ++j) {
      const int row = (wave * LOADS_J + j) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      vj[j] = (unsigned)(c0 + row) * width * 2u + chunk * 16u;
    }
  };
  int p_blk = 0, p_stage = 0;
  unsigned p_soff = 0;
  // this wave's first LDS destination inside a stage, row block and column block
  const unsigned ld_i = lds0 + wave * li * 1024, ld_j = lds0 + I_BYTES + wave * LOADS_J * 1024;
  set_operand(ly.a, ly.d_in);
  // item in 0 .. LOADS_I + LOADS_J - 1: one wave-load of the row block or of the column block
  auto issue = [&](int item, bool with_j) {
    if (item < LOADS_I)
      load_to_lds(rs, vi[item], p_soff, ld_i + p_stage * STAGE_BYTES + item * 1024);
    else if (with_j)
      load_to_lds(rs, vj[item - LOADS_I], p_soff, ld_j + p_stage * STAGE_BYTES + (item - LOADS_I) * 1024);
  };
  auto advance = [&]() {
    ++p_blk;
    p_soff += BK * 2;
    p_stage = p_stage + 1 == NSTAGE ? 0 : p_stage + 1;
    if (p_blk == nka) {
      set_operand(ly.g, ly.d_out);
      p_soff = 0;
    } else if (p_blk == nblocks) {
      // past the end of the stream: keep issuing (the waits count loads) but fetch nothing
#pragma unroll
      for (int j = 0; j < LOADS_I; ++j) vi[j] = 0x80000000u;
#pragma unroll
      for (int j = 0; j < LOADS_J; ++j) vj[j] = 0x80000000u;
      p_soff = 0;
    }
  };

  // ---- LDS -> MFMA operand addressing ---------------------------------------------------
  // lane: row (lane & 31) of a 32-row MFMA tile, k-chunk 2*ks + (lane >> 5); swizzle
  // (row >> 1) & 7 = (lane >> 1) & 7 because tile origins are multiples of 16 rows.
  unsigned rd[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    rd[ks] = lds0 + (lane & 31) * ROW_BYTES + (((2 * ks + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4);
  const unsigned a_org = wm * ROW_BYTES;
  const unsigned b_org = (inside ? (J - 2 * I) * TJ * ROW_BYTES : I_BYTES) + wn * ROW_BYTES;

  f32x16 sa[4][2], sg[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        sa[i][j][r] = 0.f;
        sg[i][j][r] = 0.f;
      }

  bf16x8 fa[2][4], fb[2][2];
  // item 0,1: column-block fragments; 2..: row-block fragments (needed in that order)
  auto read_frag = [&](int buf, int item, int stage, int ks) {
    const unsigned o = rd[ks] + stage * STAGE_BYTES;
    if (item < 2)
      fb[buf][item] = lds_read16(o + b_org + item * 32 * ROW_BYTES);
    else
      fa[buf][item - 2] = lds_read16(o + a_org + (item - 2) * 32 * ROW_BYTES);
  };

  // Loads per k-block differ (12 for a full tile, 8 when its column block is inside the row
  // block, 4 in diagonal mode) and so do the MFMAs per k-step (2 MI, with MI = 4 or 2 row tiles
  // per wave); the vmcnt immediates and the interleave must be constants, hence separate
  // instantiations of the loop.
  //
  // General plan: a wave waits for its own loads of block m, meets the others at one barrier
  // (block m is in LDS, block m-1 has been read), and runs the MFMAs with the loads of block
  // m+2 (into the stage of block m-1) and the fragment reads of the next k-step in their shadow.
  // A load has two iterations to land.
  auto run = [&](auto inside_tag, auto mi_tag) {
    constexpr bool ins = decltype(inside_tag)::value;
    constexpr int MI = decltype(mi_tag)::value;
    constexpr int LI = 2 * MI;                                  // row-block wave-loads per k-block
    constexpr int PER = ins ? LI : LI + LOADS_J;
    constexpr int PER_KS = PER / 4;                             // loads issued per k-step
    static_assert(ins || MI == 4, "diagonal mode never loads a column block");
    // load number x (0 .. PER-1) of a k-block
    auto issue_nth = [&](int x) {
      if (x < LI)
        issue(x, false);
      else
        issue(LOADS_I + x - LI, true);
    };
    for (int s = 0; s < NSTAGE - 1; ++s) {
#pragma unroll
      for (int x = 0; x < PER; ++x) issue_nth(x);
      advance();
    }
    int c_stage = 0;
    // One k-step: 2 MI MFMAs on fragment buffer KS & 1, with the fragment reads of the following
    // k-step (k-step r_ks of the block in r_stage) and the loads of window position POS in
    // their shadow.
    auto kstep = [&](f32x16 (&acc)[4][2], auto ks_tag, auto pos_tag, bool fetch, int r_stage, int r_ks) {
      constexpr int KS = decltype(ks_tag)::value, POS = decltype(pos_tag)::value;
      constexpr int cb = KS & 1, nb = cb ^ 1;
#pragma unroll
      for (int n = 0; n < 2 * MI; ++n) {
        const int i = n >> 1, j = n & 1;
        acc[i][j] = mfma16<F16>(fa[cb][i], fb[cb][j], acc[i][j]);
        DP_PIN();
        if (fetch && n < 2 + MI) read_frag(nb, n, r_stage, r_ks);
        if (POS >= 0) {
#pragma unroll
          for (int x = 0; x < PER_KS; ++x)
            if (n == load_slot(MI, PER_KS, x)) issue_nth((POS < 0 ? 0 : POS) * PER_KS + x);
        }
        DP_PIN();
      }
    };
    using K0 = std::integral_constant<int, 0>;
    using K1 = std::integral_constant<int, 1>;
    using K2 = std::integral_constant<int, 2>;
    using K3 = std::integral_constant<int, 3>;
    using NoLoads = std::integral_constant<int, -1>;
    // The barrier that certifies block m sits before the last k-step of block m-1, whose
    // fragments are in registers by then, so the first fragments of block m are read during
    // those MFMAs and no LDS latency is exposed at the block boundary.  The loads of block m+2
    // (into the stage of block m-1, which nobody reads any more) follow the barrier, spread over
    // that k-step and the first three of block m.
    // first block: its first fragments are the one exposed LDS latency of the tile
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * PER) : "memory");
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int it = 0; it < 2 + MI; ++it) read_frag(0, it, 0, 0);
#pragma unroll
    for (int x = 0; x < PER_KS; ++x) issue_nth(x);              // window position 0 has no MFMAs yet
    DP_PIN();
    kstep(sa, K0{}, K1{}, true, 0, 1);
    kstep(sa, K1{}, K2{}, true, 0, 2);
    kstep(sa, K2{}, K3{}, true, 0, 3);
    advance();
    auto iter = [&](f32x16 (&acc_old)[4][2], f32x16 (&acc_new)[4][2]) {
      const int n_stage = c_stage + 1 == NSTAGE ? 0 : c_stage + 1;
      // own loads of block m landed; own fragment reads of block m-1 returned (the loads that
      // follow the barrier overwrite that block's stage)
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((NSTAGE - 2) * PER) : "memory");
      __builtin_amdgcn_s_barrier();
      DP_PIN();
      kstep(acc_old, K3{}, K0{}, true, n_stage, 0);
      kstep(acc_new, K0{}, K1{}, true, n_stage, 1);
      kstep(acc_new, K1{}, K2{}, true, n_stage, 2);
      kstep(acc_new, K2{}, K3{}, true, n_stage, 3);
      advance();
      c_stage = n_stage;
    };
    for (int m = 1; m < nka; ++m) iter(sa, sa);
    iter(sa, sg);
    for (int m = nka + 1; m < nblocks; ++m) iter(sg, sg);
    kstep(sg, K3{}, NoLoads{}, false, 0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };
  // Compact plan, iteration kb: wait for own loads of block kb+1, barrier (block kb+1 in LDS,
  // block kb-1 no longer read), issue block kb+4, the MFMAs; the fragments of the next k-step,
  // including the first one of block kb+1, are read during the MFMAs.  Three iterations per load.
  auto run_compact = [&](auto mi_tag) {
    constexpr int MI = decltype(mi_tag)::value;
    constexpr int PER = 2 * MI, PER_KS = PER / 4;
    for (int s = 0; s < NSTAGE - 1; ++s) {
#pragma unroll
      for (int it = 0; it < PER; ++it) issue(it, false);
      advance();
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * PER) : "memory");
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 2 + MI; ++it) read_frag(0, it, 0, 0);
    int c_stage = 0;
    auto block = [&](f32x16 (&acc)[4][2], auto last_tag) {
      constexpr bool last = decltype(last_tag)::value;
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 3) * PER) : "memory");
      __builtin_amdgcn_s_barrier();
      const int n_stage = c_stage + 1 == NSTAGE ? 0 : c_stage + 1;
      DP_PIN();
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int cb = ks & 1, nb = cb ^ 1;
        const bool fetch = ks < 3 || !last;
        const int r_stage = ks < 3 ? c_stage : n_stage, r_ks = ks < 3 ? ks + 1 : 0;
#pragma unroll
        for (int n = 0; n < 2 * MI; ++n) {
          const int i = n >> 1, j = n & 1;
          acc[i][j] = mfma16<F16>(fa[cb][i], fb[cb][j], acc[i][j]);
          DP_PIN();
          if (fetch && n < 2 + MI) read_frag(nb, n, r_stage, r_ks);
#pragma unroll
          for (int x = 0; x < PER_KS; ++x)
            if (n == load_slot(MI, PER_KS, x)) issue(ks * PER_KS + x, false);
          DP_PIN();
        }
      }
      advance();
      c_stage = n_stage;
    };
    for (int kb = 0; kb < nka; ++kb) block(sa, std::false_type{});
    for (int kb = 0; kb + 1 < nkg; ++kb) block(sg, std::false_type{});
    block(sg, std::true_type{});
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };
  using Full = std::integral_constant<int, 4>;
  using Half = std::integral_constant<int, 2>;
  if (COMPACT) {
    if (diag)
      run_compact(Half{});
    else
      run_compact(Full{});
  } else if (diag) {
    run(std::true_type{}, Half{});
  } else if (inside) {
    run(std::true_type{}, Full{});
  } else {
    run(std::false_type{}, Full{});
  }

  // Token rows/columns past T were fetched as zeros: their Gram entries are zero.
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s = fmaf(sa[i][j][r], sg[i][j][r], s);
  s *= weight;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  __syncthreads();                                  // every wave is done with the stages
  float* red = reinterpret_cast<float*>(lds_raw);
  if (lane == 0) red[wave] = s;
  __syncthreads();
  if (tid == 0) partials[ly.part_begin + gt.slot] = (red[0] + red[1]) + (red[2] + red[3]);
}

}  // namespace

int ghost_big_tiles_per_sample(int T) {
  const int nj = (T + TJ - 1) / TJ, ni = (T + TI - 1) / TI;
  int n = 0;
  for (int I = 0; I < ni; ++I) n += nj - 2 * I;
  return n;
}

// Needs whole 64-wide k-blocks and 32-bit byte offsets inside a sample's slab.
bool ghost_big_supports(int T, int d, int p) {
  return d % BK == 0 && p % BK == 0 && (int64_t)(T + TI) * d * 2 < (int64_t)1 << 31 &&
         (int64_t)(T + TI) * p * 2 < (int64_t)1 << 31;
}

template <bool COMPACT, bool F16>
dp_status launch_plan(const GroupArgs& ga, float* partials, hipStream_t s) {
  static ReadyTable ready;
  auto kernel = ghost_big_kernel<COMPACT, F16>;
  dp_status st = allow_big_lds(kernel, Plan<COMPACT>::LDS_BYTES, ready);
  if (st != DP_OK) return st;
  hipLaunchKernelGGL(kernel, dim3(ga.total_blocks), dim3(NT), Plan<COMPACT>::LDS_BYTES, s, ga, partials);
  return hip_status(hipGetLastError());
}

dp_status launch_ghost_big_group(const GroupArgs& ga, float* partials, hipStream_t s) {
  bool compact = true;
  for (int l = 0; l < ga.n_layers; ++l) compact = compact && ga.layer[l].T <= TI;
  if (ga.f16) return compact ? launch_plan<true, true>(ga, partials, s) : launch_plan<false, true>(ga, partials, s);
  return compact ? launch_plan<true, false>(ga, partials, s) : launch_plan<false, false>(ga, partials, s);
}

}  // namespace dpbk
