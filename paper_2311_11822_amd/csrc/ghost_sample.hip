// Ghost norm for sequences of 129 .. 256 tokens, one workgroup per sample (appendix A.1 of the
// paper, right side of eq. "mixed ghost norm"):
//     sqnorm[i] = sum_{t,t'} (a_t . a_t') (g_t . g_t').
//
// With 256 x 128 tiles (ghost_big.hip) a sample of up to 256 tokens takes two workgroups, which
// between them read the first 128 token rows twice, and at these sizes the kernel runs at the rate
// the memory system delivers the rows (every load misses L2: each workgroup reads rows nobody else
// reads).  Here one workgroup of eight waves holds the whole upper triangle of both Gram matrices
// of its sample, so every row of a and g is read exactly once.
//
// The 256 x 256 Gram matrix is cut into 64 x 64 sub-blocks (si, sj), sj >= si: six off the
// diagonal, one wave each (2 x 2 MFMA tiles of 32 x 32, counted twice), and four on it, two per
// wave (the three tiles (0,0), (0,1), (1,1) of each; (0,1) counted twice).  Every wave reads four
// 32-row fragments per k-step.  Data path as in ghost_big.hip's compact plan: five LDS stages of
// 256 rows x 64 k, rows go global -> LDS without passing through registers, chunks of 16 bytes
// XOR-swizzled by (row >> 1) & 7, rows past T fetched past the end of the sample's buffer
// descriptor (zeros), loads issued four k-blocks ahead across the a -> g switch.
#include <type_traits>

#include "dp_internal.h"
#include "lds_dma.h"

namespace dpbk {

namespace {

constexpr int ROWS = 256, BK = 64;
constexpr int NW = 8, NT = 64 * NW;
constexpr int ROW_BYTES = 128;                        // 64 bf16
constexpr int STAGE_BYTES = ROWS * ROW_BYTES;         // 32 KiB
constexpr int NSTAGE = 5;
constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;       // 160 KiB
constexpr int LOADS = ROWS / 8 / NW;                  // wave-loads (8 rows each) per wave and k-block: 4

__device__ __forceinline__ bf16x8 lds_read16(unsigned addr) {
  return *(__attribute__((address_space(3))) bf16x8*)(uintptr_t)addr;
}

template <bool F16>
__global__ void __launch_bounds__(NT)
ghost_sample_kernel(const GroupArgs ga, float* __restrict__ partials) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  const unsigned lds0 = (unsigned)(uintptr_t)lds_raw;
  const int l = layer_of(ga, blockIdx.x);
  const GroupLayer& ly = ga.layer[l];
  const int sample = blockIdx.x - ly.tile_begin;      // one workgroup per sample
  const int T = ly.T;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // The wave's sub-blocks.  Waves 0..5: the off-diagonal sub-block (si, sj); waves 6 and 7: the
  // diagonal sub-blocks si and sj.  Either way the wave's four fragments are the 32-row blocks at
  // rows 64 si, 64 si + 32, 64 sj, 64 sj + 32.
  const bool offd = wave < 6;
  const int si = wave == 0 || wave == 1 || wave == 2 || wave == 6 ? 0 : (wave == 3 || wave == 4 ? 1 : 2);
  const int sj = wave == 0 || wave == 6 ? 1 : (wave == 1 || wave == 3 ? 2 : 3);
  unsigned frag_org[4];
  frag_org[0] = (64 * si) * ROW_BYTES;
  frag_org[1] = (64 * si + 32) * ROW_BYTES;
  frag_org[2] = (64 * sj) * ROW_BYTES;
  frag_org[3] = (64 * sj + 32) * ROW_BYTES;

  // ---- prefetch stream ---------------------------------------------------------------
  // Wave-load j of a wave covers rows (wave * LOADS + j) * 8 + (lane >> 3); the lane's LDS chunk
  // (lane & 7) holds logical chunk (lane & 7) ^ ((row >> 1) & 7).
  const int nka = ly.d_in / BK, nkg = ly.d_out / BK, nblocks = nka + nkg;
  unsigned vi[LOADS];
  i32x4 rs;
  auto set_operand = [&](const void* base, int width) {
    const unsigned slab = (unsigned)T * width * 2u;
    rs = make_rsrc(static_cast<const unsigned char*>(base) + (size_t)sample * slab, slab);
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int row = (wave * LOADS + j) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      vi[j] = (unsigned)row * width * 2u + chunk * 16u;             // rows >= T: past the slab -> zeros
    }
  };
  int p_blk = 0, p_stage = 0;
  unsigned p_soff = 0;
  const unsigned ld_base = lds0 + wave * LOADS * 1024;
  set_operand(ly.a, ly.d_in);
  auto issue = [&](int j) { load_to_lds(rs, vi[j], p_soff, ld_base + p_stage * STAGE_BYTES + j * 1024); };
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
      for (int j = 0; j < LOADS; ++j) vi[j] = 0x80000000u;
      p_soff = 0;
    }
  };

  // ---- LDS -> MFMA operand addressing ---------------------------------------------------
  // lane: row (lane & 31) of a 32-row fragment, k-chunk 2*ks + (lane >> 5); swizzle
  // (row >> 1) & 7 = (lane >> 1) & 7 because fragment origins are multiples of 32 rows.
  unsigned rd[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    rd[ks] = lds0 + (lane & 31) * ROW_BYTES + (((2 * ks + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4);

  // Tile t of the wave: off-diagonal waves use tiles 0..3 = fragments (0,2), (0,3), (1,2), (1,3);
  // diagonal waves tiles 0..5 = (0,0), (0,1), (1,1), (2,2), (2,3), (3,3).
  f32x16 sa[6], sg[6];
#pragma unroll
  for (int t = 0; t < 6; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      sa[t][r] = 0.f;
      sg[t][r] = 0.f;
    }
  bf16x8 f[2][4];
  auto read_frag = [&](int buf, int q, int stage, int ks) {
    f[buf][q] = lds_read16(rd[ks] + stage * STAGE_BYTES + frag_org[q]);
  };

  for (int s = 0; s < NSTAGE - 1; ++s) {
#pragma unroll
    for (int j = 0; j < LOADS; ++j) issue(j);
    advance();
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * LOADS) : "memory");
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 4; ++q) read_frag(0, q, 0, 0);
  int c_stage = 0;
  // One k-block: wait for own loads of block kb + 1, barrier (block kb + 1 in LDS, block kb - 1 no
  // longer read), then four k-steps; in each, the wave's MFMAs with the fragment reads of the
  // next k-step (the first one of block kb + 1 at the end) and one load of block kb + 4 in their
  // shadow.  The fragments read during the very last k-step are never used.
  auto block = [&](f32x16 (&acc)[6], auto offd_tag) {
    constexpr bool OFFD = decltype(offd_tag)::value;
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 3) * LOADS) : "memory");
    __builtin_amdgcn_s_barrier();
    const int n_stage = c_stage + 1 == NSTAGE ? 0 : c_stage + 1;
    DP_PIN();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int cb = ks & 1, nb = cb ^ 1;
      const int r_stage = ks < 3 ? c_stage : n_stage, r_ks = ks < 3 ? ks + 1 : 0;
      if (OFFD) {
        acc[0] = mfma16<F16>(f[cb][0], f[cb][2], acc[0]);
        DP_PIN();
        read_frag(nb, 0, r_stage, r_ks);
        DP_PIN();
        acc[1] = mfma16<F16>(f[cb][0], f[cb][3], acc[1]);
        DP_PIN();
        read_frag(nb, 1, r_stage, r_ks);
        issue(ks);
        DP_PIN();
        acc[2] = mfma16<F16>(f[cb][1], f[cb][2], acc[2]);
        DP_PIN();
        read_frag(nb, 2, r_stage, r_ks);
        DP_PIN();
        acc[3] = mfma16<F16>(f[cb][1], f[cb][3], acc[3]);
        DP_PIN();
        read_frag(nb, 3, r_stage, r_ks);
        DP_PIN();
      } else {
        acc[0] = mfma16<F16>(f[cb][0], f[cb][0], acc[0]);
        DP_PIN();
        acc[1] = mfma16<F16>(f[cb][0], f[cb][1], acc[1]);
        DP_PIN();
        read_frag(nb, 0, r_stage, r_ks);
        DP_PIN();
        acc[2] = mfma16<F16>(f[cb][1], f[cb][1], acc[2]);
        DP_PIN();
        read_frag(nb, 1, r_stage, r_ks);
        issue(ks);
        DP_PIN();
        acc[3] = mfma16<F16>(f[cb][2], f[cb][2], acc[3]);
        DP_PIN();
        acc[4] = mfma16<F16>(f[cb][2], f[cb][3], acc[4]);
        DP_PIN();
        read_frag(nb, 2, r_stage, r_ks);
        DP_PIN();
        acc[5] = mfma16<F16>(f[cb][3], f[cb][3], acc[5]);
        DP_PIN();
        read_frag(nb, 3, r_stage, r_ks);
        DP_PIN();
      }
    }
    advance();
    c_stage = n_stage;
  };
  if (offd) {
    for (int kb = 0; kb < nka; ++kb) block(sa, std::true_type{});
    for (int kb = 0; kb < nkg; ++kb) block(sg, std::true_type{});
  } else {
    for (int kb = 0; kb < nka; ++kb) block(sa, std::false_type{});
    for (int kb = 0; kb < nkg; ++kb) block(sg, std::false_type{});
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // Token rows/columns past T were fetched as zeros: their Gram entries are zero.
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 6; ++t) {
    float st = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) st = fmaf(sa[t][r], sg[t][r], st);
    // off-diagonal sub-blocks count twice (both Gram matrices are symmetric); in a diagonal
    // sub-block the tiles (0,0) and (1,1) lie on the diagonal and (0,1) above it
    const float w = offd ? (t < 4 ? 2.f : 0.f) : (t == 1 || t == 4 ? 2.f : 1.f);
    s = fmaf(w, st, s);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  __syncthreads();                                    // every wave is done with the stages
  float* red = reinterpret_cast<float*>(lds_raw);
  if (lane == 0) red[wave] = s;
  __syncthreads();
  if (tid == 0)
    partials[ly.part_begin + sample] = ((red[0] + red[1]) + (red[2] + red[3])) + ((red[4] + red[5]) + (red[6] + red[7]));
}

template <bool F16>
dp_status launch_t(const GroupArgs& ga, float* partials, hipStream_t s) {
  static ReadyTable ready;
  auto kernel = ghost_sample_kernel<F16>;
  dp_status st = allow_big_lds(kernel, LDS_BYTES, ready);
  if (st != DP_OK) return st;
  hipLaunchKernelGGL(kernel, dim3(ga.total_blocks), dim3(NT), LDS_BYTES, s, ga, partials);
  return hip_status(hipGetLastError());
}

}  // namespace

// Whole 64-wide k-blocks, 129 .. 256 tokens, 32-bit byte offsets inside a sample's slab.
bool ghost_sample_supports(int T, int d, int p) {
  return T > 128 && T <= ROWS && d % BK == 0 && p % BK == 0 && (int64_t)(T + ROWS) * d * 2 < (int64_t)1 << 31 &&
         (int64_t)(T + ROWS) * p * 2 < (int64_t)1 << 31;
}

// ga.layer[j]: tile_begin = first workgroup, tiles_per_sample = 1, part_begin = first partial-sum slot.
dp_status launch_ghost_sample_group(const GroupArgs& ga, float* partials, hipStream_t s) {
  return ga.f16 ? launch_t<true>(ga, partials, s) : launch_t<false>(ga, partials, s);
}

}  // namespace dpbk
