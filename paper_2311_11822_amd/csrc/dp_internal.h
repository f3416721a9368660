// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "dp_bk.h"
#include "philox.h"

namespace dpbk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define DP_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))

// One 32x32x16 matrix-core step on 16-bit operands with fp32 accumulation.  The kernels move
// operands as opaque 16-bit values (typed bf16x8 for convenience); F16 says the bits are IEEE
// binary16 rather than bfloat16, which only changes the instruction that multiplies them.
template <bool F16>
__device__ __forceinline__ f32x16 mfma16(bf16x8 a, bf16x8 b, f32x16 c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b),
                                                  c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Up to this many layers travel in one launch's kernel arguments.  (Larger groups work - the
// runtime takes 16 KiB of kernel arguments - but a single launch of cfg2's 144 layers measured
// 1 % slower in the gradient than three launches of 48, and no faster in the norms.)
constexpr int kMaxGroup = 48;

// One layer of a grouped launch.  tile_begin is the first workgroup of the layer.
struct GroupLayer {
  const void* a;
  const void* g;
  float* out;       // gradient [d_in, d_out] (clipped_grad) or unused
  int T, d_in, d_out;
  int path;
  int tile_begin;   // first block index that belongs to this layer
  int sq_index;     // layer number within the caller's stack (row of sqnorm)
  int part_begin;   // first partial-sum slot of this layer in the workspace
  int tiles_per_sample;
  int c_off;        // gradient kernels: this layer's weights are C[c_off + i] (its clipping group)
};

struct GroupArgs {
  int n_layers;
  int total_blocks;
  int B;
  int accumulate;
  int f16;          // operands are IEEE binary16 (else bfloat16)
  GroupLayer layer[kMaxGroup];
};

// Noise added in the epilogue of the large-tile gradient kernels (eq. (1) of the paper):
// element j of layer l's gradient has global index layer_off[l] + j and receives
// stddev * z_index when lo <= index < hi.  stddev == 0 switches the noise off.
struct NoiseArgs {
  float stddev;
  uint32_t step_lo, step_hi;
  uint64_t lo, hi;
  RoundKeys rk;
  uint64_t layer_off[kMaxGroup];
};

// The layer that owns workgroup (or tile) number `id`: the last one whose tile_begin is <= id.
__device__ __forceinline__ int layer_of(const GroupArgs& ga, int id) {
  int lo = 0, hi = ga.n_layers - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (id >= ga.layer[mid].tile_begin)
      lo = mid;
    else
      hi = mid - 1;
  }
  return lo;
}

// The fp32 norm kernels run one workgroup per sample on the vector ALUs; layers whose norm needs
// more multiply-adds per sample than this are refused (DP_ERR_UNSUPPORTED) instead of running
// for seconds.  2^28 multiply-adds take a few tens of milliseconds.
constexpr int64_t kF32MaxWork = (int64_t)1 << 28;

inline dp_status hip_status(hipError_t e) { return e == hipSuccess ? DP_OK : DP_ERR_HIP; }

// Kernels that need more than 64 KiB of LDS must be told so once per device; `done` is the
// caller's per-kernel table of devices already prepared.  These tables are the library's only
// mutable host state: flags that go from false to true once, so two threads that race on one at
// worst both make the (idempotent) attribute call.
constexpr int kMaxDevices = 64;
using ReadyTable = std::atomic<bool>[kMaxDevices];
template <class K>
dp_status allow_big_lds(K kernel, int bytes, ReadyTable& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DP_ERR_HIP;
  if (done[dev].load(std::memory_order_acquire)) return DP_OK;
  dp_status st = hip_status(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  if (st == DP_OK) done[dev].store(true, std::memory_order_release);
  return st;
}

// --- launchers implemented in the .hip files (all validate nothing; callers did) ---
dp_status launch_noise(float* grad, uint64_t global_offset, uint64_t count, float stddev,
                       uint64_t seed, uint64_t step, hipStream_t s);
dp_status launch_philox_blocks(uint32_t* out, uint64_t first_block, uint64_t n_blocks,
                               uint64_t seed, uint64_t step, hipStream_t s);
dp_status launch_clip_factors(const float* sqnorm, int L, int B, int mode, float R, float stability,
                              float* C_out, float* norm_out, hipStream_t s);
dp_status launch_clip_factors_grouped(const float* sqnorm, int B, const int32_t* group_begin, int M,
                                      const float* R, int mode, float stability, float* C_out,
                                      float* norm_out, hipStream_t s);
dp_status launch_bias_norm(const void* g, dp_dtype dt, int B, int T, int p, float* colsum,
                           float* sqnorm_out, hipStream_t s);
dp_status launch_clipped_bias_grad(const float* colsum, int B, int p, const float* C, float* grad_b,
                                   int accumulate, hipStream_t s);

dp_status launch_ghost_f32(const float* a, const float* g, int B, int T, int d, int p, float* out,
                           hipStream_t s);
dp_status launch_perex_f32(const float* a, const float* g, int B, int T, int d, int p, float* out,
                           hipStream_t s);
dp_status launch_clipped_grad_f32(const float* a, const float* g, int B, int T, int d, int p,
                                  const float* C, float* grad, int accumulate, hipStream_t s);

// bf16 MFMA kernels, grouped over layers.
int ghost_tiles_per_sample(int T);
int perex_tiles_per_sample(int d, int p);
int clipped_grad_tiles(int d, int p);
dp_status launch_ghost_group(const GroupArgs& ga, float* partials, hipStream_t s);
dp_status launch_perex_group(const GroupArgs& ga, float* partials, hipStream_t s);
// Same tiles and partial-sum slots with direct global->LDS loads, three k-blocks ahead (perex_dma.hip).
bool perex_dma_supports(int T, int d, int p);
dp_status launch_perex_dma_group(const GroupArgs& ga, float* partials, hipStream_t s);
dp_status launch_norm_reduce_group(const GroupArgs& ga, const float* partials, float* sqnorm_out,
                                   hipStream_t s);
dp_status launch_clipped_grad_group(const GroupArgs& ga, const float* C, hipStream_t s);
// 256x128-tile ghost-norm kernel with direct global->LDS loads (ghost_big.hip).
int ghost_big_tiles_per_sample(int T);
bool ghost_big_supports(int T, int d, int p);
dp_status launch_ghost_big_group(const GroupArgs& ga, float* partials, hipStream_t s);
// Whole-sample ghost-norm kernel for 129 .. 256 tokens (ghost_sample.hip): one workgroup and one
// partial sum per sample.
bool ghost_sample_supports(int T, int d, int p);
dp_status launch_ghost_sample_group(const GroupArgs& ga, float* partials, hipStream_t s);
// 256x256-tile kernel with direct global->LDS loads (grad_gemm.hip).
int clipped_grad_big_tiles(int d, int p);
// Of a launch of n large tiles, how many (the last ones) go to the sub-tile kernel.
int clipped_grad_big_tail_tiles(int n);
bool clipped_grad_big_supports(int T, int d, int p);
// noise == nullptr: gradients only.  out16: the layers' `out` pointers address 16-bit arrays of the
// operands' storage type (bf16 or fp16) instead of fp32.
dp_status launch_clipped_grad_big_group(const GroupArgs& ga, const float* C, const NoiseArgs* noise,
                                        hipStream_t s, bool out16 = false);

// Clip-weighted sum of kept per-sample gradients (kept.hip).  ga.layer[j]: a = kept [B, d * p] fp32,
// out = grad, tile_begin = first workgroup (kept_blocks(d, p) per layer), c_off; noise as NoiseArgs,
// layer_off[j] == ~0 switching it off for layer j.
int kept_blocks(int d, int p);
dp_status launch_kept_weighted_sum(const GroupArgs& ga, const float* C, const NoiseArgs& na, hipStream_t s);

// Layer-wise clipping in one pass for layers that fit one workgroup tile (layerwise.hip).
// Shape class of a d x p layer (0: up to 128 x 128, 1: up to 512 x 32, 2: up to 32 x 512), or -1.
int layerwise_fused_shape(int d, int p);
// ga.layer[j]: tile_begin = first workgroup, tiles_per_sample = sample chunks, part_begin = float
// offset of the layer's [chunks][d * p] sums in `partial`, sq_index = row of sqnorm / C_out.
dp_status launch_layerwise_fused(int shape, const GroupArgs& ga, const float* R, int mode, float stability,
                                 float* partial, float* sqnorm, float* C_out, hipStream_t s);
// ga.layer[j].out (+)= the layer's chunks added in order (+ noise when na.stddev != 0).
dp_status launch_layerwise_reduce(const GroupArgs& ga, const float* partial, const NoiseArgs& na, hipStream_t s);

}  // namespace dpbk
