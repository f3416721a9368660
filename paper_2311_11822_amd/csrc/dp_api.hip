// Host side of the C ABI: argument validation, grouping of layers into launches.
// No device code lives here and no device memory is allocated.
#include <math.h>
#include <algorithm>
#include <vector>

#include "dp_internal.h"
#include "tile_order.h"

using namespace dpbk;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#ifndef DP_PEREX_DMA
#define DP_PEREX_DMA true
#endif

bool dtype_ok(dp_dtype dt) { return dt == DP_F32 || dt == DP_BF16 || dt == DP_F16; }

bool dims_ok(dp_dtype dt, int B, int T, int d, int p) {
  if (B <= 0 || T <= 0 || d <= 0 || p <= 0) return false;
  if (dt != DP_F32 && ((d & 7) || (p & 7))) return false;      // 16-bit rows must be 16-byte multiples
  // index arithmetic inside the kernels is 64-bit for element offsets, 32-bit per dimension
  if ((int64_t)B * T > INT32_MAX) return false;
  return true;
}

dp_status check_layer_ptrs(const void* a, const void* g) {
  if (!a || !g) return DP_ERR_INVALID_ARG;
  if (!aligned16(a) || !aligned16(g)) return DP_ERR_INVALID_ARG;
  return DP_OK;
}

// Ghost layers with whole 64-wide k-blocks and more than a handful of tokens take the
// large-tile kernel; the rest take the 128x128-tile kernel with per-chunk edge handling.
bool ghost_uses_big(const dp_layer& ly) {
  return ly.T >= 96 && ghost_big_supports(ly.T, ly.d_in, ly.d_out);
}

// Samples of 129 .. 256 tokens take the kernel that holds a whole sample in one workgroup.
bool ghost_uses_sample(const dp_layer& ly) { return ghost_sample_supports(ly.T, ly.d_in, ly.d_out); }

int tiles_per_sample(int path, const dp_layer& ly) {
  if (path == DP_PATH_PEREX) return perex_tiles_per_sample(ly.d_in, ly.d_out);
  if (ghost_uses_sample(ly)) return 1;
  return ghost_uses_big(ly) ? ghost_big_tiles_per_sample(ly.T) : ghost_tiles_per_sample(ly.T);
}

// Launches the norm kernels of one path for the listed layers, in chunks of kMaxGroup.
// part_begin[l] is the layer's first slot in the partial-sum workspace.
enum NormKernel { kGhostBig = 0, kGhostSmall = 1, kPerex = 2, kGhostSample = 3 };
constexpr int kNormKernels = 4;

dp_status run_norm_path(NormKernel kernel, const dp_layer* layers, int* which, int n_which,
                        const int64_t* part_begin, dp_dtype dt, int B, float* partials,
                        float* sqnorm_out, hipStream_t s, const int* row_of, float* const* kept) {
  // A tile's length is the contraction it runs over (d_in + d_out for the ghost norm, T for the
  // instantiated one).  Longest first: workgroups are handed out in order, so the short tiles
  // fill the end of the launch.  Each layer writes its own workspace slots and sqnorm row, so
  // the order inside a launch is free.  (Stable insertion sort in place: this path must not
  // touch the heap, see dp_norms_multi_static.)
  auto length = [&](int l) {
    return kernel == kPerex ? (int64_t)layers[l].T : (int64_t)layers[l].d_in + layers[l].d_out;
  };
  for (int i = 1; i < n_which; ++i) {
    const int x = which[i];
    int j = i;
    for (; j > 0 && length(which[j - 1]) < length(x); --j) which[j] = which[j - 1];
    which[j] = x;
  }
  for (int begin = 0; begin < n_which; begin += kMaxGroup) {
    GroupArgs ga;
    ga.B = B;
    ga.accumulate = 0;
    ga.f16 = dt == DP_F16;
    ga.n_layers = std::min(kMaxGroup, n_which - begin);
    int64_t blocks = 0;
    for (int j = 0; j < ga.n_layers; ++j) {
      const int l = which[begin + j];
      GroupLayer& gl = ga.layer[j];
      gl.a = layers[l].a;
      gl.g = layers[l].g;
      gl.out = kernel == kPerex && kept ? kept[l] : nullptr;
      gl.T = layers[l].T;
      gl.d_in = layers[l].d_in;
      gl.d_out = layers[l].d_out;
      gl.path = kernel == kPerex ? DP_PATH_PEREX : DP_PATH_GHOST;
      gl.tile_begin = (int)blocks;
      gl.sq_index = row_of ? row_of[l] : l;
      gl.part_begin = (int)part_begin[l];
      gl.tiles_per_sample = tiles_per_sample(gl.path, layers[l]);
      gl.c_off = 0;
      blocks += (int64_t)gl.tiles_per_sample * B;
    }
    ga.total_blocks = (int)blocks;
    // instantiated norm: the kernel with the deep load pipeline unless a slab is beyond its
    // 32-bit addressing (both use the same tiles and partial-sum slots)
    bool dma = DP_PEREX_DMA;
    for (int j = 0; j < ga.n_layers; ++j)
      dma = dma && perex_dma_supports(ga.layer[j].T, ga.layer[j].d_in, ga.layer[j].d_out);
    dp_status st = kernel == kGhostBig      ? launch_ghost_big_group(ga, partials, s)
                   : kernel == kGhostSmall  ? launch_ghost_group(ga, partials, s)
                   : kernel == kGhostSample ? launch_ghost_sample_group(ga, partials, s)
                   : dma                    ? launch_perex_dma_group(ga, partials, s)
                                            : launch_perex_group(ga, partials, s);
    if (st != DP_OK) return st;
    st = launch_norm_reduce_group(ga, partials, sqnorm_out, s);
    if (st != DP_OK) return st;
  }
  return DP_OK;
}

// Total partial-sum slots, or -1 if a layer is invalid.
int64_t norm_slots(const dp_layer* layers, int L, dp_dtype dt, int B, int64_t* begin) {
  if (!layers || L <= 0 || B <= 0) return -1;
  int64_t total = 0;
  for (int l = 0; l < L; ++l) {
    if (!dims_ok(dt, B, layers[l].T, layers[l].d_in, layers[l].d_out)) return -1;
    if (layers[l].path != DP_PATH_GHOST && layers[l].path != DP_PATH_PEREX) return -1;
    if (begin) begin[l] = total;
    if (dt != DP_F32) total += (int64_t)tiles_per_sample(layers[l].path, layers[l]) * B;
    if (total > INT32_MAX) return -1;
  }
  return total;
}

// begin: room for L values; idx: room for kNormKernels * L values (the layers of each kernel).  The caller
// provides both so that this function never touches the heap.  row_of (or nullptr): layer l's
// squared norms go to row row_of[l] of sqnorm_out instead of row l.
dp_status norms_impl(const dp_layer* layers, int L, dp_dtype dt, int B, float* sqnorm_out, void* ws,
                     size_t ws_bytes, hipStream_t s, int64_t* begin, int* idx, const int* row_of = nullptr,
                     float* const* kept = nullptr) {
  if (!dtype_ok(dt)) return DP_ERR_INVALID_ARG;
  if (!sqnorm_out) return DP_ERR_INVALID_ARG;
  const int64_t slots = norm_slots(layers, L, dt, B, begin);
  if (slots < 0) return DP_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l) {
    dp_status st = check_layer_ptrs(layers[l].a, layers[l].g);
    if (st != DP_OK) return st;
  }
  if (dt == DP_F32) {
    for (int l = 0; l < L; ++l) {
      const dp_layer& ly = layers[l];
      const __int128 work = ly.path == DP_PATH_GHOST
                                ? (__int128)ly.T * ly.T / 2 * ((int64_t)ly.d_in + ly.d_out)
                                : (__int128)ly.T * ly.d_in * ly.d_out;
      if (work > kF32MaxWork) return DP_ERR_UNSUPPORTED;
    }
    for (int l = 0; l < L; ++l) {
      const dp_layer& ly = layers[l];
      const float* a = static_cast<const float*>(ly.a);
      const float* g = static_cast<const float*>(ly.g);
      float* out = sqnorm_out + (size_t)(row_of ? row_of[l] : l) * B;
      dp_status st = ly.path == DP_PATH_GHOST ? launch_ghost_f32(a, g, B, ly.T, ly.d_in, ly.d_out, out, s)
                                              : launch_perex_f32(a, g, B, ly.T, ly.d_in, ly.d_out, out, s);
      if (st != DP_OK) return st;
    }
    return DP_OK;
  }
  if (!ws || ws_bytes < (size_t)slots * sizeof(float)) return DP_ERR_WORKSPACE;
  if (!aligned16(ws)) return DP_ERR_INVALID_ARG;
  int* list[kNormKernels] = {idx, idx + L, idx + 2 * L, idx + 3 * L};
  int count[kNormKernels] = {0, 0, 0, 0};
  for (int l = 0; l < L; ++l) {
    const int k = layers[l].path == DP_PATH_PEREX ? kPerex
                  : ghost_uses_sample(layers[l])  ? kGhostSample
                  : ghost_uses_big(layers[l])     ? kGhostBig
                                                  : kGhostSmall;
    list[k][count[k]++] = l;
  }
  float* partials = static_cast<float*>(ws);
  for (int k = 0; k < kNormKernels; ++k) {
    dp_status st = run_norm_path((NormKernel)k, layers, list[k], count[k], begin, dt, B, partials, sqnorm_out, s,
                                 row_of, kept);
    if (st != DP_OK) return st;
  }
  return DP_OK;
}

dp_status norms_impl(const dp_layer* layers, int L, dp_dtype dt, int B, float* sqnorm_out, void* ws,
                     size_t ws_bytes, hipStream_t s, const int* row_of = nullptr, float* const* kept = nullptr) {
  if (!layers || L <= 0) return DP_ERR_INVALID_ARG;
  std::vector<int64_t> begin(L);
  std::vector<int> idx(kNormKernels * (size_t)L);
  return norms_impl(layers, L, dt, B, sqnorm_out, ws, ws_bytes, s, begin.data(), idx.data(), row_of, kept);
}

dp_status single_norm(dp_path path, const void* a, const void* g, dp_dtype dt, int B, int T, int d_in,
                      int d_out, float* sqnorm_out, void* ws, size_t ws_bytes, void* stream) {
  dp_layer ly;
  ly.a = a;
  ly.g = g;
  ly.T = T;
  ly.d_in = d_in;
  ly.d_out = d_out;
  ly.path = path;
  return norms_impl(&ly, 1, dt, B, sqnorm_out, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

}  // namespace

extern "C" {

const char* dp_status_string(dp_status s) {
  switch (s) {
    case DP_OK: return "ok";
    case DP_ERR_INVALID_ARG: return "invalid argument";
    case DP_ERR_UNSUPPORTED: return "unsupported";
    case DP_ERR_WORKSPACE: return "workspace missing or too small";
    case DP_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

int dp_version(void) { return 100; }

dp_path dp_choose_path(int64_t T, int64_t d_in, int64_t d_out) {
  if (T <= 0 || d_in <= 0 || d_out <= 0) return DP_PATH_GHOST;
  // 2 T^2 <= d_in d_out without overflow: compare in 128 bits.
  const __int128 lhs = (__int128)2 * T * T, rhs = (__int128)d_in * d_out;
  return lhs <= rhs ? DP_PATH_GHOST : DP_PATH_PEREX;
}

size_t dp_norm_workspace_bytes(dp_path path, dp_dtype dt, int B, int T, int d_in, int d_out) {
  dp_layer ly = {nullptr, nullptr, T, d_in, d_out, (int32_t)path};
  return dp_norms_multi_workspace_bytes(&ly, 1, dt, B);
}

size_t dp_norms_multi_workspace_bytes(const dp_layer* layers, int L, dp_dtype dt, int B) {
  if (!dtype_ok(dt)) return 0;
  const int64_t slots = norm_slots(layers, L, dt, B, nullptr);
  if (slots < 0) return 0;
  // never 0 for a valid request, so "0 = invalid" stays unambiguous
  return (size_t)(slots > 0 ? slots : 4) * sizeof(float);
}

dp_status dp_ghost_norm(const void* a, const void* g, dp_dtype dt, int B, int T, int d_in, int d_out,
                        float* sqnorm_out, void* ws, size_t ws_bytes, void* stream) {
  return single_norm(DP_PATH_GHOST, a, g, dt, B, T, d_in, d_out, sqnorm_out, ws, ws_bytes, stream);
}

dp_status dp_perex_norm(const void* a, const void* g, dp_dtype dt, int B, int T, int d_in, int d_out,
                        float* sqnorm_out, void* ws, size_t ws_bytes, void* stream) {
  return single_norm(DP_PATH_PEREX, a, g, dt, B, T, d_in, d_out, sqnorm_out, ws, ws_bytes, stream);
}

dp_status dp_norms_multi(const dp_layer* layers, int L, dp_dtype dt, int B, float* sqnorm_out, void* ws,
                         size_t ws_bytes, void* stream) {
  return norms_impl(layers, L, dt, B, sqnorm_out, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

dp_status dp_clip_factors(const float* sqnorm, int L, int B, dp_clip_mode mode, float R, float stability,
                          float* C_out, float* norm_out, void* stream) {
  if (!sqnorm || !C_out || L <= 0 || B <= 0) return DP_ERR_INVALID_ARG;
  if (mode != DP_CLIP_STANDARD && mode != DP_CLIP_AUTOMATIC) return DP_ERR_INVALID_ARG;
  if (!(R > 0.f)) return DP_ERR_INVALID_ARG;                      // rejects NaN too
  if (!(stability >= 0.f) || isinf(stability)) return DP_ERR_INVALID_ARG;
  return launch_clip_factors(sqnorm, L, B, (int)mode, R, stability, C_out, norm_out,
                             static_cast<hipStream_t>(stream));
}

}  // extern "C"

namespace {

// Clip-weighted gradients of a stack; layer l uses the weights C[c_off[l] + i] (c_off == nullptr:
// every layer uses C[i]).
// Noise request of dp_clipped_grad_noise_multi, validated.
struct NoiseSpec {
  const uint64_t* grad_offset;   // host, [L]
  uint64_t lo, hi;               // global element range that receives noise
  float stddev;
  uint64_t seed, step;
};

// Separate noise pass on the part of layer l's gradient that lies inside the range.
dp_status noise_after(const NoiseSpec* noise, int l, const dp_layer& ly, float* grad, hipStream_t s) {
  if (!noise) return DP_OK;
  const uint64_t begin = noise->grad_offset[l], end = begin + (uint64_t)ly.d_in * ly.d_out;
  const uint64_t lo = std::max(begin, noise->lo), hi = std::min(end, noise->hi);
  if (lo >= hi) return DP_OK;
  return launch_noise(grad + (lo - begin), lo, hi - lo, noise->stddev, noise->seed, noise->step, s);
}

// out16: grads[l] address 16-bit arrays of the operands' storage type; only the large-tile kernels
// write those, with the noise in their epilogue, so every layer must qualify for them.
dp_status clipped_grad_impl(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                            const int* c_off, float* const* grads, int accumulate, void* stream,
                            const NoiseSpec* noise = nullptr, bool out16 = false) {
  if (!dtype_ok(dt)) return DP_ERR_INVALID_ARG;
  if (!layers || !grads || !C || L <= 0 || B <= 0) return DP_ERR_INVALID_ARG;
  if (accumulate != 0 && accumulate != 1) return DP_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l) {
    if (!dims_ok(dt, B, layers[l].T, layers[l].d_in, layers[l].d_out)) return DP_ERR_INVALID_ARG;
    dp_status st = check_layer_ptrs(layers[l].a, layers[l].g);
    if (st != DP_OK) return st;
    if (!grads[l] || !aligned16(grads[l])) return DP_ERR_INVALID_ARG;
    if ((int64_t)clipped_grad_tiles(layers[l].d_in, layers[l].d_out) > INT32_MAX / 2) return DP_ERR_INVALID_ARG;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (out16) {
    if (dt == DP_F32) return DP_ERR_UNSUPPORTED;
    for (int l = 0; l < L; ++l) {
      const dp_layer& ly = layers[l];
      if (!(ly.d_in >= 128 && ly.d_out >= 128 && clipped_grad_big_supports(ly.T, ly.d_in, ly.d_out)))
        return DP_ERR_UNSUPPORTED;
      if (noise && (noise->grad_offset[l] & 3)) return DP_ERR_UNSUPPORTED;
    }
  }
  if (dt == DP_F32) {
    for (int l = 0; l < L; ++l) {
      dp_status st = launch_clipped_grad_f32(static_cast<const float*>(layers[l].a),
                                             static_cast<const float*>(layers[l].g), B, layers[l].T,
                                             layers[l].d_in, layers[l].d_out, C + (c_off ? c_off[l] : 0),
                                             grads[l], accumulate, s);
      if (st != DP_OK) return st;
      st = noise_after(noise, l, layers[l], grads[l], s);
      if (st != DP_OK) return st;
    }
    return DP_OK;
  }
  // Layers wide enough to fill 256x256 tiles take the large-tile kernel; the rest (and slabs
  // beyond its 32-bit addressing) take the 8-wave kernel with per-element edge handling.
  std::vector<int> big, small;
  for (int l = 0; l < L; ++l) {
    const dp_layer& ly = layers[l];
    const bool use_big = ly.d_in >= 128 && ly.d_out >= 128 && clipped_grad_big_supports(ly.T, ly.d_in, ly.d_out);
    (use_big ? big : small).push_back(l);
  }
  for (int pass = 0; pass < 2; ++pass) {
    const std::vector<int>& which = pass == 0 ? big : small;
    size_t pos = 0;
    while (pos < which.size()) {
      GroupArgs ga;
      ga.B = B;
      ga.accumulate = accumulate;
      ga.f16 = dt == DP_F16;
      ga.n_layers = 0;
      int64_t blocks = 0;
      while (pos < which.size() && ga.n_layers < kMaxGroup) {
        const int l = which[pos];
        const int64_t tiles = pass == 0 ? clipped_grad_big_tiles(layers[l].d_in, layers[l].d_out)
                                        : clipped_grad_tiles(layers[l].d_in, layers[l].d_out);
        if (ga.n_layers > 0 && blocks + tiles > INT32_MAX / 2) break;
        GroupLayer& gl = ga.layer[ga.n_layers++];
        gl.a = layers[l].a;
        gl.g = layers[l].g;
        gl.out = grads[l];
        gl.T = layers[l].T;
        gl.d_in = layers[l].d_in;
        gl.d_out = layers[l].d_out;
        gl.path = 0;
        gl.tile_begin = (int)blocks;
        gl.sq_index = l;
        gl.part_begin = 0;
        gl.tiles_per_sample = (int)tiles;
        gl.c_off = c_off ? c_off[l] : 0;
        blocks += tiles;
        ++pos;
      }
      ga.total_blocks = (int)blocks;
      // The large-tile kernels add the noise in their epilogue when every layer of the launch
      // starts on a generator block (offset a multiple of 4); otherwise, and for the small-layer
      // kernel, the noise pass runs on the layer's slice afterwards.
      bool fused = noise && pass == 0;
      NoiseArgs na;
      if (fused) {
        for (int j = 0; j < ga.n_layers; ++j) {
          na.layer_off[j] = noise->grad_offset[ga.layer[j].sq_index];
          fused = fused && (na.layer_off[j] & 3) == 0;
        }
      }
      if (fused) {
        na.stddev = noise->stddev;
        na.step_lo = (uint32_t)noise->step;
        na.step_hi = (uint32_t)(noise->step >> 32);
        na.lo = noise->lo;
        na.hi = noise->hi;
        na.rk = make_round_keys(noise->seed);
      }
      dp_status st = pass == 0 ? launch_clipped_grad_big_group(ga, C, fused ? &na : nullptr, s, out16)
                               : launch_clipped_grad_group(ga, C, s);
      if (st != DP_OK) return st;
      if (noise && !fused) {
        for (int j = 0; j < ga.n_layers; ++j) {
          const int l = ga.layer[j].sq_index;
          st = noise_after(noise, l, layers[l], grads[l], s);
          if (st != DP_OK) return st;
        }
      }
    }
  }
  return DP_OK;
}

// Sum_i C_i G_i from kept per-sample gradients for the layers that have them (kept[l] != nullptr),
// up to kMaxGroup layers per launch.  c_off (or nullptr): layer l's weights are C[c_off[l] + i].
// noise (or nullptr): added by the same kernel when the layer starts on a generator block, else
// by a pass afterwards.
dp_status kept_sum_impl(const dp_layer* layers, int L, int B, const float* C, const int* c_off,
                        float* const* kept, float* const* grads, const NoiseSpec* noise, int accumulate,
                        hipStream_t s) {
  const bool noisy = noise != nullptr && noise->stddev > 0.f;
  NoiseArgs na = {};
  if (noisy) {
    na.stddev = noise->stddev;
    na.step_lo = (uint32_t)noise->step;
    na.step_hi = (uint32_t)(noise->step >> 32);
    na.lo = noise->lo;
    na.hi = noise->hi;
    na.rk = make_round_keys(noise->seed);
  }
  int l = 0;
  while (l < L) {
    GroupArgs ga;
    ga.B = B;
    ga.accumulate = accumulate;
    ga.f16 = 0;
    ga.n_layers = 0;
    int64_t blocks = 0;
    int members[kMaxGroup];
    for (; l < L && ga.n_layers < kMaxGroup; ++l) {
      if (!kept || !kept[l]) continue;
      const int nb = kept_blocks(layers[l].d_in, layers[l].d_out);
      if (ga.n_layers > 0 && blocks + nb > INT32_MAX / 2) break;
      GroupLayer& gl = ga.layer[ga.n_layers];
      gl.a = kept[l];
      gl.g = nullptr;
      gl.out = grads[l];
      gl.T = layers[l].T;
      gl.d_in = layers[l].d_in;
      gl.d_out = layers[l].d_out;
      gl.path = DP_PATH_PEREX;
      gl.tile_begin = (int)blocks;
      gl.sq_index = l;
      gl.part_begin = 0;
      gl.tiles_per_sample = nb;
      gl.c_off = c_off ? c_off[l] : 0;
      na.layer_off[ga.n_layers] =
          noisy && (noise->grad_offset[l] & 3) == 0 ? noise->grad_offset[l] : ~(uint64_t)0;
      members[ga.n_layers] = l;
      blocks += nb;
      ++ga.n_layers;
    }
    if (ga.n_layers == 0) break;
    ga.total_blocks = (int)blocks;
    dp_status st = launch_kept_weighted_sum(ga, C, na, s);
    if (st != DP_OK) return st;
    for (int j = 0; j < ga.n_layers; ++j)
      if (noisy && na.layer_off[j] == ~(uint64_t)0) {
        st = noise_after(noise, members[j], layers[members[j]], grads[members[j]], s);
        if (st != DP_OK) return st;
      }
  }
  return DP_OK;
}

}  // namespace

extern "C" {

dp_status dp_clipped_grad_multi(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                float* const* grads, int accumulate, void* stream) {
  return clipped_grad_impl(layers, L, dt, B, C, nullptr, grads, accumulate, stream);
}

dp_status dp_clipped_grad_noise_multi(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                      float* const* grads, const uint64_t* grad_offset, int accumulate,
                                      uint64_t shard_offset, uint64_t shard_count, float sigma, float R,
                                      uint64_t seed, uint64_t step, void* stream) {
  if (!(sigma >= 0.f) || isinf(sigma)) return DP_ERR_INVALID_ARG;
  if (!(R > 0.f)) return DP_ERR_INVALID_ARG;
  if (shard_offset + shard_count < shard_offset) return DP_ERR_INVALID_ARG;   // wraps 2^64
  if (sigma == 0.f || shard_count == 0)                                        // nothing to add
    return clipped_grad_impl(layers, L, dt, B, C, nullptr, grads, accumulate, stream);
  if (isinf(R) || !grad_offset || !layers || L <= 0) return DP_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l) {
    const uint64_t n = (uint64_t)std::max(layers[l].d_in, 0) * (uint64_t)std::max(layers[l].d_out, 0);
    if (grad_offset[l] + n < grad_offset[l]) return DP_ERR_INVALID_ARG;
  }
  NoiseSpec spec;
  spec.grad_offset = grad_offset;
  spec.lo = shard_offset;
  spec.hi = shard_offset + shard_count;
  spec.stddev = sigma * R;
  spec.seed = seed;
  spec.step = step;
  return clipped_grad_impl(layers, L, dt, B, C, nullptr, grads, accumulate, stream, &spec);
}

dp_status dp_clipped_grad_noise_multi_h16(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                          void* const* grads16, const uint64_t* grad_offset, int accumulate,
                                          uint64_t shard_offset, uint64_t shard_count, float sigma, float R,
                                          uint64_t seed, uint64_t step, void* stream) {
  if (!(sigma >= 0.f) || isinf(sigma)) return DP_ERR_INVALID_ARG;
  if (!(R > 0.f)) return DP_ERR_INVALID_ARG;
  if (shard_offset + shard_count < shard_offset) return DP_ERR_INVALID_ARG;
  float* const* grads = reinterpret_cast<float* const*>(grads16);      // the kernels store 16-bit values there
  if (sigma == 0.f || shard_count == 0)
    return clipped_grad_impl(layers, L, dt, B, C, nullptr, grads, accumulate, stream, nullptr, true);
  if (isinf(R) || !grad_offset || !layers || L <= 0) return DP_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l) {
    const uint64_t n = (uint64_t)std::max(layers[l].d_in, 0) * (uint64_t)std::max(layers[l].d_out, 0);
    if (grad_offset[l] + n < grad_offset[l]) return DP_ERR_INVALID_ARG;
  }
  NoiseSpec spec;
  spec.grad_offset = grad_offset;
  spec.lo = shard_offset;
  spec.hi = shard_offset + shard_count;
  spec.stddev = sigma * R;
  spec.seed = seed;
  spec.step = step;
  return clipped_grad_impl(layers, L, dt, B, C, nullptr, grads, accumulate, stream, &spec, true);
}

dp_status dp_clipped_grad_grouped(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                  const int32_t* group_of_layer, int M, float* const* grads,
                                  int accumulate, void* stream) {
  if (!group_of_layer || L <= 0 || M <= 0 || B <= 0 || (int64_t)M * B > INT32_MAX) return DP_ERR_INVALID_ARG;
  std::vector<int> c_off(L);
  for (int l = 0; l < L; ++l) {
    if (group_of_layer[l] < 0 || group_of_layer[l] >= M) return DP_ERR_INVALID_ARG;
    c_off[l] = group_of_layer[l] * B;
  }
  return clipped_grad_impl(layers, L, dt, B, C, c_off.data(), grads, accumulate, stream);
}

dp_status dp_clip_factors_grouped(const float* sqnorm, int L, int B, const int32_t* group_begin, int M,
                                  const float* R, dp_clip_mode mode, float stability, float* C_out,
                                  float* norm_out, void* stream) {
  if (!sqnorm || !C_out || !group_begin || !R || L <= 0 || B <= 0 || M <= 0) return DP_ERR_INVALID_ARG;
  if (mode != DP_CLIP_STANDARD && mode != DP_CLIP_AUTOMATIC) return DP_ERR_INVALID_ARG;
  if (!(stability >= 0.f) || isinf(stability)) return DP_ERR_INVALID_ARG;
  if (group_begin[0] != 0 || group_begin[M] != L) return DP_ERR_INVALID_ARG;
  for (int m = 0; m < M; ++m) {
    if (group_begin[m + 1] < group_begin[m]) return DP_ERR_INVALID_ARG;     // empty groups are allowed
    if (!(R[m] > 0.f)) return DP_ERR_INVALID_ARG;
  }
  return launch_clip_factors_grouped(sqnorm, B, group_begin, M, R, (int)mode, stability, C_out, norm_out,
                                     static_cast<hipStream_t>(stream));
}

float dp_group_noise_threshold(const float* R, int M) {
  if (!R || M <= 0) return 0.f;
  double s = 0.0;
  for (int m = 0; m < M; ++m) s += (double)R[m] * R[m];
  return (float)sqrt(s);
}

dp_status dp_bias_norm(const void* g, dp_dtype dt, int B, int T, int d_out, float* colsum,
                       float* sqnorm_out, void* stream) {
  if (!dtype_ok(dt)) return DP_ERR_INVALID_ARG;
  if (!g || !colsum || !sqnorm_out || !aligned16(g)) return DP_ERR_INVALID_ARG;
  if (!dims_ok(dt, B, T, 8, d_out)) return DP_ERR_INVALID_ARG;
  if (B > 65535) return DP_ERR_UNSUPPORTED;
  return launch_bias_norm(g, dt, B, T, d_out, colsum, sqnorm_out, static_cast<hipStream_t>(stream));
}

dp_status dp_clipped_bias_grad(const float* colsum, int B, int d_out, const float* C, float* grad_b,
                               int accumulate, void* stream) {
  if (!colsum || !C || !grad_b || B <= 0 || d_out <= 0) return DP_ERR_INVALID_ARG;
  if (accumulate != 0 && accumulate != 1) return DP_ERR_INVALID_ARG;
  return launch_clipped_bias_grad(colsum, B, d_out, C, grad_b, accumulate, static_cast<hipStream_t>(stream));
}

dp_status dp_clipped_grad(const void* a, const void* g, dp_dtype dt, int B, int T, int d_in, int d_out,
                          const float* C, float* grad, int accumulate, void* stream) {
  dp_layer ly = {a, g, T, d_in, d_out, 0};
  float* grads[1] = {grad};
  return dp_clipped_grad_multi(&ly, 1, dt, B, C, grads, accumulate, stream);
}

dp_status dp_add_noise(float* grad_slice, uint64_t global_offset, uint64_t count, float sigma, float R,
                       uint64_t seed, uint64_t step, void* stream) {
  if (!(sigma >= 0.f) || isinf(sigma)) return DP_ERR_INVALID_ARG;
  if (!(R > 0.f)) return DP_ERR_INVALID_ARG;
  if (global_offset + count < global_offset) return DP_ERR_INVALID_ARG;   // wraps 2^64
  if (sigma == 0.f || count == 0) return DP_OK;                            // non-private: nothing to add
  if (isinf(R)) return DP_ERR_INVALID_ARG;
  if (!grad_slice || (reinterpret_cast<uintptr_t>(grad_slice) & 3u)) return DP_ERR_INVALID_ARG;
  return launch_noise(grad_slice, global_offset, count, sigma * R, seed, step,
                      static_cast<hipStream_t>(stream));
}

dp_status dp_philox_blocks(uint32_t* out, uint64_t first_block, uint64_t n_blocks, uint64_t seed,
                           uint64_t step, void* stream) {
  if (!out || !aligned16(out)) return DP_ERR_INVALID_ARG;
  if (n_blocks == 0) return DP_OK;
  if (first_block + n_blocks < first_block) return DP_ERR_INVALID_ARG;
  return launch_philox_blocks(out, first_block, n_blocks, seed, step, static_cast<hipStream_t>(stream));
}

}  // extern "C"


// ---------------------------------------------------------------------------------
// Instantiated layers with their per-sample gradients kept between the two halves.
// ---------------------------------------------------------------------------------
namespace {

// kept[l] may be given only for 16-bit layers on the instantiated path, 16-byte aligned.
dp_status check_kept(const dp_layer* layers, int L, dp_dtype dt, float* const* kept) {
  if (!kept) return DP_OK;
  for (int l = 0; l < L; ++l) {
    if (!kept[l]) continue;
    if (dt == DP_F32) return DP_ERR_UNSUPPORTED;
    if (layers[l].path != DP_PATH_PEREX || !aligned16(kept[l])) return DP_ERR_INVALID_ARG;
    if ((int64_t)layers[l].d_in * layers[l].d_out > INT32_MAX - 4096) return DP_ERR_INVALID_ARG;   // int element index
  }
  return DP_OK;
}

}  // namespace

extern "C" {

dp_status dp_norms_multi_keep(const dp_layer* layers, int L, dp_dtype dt, int B, float* sqnorm_out,
                              float* const* kept, void* ws, size_t ws_bytes, void* stream) {
  if (!layers || L <= 0) return DP_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l)
    if (layers[l].path != DP_PATH_GHOST && layers[l].path != DP_PATH_PEREX) return DP_ERR_INVALID_ARG;
  dp_status st = check_kept(layers, L, dt, kept);
  if (st != DP_OK) return st;
  return norms_impl(layers, L, dt, B, sqnorm_out, ws, ws_bytes, static_cast<hipStream_t>(stream), nullptr, kept);
}

dp_status dp_clipped_grad_kept_multi(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                     float* const* kept, float* const* grads, const uint64_t* grad_offset,
                                     int accumulate, uint64_t shard_offset, uint64_t shard_count, float sigma,
                                     float R, uint64_t seed, uint64_t step, void* stream) {
  if (!layers || !grads || !C || L <= 0 || B <= 0 || !dtype_ok(dt)) return DP_ERR_INVALID_ARG;
  if (accumulate != 0 && accumulate != 1) return DP_ERR_INVALID_ARG;
  if (!(sigma >= 0.f) || isinf(sigma) || !(R > 0.f)) return DP_ERR_INVALID_ARG;
  if (shard_offset + shard_count < shard_offset) return DP_ERR_INVALID_ARG;
  const bool noisy = sigma > 0.f && shard_count > 0;
  if (noisy && (isinf(R) || !grad_offset)) return DP_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l) {
    if (!dims_ok(dt, B, layers[l].T, layers[l].d_in, layers[l].d_out)) return DP_ERR_INVALID_ARG;
    if (layers[l].path != DP_PATH_GHOST && layers[l].path != DP_PATH_PEREX) return DP_ERR_INVALID_ARG;
    if (!grads[l] || !aligned16(grads[l])) return DP_ERR_INVALID_ARG;
    const uint64_t n = (uint64_t)layers[l].d_in * (uint64_t)layers[l].d_out;
    if (noisy && grad_offset[l] + n < grad_offset[l]) return DP_ERR_INVALID_ARG;
  }
  dp_status st = check_kept(layers, L, dt, kept);
  if (st != DP_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  NoiseSpec spec;
  spec.grad_offset = grad_offset;
  spec.lo = shard_offset;
  spec.hi = shard_offset + shard_count;
  spec.stddev = noisy ? sigma * R : 0.f;
  spec.seed = seed;
  spec.step = step;
  // (1) layers without kept gradients: the contraction over a and g
  std::vector<dp_layer> sub;
  std::vector<float*> sub_grads;
  std::vector<uint64_t> sub_off;
  for (int l = 0; l < L; ++l)
    if (!kept || !kept[l]) {
      sub.push_back(layers[l]);
      sub_grads.push_back(grads[l]);
      sub_off.push_back(noisy ? grad_offset[l] : 0);
    }
  if (!sub.empty()) {
    NoiseSpec sub_spec = spec;
    sub_spec.grad_offset = sub_off.data();
    st = clipped_grad_impl(sub.data(), (int)sub.size(), dt, B, C, nullptr, sub_grads.data(), accumulate, stream,
                           noisy ? &sub_spec : nullptr);
    if (st != DP_OK) return st;
  }
  // (2) layers with kept gradients: weighted sums
  return kept_sum_impl(layers, L, B, C, nullptr, kept, grads, noisy ? &spec : nullptr, accumulate, s);
}

}  // extern "C"

// ---------------------------------------------------------------------------------
// Layer-wise clipping without book-keeping (section 3.3 (II); appendix on the hook-free form).
// ---------------------------------------------------------------------------------
namespace {

// A pass ends once its a and g exceed half the memory-side cache, but not before it holds enough
// gradient tiles for four rounds of workgroups: launches that leave compute units idle cost more
// than re-reading a and g from memory (measured on a GPT-2-small stack: passes of 4 layers
// 2.3 ms, 8 layers 1.39 ms, 16 layers 1.38 ms, all norms then all gradients 1.31 ms).
constexpr int64_t kPassBytes = (int64_t)128 << 20;
constexpr int64_t kPassTiles = 1024;

// Which layers the one-pass kernel takes, and its sample chunks.
struct FusedPlan {
  std::vector<int> shape;        // per layer: shape class or -1
  int n_fused = 0;
  int chunks = 1;                // sample chunks per fused layer
  int64_t floats = 0;            // partial sums of all fused layers
  // Other layers on the instantiated path keep their per-sample gradients G_i between the norm and
  // the weighted sum (as dp_norms_multi_keep does): float offset of layer l's [B, d, p] block in
  // the kept region of the workspace, or -1.  Layers are taken in order while the region stays
  // within kKeptMaxBytes; the rest contract a and g a second time.
  std::vector<int64_t> kept_off;
  int64_t kept_floats = 0;
};
constexpr int64_t kKeptMaxBytes = (int64_t)2 << 30;

FusedPlan plan_fused(const dp_layer* layers, int L, dp_dtype dt, int B) {
  FusedPlan fp;
  fp.shape.assign(L, -1);
  fp.kept_off.assign(L, -1);
  if (dt == DP_F32) return fp;
  for (int l = 0; l < L; ++l)
    if (layers[l].path == DP_PATH_PEREX) {
      fp.shape[l] = layerwise_fused_shape(layers[l].d_in, layers[l].d_out);
      fp.n_fused += fp.shape[l] >= 0;
      const int64_t n = (int64_t)B * layers[l].d_in * layers[l].d_out;
      if (fp.shape[l] < 0 && n <= INT32_MAX - 4096 && (fp.kept_floats + n) * 4 <= kKeptMaxBytes) {
        fp.kept_off[l] = fp.kept_floats;
        fp.kept_floats += (n + 3) & ~(int64_t)3;                  // blocks stay 16-byte aligned
      }
    }
  if (fp.n_fused == 0) return fp;
  // enough workgroups to fill the 256 compute units when the batch allows
  const int want = std::min(B, std::max(1, 256 / fp.n_fused));
  const int per = (B + want - 1) / want;
  fp.chunks = (B + per - 1) / per;
  for (int l = 0; l < L; ++l)
    if (fp.shape[l] >= 0) fp.floats += (int64_t)fp.chunks * layers[l].d_in * layers[l].d_out;
  return fp;
}

size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

}  // namespace

extern "C" {

size_t dp_layerwise_workspace_bytes(const dp_layer* layers, int L, dp_dtype dt, int B) {
  const size_t norms = dp_norms_multi_workspace_bytes(layers, L, dt, B);
  if (norms == 0) return 0;
  const FusedPlan fp = plan_fused(layers, L, dt, B);
  if (fp.floats > INT32_MAX) return 0;
  return align16(norms) + align16((size_t)fp.floats * sizeof(float)) + (size_t)fp.kept_floats * sizeof(float);
}

dp_status dp_layerwise_clipped_grad(const dp_layer* layers, int L, dp_dtype dt, int B, const float* R,
                                    dp_clip_mode mode, float stability, float* const* grads,
                                    const uint64_t* grad_offset, int accumulate, uint64_t shard_offset,
                                    uint64_t shard_count, float sigma, uint64_t seed, uint64_t step,
                                    float* sqnorm_out, float* C_out, void* ws, size_t ws_bytes,
                                    int layers_per_pass, void* stream) {
  if (!dtype_ok(dt) || !layers || !R || !grads || !sqnorm_out || !C_out || L <= 0 || B <= 0) return DP_ERR_INVALID_ARG;
  if (mode != DP_CLIP_STANDARD && mode != DP_CLIP_AUTOMATIC) return DP_ERR_INVALID_ARG;
  if (!(stability >= 0.f) || isinf(stability)) return DP_ERR_INVALID_ARG;
  if (accumulate != 0 && accumulate != 1) return DP_ERR_INVALID_ARG;
  if (layers_per_pass < 0 || (int64_t)L * B > INT32_MAX) return DP_ERR_INVALID_ARG;
  if (!(sigma >= 0.f) || isinf(sigma)) return DP_ERR_INVALID_ARG;
  if (shard_offset + shard_count < shard_offset) return DP_ERR_INVALID_ARG;
  double r2 = 0.0;
  for (int l = 0; l < L; ++l) {
    if (!(R[l] > 0.f)) return DP_ERR_INVALID_ARG;
    r2 += (double)R[l] * R[l];
    if (!dims_ok(dt, B, layers[l].T, layers[l].d_in, layers[l].d_out)) return DP_ERR_INVALID_ARG;
    if (layers[l].path != DP_PATH_GHOST && layers[l].path != DP_PATH_PEREX) return DP_ERR_INVALID_ARG;
    dp_status st = check_layer_ptrs(layers[l].a, layers[l].g);
    if (st != DP_OK) return st;
    if (!grads[l] || !aligned16(grads[l])) return DP_ERR_INVALID_ARG;
  }
  const bool noisy = sigma > 0.f && shard_count > 0;
  const float stddev = noisy ? (float)(sigma * sqrt(r2)) : 0.f;          // eq. (1): sigma ||(R_1..R_L)||
  if (noisy) {
    if (!grad_offset || isinf(stddev)) return DP_ERR_INVALID_ARG;
    for (int l = 0; l < L; ++l) {
      const uint64_t n = (uint64_t)layers[l].d_in * (uint64_t)layers[l].d_out;
      if (grad_offset[l] + n < grad_offset[l]) return DP_ERR_INVALID_ARG;
    }
  }
  const size_t need = dp_layerwise_workspace_bytes(layers, L, dt, B);
  if (need == 0) return DP_ERR_INVALID_ARG;
  if (!ws || ws_bytes < need) return DP_ERR_WORKSPACE;
  if (!aligned16(ws)) return DP_ERR_INVALID_ARG;
  const FusedPlan fp = plan_fused(layers, L, dt, B);
  float* fused_partial = reinterpret_cast<float*>(static_cast<unsigned char*>(ws) +
                                                  align16(dp_norms_multi_workspace_bytes(layers, L, dt, B)));
  float* kept_region = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(fused_partial) +
                                                align16((size_t)fp.floats * sizeof(float)));
  hipStream_t s = static_cast<hipStream_t>(stream);

  NoiseArgs na = {};
  na.stddev = stddev;
  na.step_lo = (uint32_t)step;
  na.step_hi = (uint32_t)(step >> 32);
  na.lo = shard_offset;
  na.hi = shard_offset + shard_count;
  na.rk = make_round_keys(seed);

  int64_t fused_off = 0;
  for (int l0 = 0; l0 < L;) {
    // one pass: consecutive layers whose a and g stay in the memory-side cache between the norm
    // kernels and the gradient kernels (or layers_per_pass of them when the caller says so)
    int l1 = l0;
    int64_t bytes = 0, tiles = 0;
    const int64_t esize = dt == DP_F32 ? 4 : 2;
    while (l1 < L) {
      const bool small = fp.shape[l1] >= 0;
      const int64_t lb = small ? 0 : (int64_t)B * layers[l1].T * ((int64_t)layers[l1].d_in + layers[l1].d_out) * esize;
      if (l1 > l0 && (layers_per_pass > 0 ? l1 - l0 >= layers_per_pass
                                          : bytes + lb > kPassBytes && tiles >= kPassTiles)) break;
      bytes += lb;
      tiles += small ? 0 : clipped_grad_big_tiles(layers[l1].d_in, layers[l1].d_out);
      ++l1;
    }
    // (1) layers that fit one workgroup tile: norm, clip factor and weighted sum in one kernel
    for (int shape = 0; shape < 3; ++shape) {
      int l = l0;
      while (l < l1) {
        GroupArgs ga;
        ga.B = B;
        ga.accumulate = accumulate;
        ga.f16 = dt == DP_F16;
        ga.n_layers = 0;
        float Rg[kMaxGroup];
        int blocks = 0;
        for (; l < l1 && ga.n_layers < kMaxGroup; ++l) {
          if (fp.shape[l] != shape) continue;
          GroupLayer& gl = ga.layer[ga.n_layers];
          gl.a = layers[l].a;
          gl.g = layers[l].g;
          gl.out = grads[l];
          gl.T = layers[l].T;
          gl.d_in = layers[l].d_in;
          gl.d_out = layers[l].d_out;
          gl.path = DP_PATH_PEREX;
          gl.tile_begin = blocks;
          gl.sq_index = l;
          gl.part_begin = (int)fused_off;
          gl.tiles_per_sample = fp.chunks;
          gl.c_off = 0;
          Rg[ga.n_layers] = R[l];
          na.layer_off[ga.n_layers] = noisy ? grad_offset[l] : 0;
          fused_off += (int64_t)fp.chunks * gl.d_in * gl.d_out;
          blocks += fp.chunks;
          ++ga.n_layers;
        }
        if (ga.n_layers == 0) break;
        ga.total_blocks = blocks;
        dp_status st = launch_layerwise_fused(shape, ga, Rg, (int)mode, stability, fused_partial, sqnorm_out, C_out, s);
        if (st != DP_OK) return st;
        st = launch_layerwise_reduce(ga, fused_partial, na, s);
        if (st != DP_OK) return st;
      }
    }
    // (2) the other layers of the pass: norms, clip factors, weighted gradients
    //     (instantiated layers keep G_i in the workspace: their gradient is sum_i C_i G_i)
    std::vector<dp_layer> sub;
    std::vector<int> row, c_off;
    std::vector<float*> sub_grads, sub_kept;
    std::vector<uint64_t> sub_off;
    bool any_kept = false;
    for (int l = l0; l < l1; ++l)
      if (fp.shape[l] < 0) {
        sub.push_back(layers[l]);
        row.push_back(l);
        c_off.push_back(l * B);
        sub_grads.push_back(grads[l]);
        sub_off.push_back(noisy ? grad_offset[l] : 0);
        sub_kept.push_back(fp.kept_off[l] >= 0 ? kept_region + fp.kept_off[l] : nullptr);
        any_kept = any_kept || fp.kept_off[l] >= 0;
      }
    if (!sub.empty()) {
      const int n = (int)sub.size();
      dp_status st = norms_impl(sub.data(), n, dt, B, sqnorm_out, ws, ws_bytes, s, row.data(),
                                any_kept ? sub_kept.data() : nullptr);
      if (st != DP_OK) return st;
      std::vector<int32_t> begin(l1 - l0 + 1);
      for (int l = l0; l <= l1; ++l) begin[l - l0] = l;
      st = launch_clip_factors_grouped(sqnorm_out, B, begin.data(), l1 - l0, R + l0, (int)mode, stability,
                                       C_out + (size_t)l0 * B, nullptr, s);
      if (st != DP_OK) return st;
      NoiseSpec spec;
      spec.grad_offset = sub_off.data();
      spec.lo = shard_offset;
      spec.hi = shard_offset + shard_count;
      spec.stddev = stddev;
      spec.seed = seed;
      spec.step = step;
      // layers without kept gradients: the contraction over a and g
      std::vector<dp_layer> rest;
      std::vector<int> rest_c;
      std::vector<float*> rest_grads;
      std::vector<uint64_t> rest_off;
      for (int j = 0; j < n; ++j)
        if (!sub_kept[j]) {
          rest.push_back(sub[j]);
          rest_c.push_back(c_off[j]);
          rest_grads.push_back(sub_grads[j]);
          rest_off.push_back(sub_off[j]);
        }
      if (!rest.empty()) {
        NoiseSpec rest_spec = spec;
        rest_spec.grad_offset = rest_off.data();
        st = clipped_grad_impl(rest.data(), (int)rest.size(), dt, B, C_out, rest_c.data(), rest_grads.data(),
                               accumulate, stream, noisy ? &rest_spec : nullptr);
        if (st != DP_OK) return st;
      }
      if (any_kept) {
        st = kept_sum_impl(sub.data(), n, B, C_out, c_off.data(), sub_kept.data(), sub_grads.data(),
                           noisy ? &spec : nullptr, accumulate, s);
        if (st != DP_OK) return st;
      }
    }
    l0 = l1;
  }
  return DP_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------------
// dp_norms_multi for callers that cannot allocate: the per-tile partial sums go to a fixed
// array in the library's own device image instead of a caller-provided workspace.
// ---------------------------------------------------------------------------------
namespace {

constexpr size_t kStaticScratchBytes = (size_t)1 << 20;        // 262144 partial sums
constexpr int kStaticMaxLayers = 1024;

// One copy per device, at its own address; `scratch` itself is only a handle on the host side.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::atomic<void*> scratch_address[kMaxDevices];

// Device address of `scratch` on the current device, resolved once per device.
dp_status static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DP_ERR_HIP;
  void* p = scratch_address[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DP_ERR_HIP;
    scratch_address[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return DP_OK;
}

}  // namespace

extern "C" dp_status dp_norms_multi_static(const dp_layer* layers, int L, dp_dtype dt, int B,
                                           float* sqnorm_out, void* stream) {
  if (!layers || L <= 0) return DP_ERR_INVALID_ARG;
  if (L > kStaticMaxLayers) return DP_ERR_WORKSPACE;
  const size_t need = dp_norms_multi_workspace_bytes(layers, L, dt, B);
  if (need == 0) return DP_ERR_INVALID_ARG;
  if (need > kStaticScratchBytes) return DP_ERR_WORKSPACE;
  void* ws = nullptr;
  dp_status st = static_scratch(&ws);
  if (st != DP_OK) return st;
  // Every partial sum that is read was written by this call's kernels first, so nothing in the
  // array has to start at zero.
  int64_t begin[kStaticMaxLayers];
  int idx[kNormKernels * kStaticMaxLayers];
  return norms_impl(layers, L, dt, B, sqnorm_out, ws, kStaticScratchBytes, static_cast<hipStream_t>(stream),
                    begin, idx);
}

// ---------------------------------------------------------------------------------
// Tile orders of the large-tile kernels, replayed on the host (pure functions, for tests).
// ---------------------------------------------------------------------------------
extern "C" {

int64_t dp_clipped_grad_tile_order(int d_in, int d_out, int32_t* tile_row0, int32_t* tile_col0,
                                   int64_t capacity) {
  if (d_in <= 0 || d_out <= 0 || capacity < 0) return -1;
  const int64_t n = clipped_grad_big_tiles(d_in, d_out);
  if (n > INT32_MAX / 2) return -1;
  const int n_tail = clipped_grad_big_tail_tiles((int)n), n_main = (int)n - n_tail;
  const int tiles_m = (d_in + 255) / 256, tiles_n = (d_out + 255) / 256;
  for (int64_t b = 0; b < n && b < capacity; ++b) {
    // workgroups of the large-tile kernel first, then the tiles left to the sub-tile kernel
    const int t = b < n_main ? grad_logical_tile((int)b, n_main) : (int)b;
    int tm, tn;
    grad_tile_of(tiles_m, tiles_n, t, tm, tn);
    if (tile_row0) tile_row0[b] = tm * 256;
    if (tile_col0) tile_col0[b] = tn * 256;
  }
  return n;
}

int64_t dp_ghost_tile_order(int T, int B, int32_t* sample, int32_t* token_row0, int32_t* token_col0,
                            int32_t* slot, int64_t capacity) {
  if (T <= 0 || B <= 0 || capacity < 0) return -1;
  const int tps = ghost_big_tiles_per_sample(T);
  const int64_t n = (int64_t)tps * B;
  if (n > INT32_MAX / 2) return -1;
  for (int64_t b = 0; b < n && b < capacity; ++b) {
    const GhostTile t = ghost_tile_of(T, tps, ghost_logical_tile((int)b, (int)n));
    if (sample) sample[b] = t.sample;
    if (token_row0) token_row0[b] = t.I * 256;
    if (token_col0) token_col0[b] = t.J * 128;
    if (slot) slot[b] = t.slot;
  }
  return n;
}

}  // extern "C"
