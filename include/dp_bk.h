/*
 * dp_bk.h -- C ABI of the Book-Keeping (BK) per-sample clipped-gradient path for
 * linear layers on AMD MI355X (gfx950).
 *
 * The path is the "DP back-propagation" of the paper's section 3 for one
 * micro-batch on one worker, before any ZeRO communication:
 *
 *     per-layer, per-sample squared gradient norms   (appendix A.1, mixed ghost norm)
 *  -> sum over layers, clip factor C_i               (section 2.1, eq. (1), M = 1 group)
 *  -> clipped weighted gradient  a^T diag(C) g       (section 3, "DP gradient")
 *  -> + sigma * R * N(0, I) on a contiguous shard    (eq. (1); ZeRO gradient partition, section 2.2)
 *
 * Notation (section 3): layer input a [B, T, d_in], output gradient g = dL/ds
 * [B, T, d_out], weight gradient [d_in, d_out]; B samples, T tokens per sample.
 *
 * General conventions
 *  - Every data pointer is a DEVICE pointer unless marked "host".  The library
 *    never dereferences a device pointer on the host.
 *  - Tensors are dense and row-major with the last index contiguous.  bf16
 *    tensors must be 16-byte aligned, fp32 tensors 16-byte aligned.
 *  - The caller owns every buffer.  The library allocates no device memory and
 *    never synchronises: work is enqueued on `stream` (a hipStream_t passed as
 *    void*; NULL is the default stream) and the call returns at once.  Calls on
 *    one stream execute in order.  The only state the library keeps between calls
 *    is a per-device table of flags recording which kernels have been allowed
 *    their large LDS allocation (set once, atomically; calls from several host
 *    threads are safe).
 *  - Results are deterministic: no floating-point atomics are used and every sum
 *    is taken in a fixed order, so the same inputs give the same bits on every run.
 *  - Errors are return codes.  Arguments are validated on the host before
 *    anything is launched: a validation error (DP_ERR_INVALID_ARG,
 *    DP_ERR_UNSUPPORTED, DP_ERR_WORKSPACE) means nothing has been enqueued.  A
 *    launch the runtime refuses gives DP_ERR_HIP; the multi-layer calls consist of
 *    several launches, so earlier ones may already be queued then.
 *  - DP_F32 layers run on the vector ALUs, one workgroup per sample in the norm
 *    kernels: they are meant for layers of a few thousand elements.  A norm that
 *    needs more than 2^28 multiply-adds per sample (T^2 (d_in + d_out) / 2 for the
 *    ghost norm, T d_in d_out for the instantiated one) is refused with
 *    DP_ERR_UNSUPPORTED; store such layers in a 16-bit type.
 */
#ifndef DP_BK_H
#define DP_BK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DP_OK = 0,
  DP_ERR_INVALID_ARG = 1,  /* NULL pointer, non-positive size, bad enum, misalignment, bad R/sigma */
  DP_ERR_UNSUPPORTED = 2,  /* valid request this build has no kernel for */
  DP_ERR_WORKSPACE = 3,    /* workspace missing or smaller than dp_norm_workspace_bytes() */
  DP_ERR_HIP = 4           /* the HIP runtime refused a launch */
} dp_status;

/* Storage type of a and g.  The 16-bit types are multiplied on the matrix cores and summed in
 * fp32; every output is fp32.  DP_F16 is IEEE binary16 with subnormals honoured.  No loss scale
 * is applied or expected anywhere (section 3.4, "Mixed-precision training with DP": the clip
 * factor already does the scaling; and with fp32 sums the Gram entries and per-sample norms
 * of the loss-scaling table cannot overflow).  For 16-bit types d_in and d_out must be multiples
 * of 8. */
typedef enum { DP_F32 = 0, DP_BF16 = 1, DP_F16 = 2 } dp_dtype;
typedef enum { DP_CLIP_STANDARD = 0, DP_CLIP_AUTOMATIC = 1 } dp_clip_mode;
typedef enum { DP_PATH_GHOST = 0, DP_PATH_PEREX = 1 } dp_path;

/* One linear layer's book-kept tensors (appendix A.2: activations and output gradients of
 * every layer stay resident until the clip factors are known). */
typedef struct {
  const void* a;   /* device, [B, T, d_in]  */
  const void* g;   /* device, [B, T, d_out] */
  int32_t T;       /* tokens per sample at this layer */
  int32_t d_in;
  int32_t d_out;
  int32_t path;    /* dp_path used for this layer's norm (ignored by dp_clipped_grad_multi) */
} dp_layer;

const char* dp_status_string(dp_status s);

/* Library/ABI version: major*10000 + minor*100 + patch. */
int dp_version(void);

/*
 * Mixed ghost norm selection (appendix A.1: "the cheaper of two techniques at each layer").
 * Pure host function.  Rule: ghost norm iff 2*T^2 <= d_in*d_out (the two T x T Gram
 * matrices take no more room than one instantiated d_in x d_out gradient); ties go to
 * the ghost norm.  Returns DP_PATH_GHOST for non-positive arguments.
 */
dp_path dp_choose_path(int64_t T, int64_t d_in, int64_t d_out);

/*
 * Bytes of device workspace that dp_ghost_norm / dp_perex_norm need for one layer
 * (per-workgroup partial sums that are then added in a fixed order).  Returns 0 for
 * invalid arguments.
 */
size_t dp_norm_workspace_bytes(dp_path path, dp_dtype dt, int B, int T, int d_in, int d_out);

/*
 * Ghost norm (appendix A.1, eq. "mixed ghost norm", right-hand side):
 *   sqnorm_out[i] = sum_{t,t'} (a[i,t,:] . a[i,t',:]) * (g[i,t,:] . g[i,t',:]),   i < B.
 * The two T x T Gram matrices are never written to memory.  bf16 inputs are multiplied
 * exactly and accumulated in fp32.
 *   a, g        device inputs, [B,T,d_in] and [B,T,d_out] of type dt
 *   sqnorm_out  device, [B] fp32, overwritten
 *   ws          device scratch of at least dp_norm_workspace_bytes(DP_PATH_GHOST, ...) bytes,
 *               16-byte aligned; contents undefined afterwards
 * bf16 requires d_in and d_out to be multiples of 8 (16-byte rows).
 */
dp_status dp_ghost_norm(const void* a, const void* g, dp_dtype dt, int B, int T, int d_in,
                        int d_out, float* sqnorm_out, void* ws, size_t ws_bytes, void* stream);

/*
 * Per-sample gradient instantiation norm (appendix A.1, left-hand side):
 *   sqnorm_out[i] = || a[i]^T g[i] ||_F^2,   a[i]^T g[i] in R^{d_in x d_out}.
 * The per-sample gradients live only in accumulator registers.  Same arguments,
 * alignment rules and workspace protocol as dp_ghost_norm (with DP_PATH_PEREX).
 */
dp_status dp_perex_norm(const void* a, const void* g, dp_dtype dt, int B, int T, int d_in,
                        int d_out, float* sqnorm_out, void* ws, size_t ws_bytes, void* stream);

/*
 * Cross-layer accumulation and clip factor (section 2.1; all-layer clipping, one group):
 *   norm_i = sqrt(max(0, sum_l sqnorm[l*B + i]))            (layers added in a fixed order)
 *   DP_CLIP_STANDARD :  C_i = min(R / norm_i, 1)            (norm_i = 0 gives C_i = 1)
 *   DP_CLIP_AUTOMATIC:  C_i = R / (norm_i + stability)      (the paper prints R = 1, stability 0.01;
 *                                                            norm_i + stability = 0 gives C_i = 0)
 * A sum that is NaN gives norm_i = C_i = NaN in both modes (the sample's gradient is not a
 * number and the weighted gradient will show it); an infinite norm gives C_i = 0.
 *   sqnorm    device, [L, B] fp32 row-major
 *   C_out     device, [B] fp32
 *   norm_out  device, [B] fp32, or NULL
 * R must be > 0 (+infinity allowed: standard clipping then gives C = 1); stability >= 0.
 * Layer-wise clipping is this call with L = 1 per layer.
 */
dp_status dp_clip_factors(const float* sqnorm, int L, int B, dp_clip_mode mode, float R,
                          float stability, float* C_out, float* norm_out, void* stream);

/*
 * Clip-weighted gradient (section 3, "DP gradient" without the noise term):
 *   grad[j, k] (+)= sum_i C[i] * sum_t a[i,t,j] * g[i,t,k],   j < d_in, k < d_out.
 * C[i] is applied in fp32 to sample i's exact partial product, never to the bf16 inputs.
 * Samples with C[i] == 0 are not read.  The 16-bit kernels keep one accumulator, expressed in
 * units of the current sample's weight, and multiply it by C[i] / C[i+1] between samples: any
 * finite weights work whose ratios C[i] / C[j] (j the next sample with a non-zero weight) times
 * the largest partial sum stay inside fp32 range -- in particular every set of clip factors of
 * section 2.1, which lie in (0, 1] or in (0, R / stability]; ratios up to 1e10 either way are
 * tested.  Beyond that range (for instance a subnormal weight next to a normal one) the result
 * overflows to inf or NaN rather than being silently wrong.  A NaN weight gives a NaN gradient.
 *   C           device, [B] fp32
 *   grad        device, [d_in, d_out] fp32 row-major
 *   accumulate  0: overwrite grad; 1: add to it (gradient accumulation over micro-batches)
 * bf16 requires d_in and d_out to be multiples of 8.
 */
dp_status dp_clipped_grad(const void* a, const void* g, dp_dtype dt, int B, int T, int d_in,
                          int d_out, const float* C, float* grad, int accumulate, void* stream);

/*
 * Gaussian mechanism on one rank's contiguous gradient shard (eq. (1) with one group):
 *   grad_slice[e - global_offset] += sigma * R * z_e,   e in [global_offset, global_offset+count)
 * z_e ~ N(0,1) is a pure function of (seed, step, e): Philox4x32-10 block k = e >> 2 with
 * counter (k_lo, k_hi, step_lo, step_hi) and key (seed_lo, seed_hi) gives (x0,x1,x2,x3);
 * u = ((x >> 9) + 0.5) * 2^-23; (z_{4k}, z_{4k+1}) = sqrt(-2 ln u(x0)) * (cos, sin)(2 pi u(x1)),
 * (z_{4k+2}, z_{4k+3}) likewise from (x2, x3).  Any sharding of the flattened gradient
 * therefore draws the same noise.  A (seed, step) pair must not be reused.
 *   grad_slice     device, fp32, points at element global_offset; 4-byte aligned
 *   sigma          noise multiplier, >= 0; sigma == 0 enqueues nothing (R may be +inf then)
 *   R              clipping threshold, > 0 and finite when sigma > 0
 */
dp_status dp_add_noise(float* grad_slice, uint64_t global_offset, uint64_t count, float sigma,
                       float R, uint64_t seed, uint64_t step, void* stream);

/*
 * Raw generator stream, for verification: out[4*j .. 4*j+3] = Philox4x32-10 output of block
 * first_block + j under the counter/key layout documented at dp_add_noise.
 *   out  device, uint32 [4*n_blocks], 16-byte aligned
 */
dp_status dp_philox_blocks(uint32_t* out, uint64_t first_block, uint64_t n_blocks, uint64_t seed,
                           uint64_t step, void* stream);

/*
 * Grouped forms over a stack of layers: one launch covers every layer, so small layers
 * (GPT-2-sized: tens of tiles each) still fill the 256 compute units.  Semantics are exactly
 * L calls of the per-layer function.
 *
 * dp_norms_multi: sqnorm_out[l*B + i] for every layer l, by layers[l].path.
 *   layers    HOST array of L descriptors (copied before the call returns)
 *   ws        device scratch, >= dp_norms_multi_workspace_bytes(...), 16-byte aligned
 *             (fp32 layers need none: ws may be NULL when dt == DP_F32)
 * dp_clipped_grad_multi: grads[l] as dp_clipped_grad for every layer.
 *   grads     HOST array of L device pointers, grads[l] -> [d_in_l, d_out_l] fp32, 16-byte aligned
 * Layer descriptors travel in kernel arguments (at most 48 layers per launch; longer stacks
 * take several launches), so both calls are safe under stream capture.
 */
size_t dp_norms_multi_workspace_bytes(const dp_layer* layers, int L, dp_dtype dt, int B);
dp_status dp_norms_multi(const dp_layer* layers, int L, dp_dtype dt, int B, float* sqnorm_out,
                         void* ws, size_t ws_bytes, void* stream);
dp_status dp_clipped_grad_multi(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                float* const* grads, int accumulate, void* stream);

/*
 * dp_norms_multi without a workspace argument, for callers that cannot allocate device memory
 * where they call it: code under HIP stream capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The per-tile partial sums go to a fixed 1 MiB array that is part of the library's
 * device image (one copy per GPU, held until the process ends); the call allocates and frees
 * nothing, on the device or on the host, and gives bit for bit the results of dp_norms_multi.
 *   DP_ERR_WORKSPACE  the stack needs more than 1 MiB of partial sums (more than 262144 tiles
 *                     times samples; dp_norms_multi_workspace_bytes tells) or has more than 1024
 *                     layers: use dp_norms_multi with a workspace of your own
 * The first call on each device looks up the array's device address (no allocation, but do it
 * once outside stream capture).  All calls on one GPU share the array: calls that may overlap
 * in time on one GPU (different streams, several host threads) race on it and must be
 * serialised by the caller; calls on one stream are ordered and safe.
 */
dp_status dp_norms_multi_static(const dp_layer* layers, int L, dp_dtype dt, int B, float* sqnorm_out,
                                void* stream);

/*
 * dp_clipped_grad_multi with the noise of eq. (1) added in the same pass ("DP gradient" of
 * section 3 in one step): the result is what dp_clipped_grad_multi followed by dp_add_noise on
 * the same elements gives, value for value, without the second pass over the gradient.  For
 * callers whose clipped sums are already final when they are formed: one device, or each rank
 * adding its own share of the noise before the reduction (the appendix on the user interface).
 *
 * Element j of layer l's gradient has global index grad_offset[l] + j; it receives
 * sigma * R * z_index when shard_offset <= index < shard_offset + shard_count (z as documented
 * at dp_add_noise: the same generator, seed, step and indexing), and no noise otherwise.
 *   grad_offset  HOST array of L global element offsets (the layers' places in the flattened
 *                model; they need not be contiguous or ordered, but must not overlap)
 *   sigma, R     as dp_add_noise (sigma >= 0, finite; R > 0; sigma == 0 adds nothing)
 * Layers that the large-tile kernels compute and whose grad_offset is a multiple of 4 get the
 * noise in the kernel's epilogue; for all others the noise pass runs on the layer's slice
 * after its gradient.  Errors as dp_clipped_grad_multi and dp_add_noise.
 */
dp_status dp_clipped_grad_noise_multi(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                      float* const* grads, const uint64_t* grad_offset, int accumulate,
                                      uint64_t shard_offset, uint64_t shard_count, float sigma, float R,
                                      uint64_t seed, uint64_t step, void* stream);

/*
 * dp_clipped_grad_noise_multi with the gradient stored in 16 bits, in the storage type of a and g
 * (mixed-precision training keeps parameters, activations and gradients in half precision:
 * section 2.3): the fp32 value that dp_clipped_grad_noise_multi would store -- weighted sum, plus
 * the old value widened to fp32 when accumulate == 1, plus the noise -- is rounded once, to nearest
 * even, to bf16 (dt == DP_BF16) or IEEE binary16 (dt == DP_F16).
 *   grads16   HOST array of L device pointers, grads16[l] -> [d_in_l, d_out_l] of type dt, 16-byte aligned
 * Only the large-tile kernels write 16-bit gradients: every layer needs d_in, d_out >= 128, T a
 * multiple of 32, a sample's a and g below 2 GiB each, and (when sigma > 0) a grad_offset that is a
 * multiple of 4; otherwise, and for dt == DP_F32, DP_ERR_UNSUPPORTED (nothing is enqueued).
 */
dp_status dp_clipped_grad_noise_multi_h16(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                          void* const* grads16, const uint64_t* grad_offset, int accumulate,
                                          uint64_t shard_offset, uint64_t shard_count, float sigma, float R,
                                          uint64_t seed, uint64_t step, void* stream);

/*
 * Group-wise clipping (eq. (1) with M groups; section 2.1, "Mathematical gradient partition":
 * all-layer clipping is one group, layer-wise clipping one group per layer, the paper's default).
 * The rows of sqnorm (one per layer weight, plus one per bias when biases are trained) are
 * partitioned into M contiguous groups: group m owns rows [group_begin[m], group_begin[m+1]) and
 * has its own threshold R[m]:
 *   norm_{m,i} = sqrt(max(0, sum of the group's rows at sample i)),  C_{m,i} = clip(norm_{m,i}; R[m]).
 *   sqnorm       device, [L, B] fp32
 *   group_begin  HOST, [M+1] ascending, group_begin[0] = 0, group_begin[M] = L (empty groups allowed)
 *   R            HOST, [M], each > 0
 *   C_out        device, [M, B] fp32;  norm_out device [M, B] or NULL
 * dp_clipped_grad_grouped is dp_clipped_grad_multi with layer l weighted by row group_of_layer[l]
 * (HOST, [L], values in [0, M)) of C [M, B].
 * The noise of eq. (1) has standard deviation sigma * ||[R_1..R_M]||_2: pass
 * dp_group_noise_threshold(R, M) as the R of dp_add_noise.
 */
dp_status dp_clip_factors_grouped(const float* sqnorm, int L, int B, const int32_t* group_begin, int M,
                                  const float* R, dp_clip_mode mode, float stability, float* C_out,
                                  float* norm_out, void* stream);
dp_status dp_clipped_grad_grouped(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                  const int32_t* group_of_layer, int M, float* const* grads,
                                  int accumulate, void* stream);
float dp_group_noise_threshold(const float* R, int M);

/*
 * Book-keeping for layers on the instantiated path (appendix A.2 applied to the left side of
 * appendix A.1's equation): the norm kernel already forms every per-sample gradient
 * G_{l,i} = a_{l,i}^T g_{l,i}; when the caller gives it room, it keeps them, and the
 * clip-weighted gradient is then sum_i C_i G_{l,i} -- a stream over B arrays of d_in * d_out floats
 * instead of a second contraction over the T tokens of a and g.  The rule that puts a layer on
 * this path (2 T^2 > d_in * d_out) also makes the kept gradients smaller than the layer's two
 * Gram matrices would be.
 * dp_norms_multi_keep: dp_norms_multi, and for every layer with kept[l] != NULL also
 *   kept[l][i, j, k] = sum_t a[i,t,j] g[i,t,k]   (fp32, [B, d_in, d_out], overwritten).
 *   kept   HOST array of L device pointers (16-byte aligned) or NULLs; NULL array = keep nothing.
 *          A non-NULL entry needs path == DP_PATH_PEREX and 16-bit storage (else
 *          DP_ERR_INVALID_ARG / DP_ERR_UNSUPPORTED).
 * dp_clipped_grad_kept_multi: dp_clipped_grad_noise_multi, with the layers that have kept[l] != NULL
 *   computed from kept[l] (a and g of those layers are not read; their descriptors still give
 *   the shapes).  Samples are added in index order in fp32; samples with C[i] == 0 are not read.
 *   grad_offset may be NULL when sigma == 0 or shard_count == 0.
 */
dp_status dp_norms_multi_keep(const dp_layer* layers, int L, dp_dtype dt, int B, float* sqnorm_out,
                              float* const* kept, void* ws, size_t ws_bytes, void* stream);
dp_status dp_clipped_grad_kept_multi(const dp_layer* layers, int L, dp_dtype dt, int B, const float* C,
                                     float* const* kept, float* const* grads, const uint64_t* grad_offset,
                                     int accumulate, uint64_t shard_offset, uint64_t shard_count, float sigma,
                                     float R, uint64_t seed, uint64_t step, void* stream);

/*
 * Layer-wise clipping without book-keeping (section 3.3 (II), and the per-layer formula of the
 * appendix on the hook-free implementation).  With one clipping group per layer, C_{l,i} depends
 * on layer l alone, so nothing forces "all norms first, then all gradients": the stack is walked
 * in passes of consecutive layers, and each pass runs norms -> clip factors -> weighted
 * gradients (+ noise) before the next is touched, so a pass's a and g are still in the
 * memory-side cache when the gradient kernels read them again.  A layer on the instantiated
 * path (path == DP_PATH_PEREX, 16-bit storage) whose whole gradient fits one workgroup tile (up to
 * 128 x 128, 512 x 32 or 32 x 512) is done in ONE kernel that reads a and g once: per sample it
 * forms G_i = a_i^T g_i in registers, takes ||G_i||, C_i = clip(||G_i||; R_l) and adds C_i G_i.
 * A larger layer on the instantiated path keeps its G_i ([B, d_in, d_out] fp32) in the workspace
 * between its norm kernel and a weighted sum, as dp_norms_multi_keep + dp_clipped_grad_kept_multi
 * do, so its a and g are read once as well; layers are given room in stack order up to 2 GiB in
 * total, the rest contract a and g a second time.
 * The result is that of dp_norms_multi + dp_clip_factors_grouped (one group per layer)
 * + dp_clipped_grad_grouped + dp_add_noise with R = dp_group_noise_threshold(R, L):
 *   grads[l] (+)= sum_i C[l,i] a_{l,i}^T g_{l,i} + sigma ||(R_1..R_L)||_2 z   on the shard's elements.
 *   R            HOST, [L], each > 0 (finite when sigma > 0)
 *   grads        HOST array of L device pointers, as dp_clipped_grad_multi
 *   grad_offset  HOST, [L] global element offsets as dp_clipped_grad_noise_multi (may be NULL when
 *                sigma == 0 or shard_count == 0)
 *   sqnorm_out, C_out   device, [L, B] fp32, overwritten
 *   ws           device scratch >= dp_layerwise_workspace_bytes(...), 16-byte aligned
 *   layers_per_pass   0: a pass ends once it holds 128 MiB of a and g and 1024 gradient tiles;
 *                     > 0: that many layers per pass
 */
size_t dp_layerwise_workspace_bytes(const dp_layer* layers, int L, dp_dtype dt, int B);
dp_status dp_layerwise_clipped_grad(const dp_layer* layers, int L, dp_dtype dt, int B, const float* R,
                                    dp_clip_mode mode, float stability, float* const* grads,
                                    const uint64_t* grad_offset, int accumulate, uint64_t shard_offset,
                                    uint64_t shard_count, float sigma, uint64_t seed, uint64_t step,
                                    float* sqnorm_out, float* C_out, void* ws, size_t ws_bytes,
                                    int layers_per_pass, void* stream);

/*
 * Bias gradients (appendix A.1, last paragraph): the per-sample bias gradient is 1^T dL/ds_i, the
 * sum of sample i's T rows of g; its norm is taken by instantiation.
 * dp_bias_norm:  colsum[i, k] = sum_t g[i, t, k]  and  sqnorm_out[i] = sum_k colsum[i, k]^2.
 *   g           device, [B, T, d_out] of type dt (bf16: d_out a multiple of 8), 16-byte aligned
 *   colsum      device, [B, d_out] fp32, overwritten; keep it for dp_clipped_bias_grad
 *   sqnorm_out  device, [B] fp32, overwritten (use it as one more row of sqnorm)
 * dp_clipped_bias_grad:  grad_b[k] (+)= sum_i C[i] * colsum[i, k]   (g is not read again).
 *   C device [B];  grad_b device [d_out] fp32;  accumulate 0 or 1
 */
dp_status dp_bias_norm(const void* g, dp_dtype dt, int B, int T, int d_out, float* colsum,
                       float* sqnorm_out, void* stream);
dp_status dp_clipped_bias_grad(const float* colsum, int B, int d_out, const float* C, float* grad_b,
                               int accumulate, void* stream);

/*
 * Order in which the large-tile matrix-core kernels visit their output tiles, replayed on the
 * host (pure functions; nothing is launched).  They exist so that a test without a GPU can check
 * that every tile of a layer is computed exactly once for any shape; the arrays may be NULL.
 * dp_clipped_grad_tile_order: tile b of a one-layer launch of the clip-weighted gradient
 *   (section 3, "DP gradient") starts at row tile_row0[b], column tile_col0[b] of the
 *   [d_in, d_out] gradient; tiles are 256 x 256.
 * dp_ghost_tile_order: workgroup b of a one-layer ghost-norm launch (appendix A.1) computes, for
 *   sample[b], the 256 x 128 block of the two Gram matrices at token rows token_row0[b], token
 *   columns token_col0[b] (always on or above the diagonal), and writes partial sum slot[b].
 * Both return the number of tiles (at most `capacity` entries are written), or -1 for invalid
 * arguments.  All pointers are HOST pointers.
 */
int64_t dp_clipped_grad_tile_order(int d_in, int d_out, int32_t* tile_row0, int32_t* tile_col0,
                                   int64_t capacity);
int64_t dp_ghost_tile_order(int T, int B, int32_t* sample, int32_t* token_row0, int32_t* token_col0,
                            int32_t* slot, int64_t capacity);

#ifdef __cplusplus
}
#endif
#endif /* DP_BK_H */
