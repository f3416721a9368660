// Order in which the large-tile kernels visit their output tiles.  Pure index arithmetic,
// compiled for the device (the kernels) and for the host (dp_clipped_grad_tile_order and
// dp_ghost_tile_order, which let a CPU test check that every tile is visited exactly once).
#pragma once

#include <hip/hip_runtime.h>

namespace dpbk {

__host__ __device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }
__host__ __device__ __forceinline__ int imax(int a, int b) { return a > b ? a : b; }

// Workgroup id -> work item such that every XCD takes a contiguous eighth of the items:
// workgroup b runs on XCD b % 8 (round-robin dispatch), and XCD x gets items
// [start_x, start_x + n_x) in the order its workgroups are dispatched.  Items that share operand
// panels are numbered consecutively by the callers, so they meet in one XCD's L2.
__host__ __device__ __forceinline__ int contiguous_eighth(int block, int total) {
  const int per = total >> 3, rest = total & 7, xcd = block & 7, idx = block >> 3;
  return xcd < rest ? xcd * (per + 1) + idx : rest * (per + 1) + (xcd - rest) * per + idx;
}

// ---------------------------------------------------------------------------------
// Clip-weighted gradient: 256 x 256 tiles of the [d_in, d_out] gradient.  Tile number `rem` of a
// layer with tiles_m x tiles_n tiles -> tile row and column.  32 consecutive numbers form a patch
// of 4 tile rows x 8 tile columns and 8 consecutive patches a 16 x 16 super-patch (clamped at the
// layer's edges): the 32 compute units of one XCD then pull 12 operand panels per 32 tiles
// through that XCD's L2, and the 8 XCDs 32 panels per 256 tiles through the memory-side cache.
// ---------------------------------------------------------------------------------
__host__ __device__ __forceinline__ void grad_tile_of(int tiles_m, int tiles_n, int rem, int& tm, int& tn) {
  const int sr = imin(rem / (16 * tiles_n), (tiles_m - 1) / 16);      // super-patch row
  rem -= sr * 16 * tiles_n;
  const int hm = imin(16, tiles_m - 16 * sr);
  const int sc = imin(rem / (hm * 16), (tiles_n - 1) / 16);           // super-patch column
  rem -= sc * hm * 16;
  const int wn = imin(16, tiles_n - 16 * sc);
  const int pr = imin(rem / (4 * wn), (hm - 1) / 4);                  // patch row inside it
  rem -= pr * 4 * wn;
  const int ph = imin(4, hm - 4 * pr);
  const int pc = imin(rem / (ph * 8), (wn - 1) / 8);                  // patch column
  rem -= pc * ph * 8;
  tm = 16 * sr + 4 * pr + rem % ph;
  tn = 16 * sc + 8 * pc + rem / ph;
}

// Workgroup id -> tile number of the launch for the gradient kernel.  Workgroup b runs on XCD
// b % 8 (round-robin dispatch) and about 256 consecutive ids are resident at a time.  Within each
// run of 256 ids, XCD x gets the x-th group of 32 consecutive tile numbers, i.e. one 4 x 8 patch.
__host__ __device__ __forceinline__ int grad_logical_tile(int block, int total) {
  constexpr int ROUND = 256;
  const int base = (block / ROUND) * ROUND, q = block - base;
  return base + contiguous_eighth(q, imin(ROUND, total - base));
}

// ---------------------------------------------------------------------------------
// Ghost norm: 256 x 128 tiles (I, J), J >= 2 I, of the T x T Gram matrices of each sample,
// numbered sample by sample and, inside a sample, tile row by tile row (row I has nj - 2 I tiles).
// Consecutive tiles then share their 256-token row block, and every run of 32 tiles that an XCD
// takes holds a mix of diagonal tiles (a quarter of the loads), tiles whose column block lies
// inside the row block, and full tiles, so the XCDs' L2 caches see an even load over time.
// (Measured alternative: numbering by 1024 x 1024-token super-blocks, so that the 32 tiles of an
// XCD touch as few distinct rows as possible, cut the bytes fetched past L2 by a quarter at
// T = 2048 and was 6 % slower: runs of 32 full tiles next to runs of cheap ones.)
// ---------------------------------------------------------------------------------
struct GhostTile {
  int sample;
  int I, J;     // tile row (256 tokens) and tile column (128 tokens)
  int slot;     // index of the tile's partial sum among the layer's: sample * tiles_per_sample + position
};

__host__ __device__ __forceinline__ GhostTile ghost_tile_of(int T, int tiles_per_sample, int e) {
  const int nj = (T + 127) / 128;
  GhostTile t;
  t.sample = e / tiles_per_sample;
  t.slot = e;
  int q = e - t.sample * tiles_per_sample, I = 0;
  while (q >= nj - 2 * I) {
    q -= nj - 2 * I;
    ++I;
  }
  t.I = I;
  t.J = 2 * I + q;
  return t;
}

// Workgroup id -> tile number of the launch for the ghost-norm kernel.  Each XCD takes runs of
// 32 consecutive tile numbers.  Tiles of different layers differ in length (d_in + d_out), so
// the runs are dealt to the XCDs cyclically and the deal rotates by one XCD per round of 256
// tiles: every XCD then sees every part of the launch, whatever the period of the layer pattern
// (contiguous eighths of the launch leave the XCDs with unequal work).
__host__ __device__ __forceinline__ int ghost_logical_tile(int block, int total) {
  constexpr int CHUNK = 32, ROUND = 8 * CHUNK;
  const int round = block / ROUND, base = round * ROUND, qd = block - base;
  const int xcd = qd & 7, idx = qd >> 3;
  if (base + ROUND <= total) return base + ((xcd - round) & 7) * CHUNK + idx;
  // last, partial round: contiguous eighths
  return base + contiguous_eighth(qd, total - base);
}

}  // namespace dpbk
