// Order in which the large-tile kernels visit their output tiles.  Pure index arithmetic,
// compiled for the device (the kernels) and for the host (dp_clipped_grad_tile_order and
// dp_ghost_tile_order, which let a CPU test check that every tile is visited exactly once).
#pragma once

#include <hip/hip_runtime.h>

namespace dpbk {

__host__ __device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }
__host__ __device__ __forceinline__ int imax(int a, int b) { return a > b ? a : b; }

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
  const int n = imin(ROUND, total - base);
  const int per = n >> 3, rest = n & 7, xcd = q & 7, idx = q >> 3;
  return base + (xcd < rest ? xcd * (per + 1) + idx : rest * (per + 1) + (xcd - rest) * per + idx);
}

// ---------------------------------------------------------------------------------
// Ghost norm: 256 x 128 tiles (I, J), J >= 2 I, of the T x T Gram matrices of each sample.
//
// All tiles of one sample read that sample's token rows, tile (I, J) the 256 rows of block I and
// the 128 rows of block J, over the whole width d_in + d_out.  A sample's rows at T = 2048 are
// far larger than an XCD's L2, so rows are shared only by tiles that sweep the width together:
// the 32 tiles an XCD runs at a time should touch as few distinct rows as possible.  The Gram
// matrix is cut into super-blocks of 4 tile rows x 8 tile columns (1024 x 1024 tokens).  An
// off-diagonal super-block holds 32 tiles that read 2048 rows between them; a diagonal one holds
// the 20 tiles of a triangle, which read 1024.  Enumeration of a layer: first the off-diagonal
// super-blocks of every sample (each one a run of 32 consecutive numbers, which is what one XCD
// takes per round), then the diagonal ones.  For T <= 1024 there is one diagonal super-block and
// the order is sample by sample, tile row by tile row.
// ---------------------------------------------------------------------------------
struct GhostTile {
  int sample;
  int I, J;     // tile row (256 tokens) and tile column (128 tokens)
  int slot;     // sample * tiles_per_sample + position: index of the tile's partial sum
};

// Tiles of one sample that lie in off-diagonal super-blocks.
__host__ __device__ __forceinline__ int ghost_offdiag_tiles(int ni, int nj) {
  const int ns = (ni + 3) / 4;
  int n = 0;
  for (int si = 0; si < ns; ++si) {
    const int hi = imin(4, ni - 4 * si);
    for (int sj = si + 1; sj < ns; ++sj) n += hi * imin(8, nj - 8 * sj);
  }
  return n;
}

__host__ __device__ __forceinline__ GhostTile ghost_tile_of(int T, int B, int tiles_per_sample, int e) {
  const int nj = (T + 127) / 128, ni = (T + 255) / 256, ns = (ni + 3) / 4;
  const int n_off = ghost_offdiag_tiles(ni, nj), n_diag = tiles_per_sample - n_off;
  GhostTile t;
  int r;                                                   // position among the sample's tiles
  if (e < B * n_off) {
    t.sample = e / n_off;
    r = e - t.sample * n_off;
  } else {
    e -= B * n_off;
    t.sample = e / n_diag;
    r = n_off + (e - t.sample * n_diag);
  }
  t.slot = t.sample * tiles_per_sample + r;
  t.I = 0;
  t.J = 0;
  if (r < n_off) {
    for (int si = 0; si < ns; ++si) {
      const int hi = imin(4, ni - 4 * si);
      for (int sj = si + 1; sj < ns; ++sj) {
        const int cnt = hi * imin(8, nj - 8 * sj);
        if (r < cnt) {
          t.I = 4 * si + r % hi;
          t.J = 8 * sj + r / hi;
          return t;
        }
        r -= cnt;
      }
    }
    return t;                                              // not reached for e in range
  }
  r -= n_off;
  for (int si = 0; si < ns; ++si) {
    const int hi = imin(4, ni - 4 * si), w = imin(8, nj - 8 * si);
    for (int i = 0; i < hi; ++i) {
      const int cnt = imax(0, w - 2 * i);
      if (r < cnt) {
        t.I = 4 * si + i;
        t.J = 8 * si + 2 * i + r;
        return t;
      }
      r -= cnt;
    }
  }
  return t;                                                // not reached for e in range
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
  const int m = total - base, per = m >> 3, rest = m & 7;
  return base + (xcd < rest ? xcd * (per + 1) + idx : rest * (per + 1) + (xcd - rest) * per + idx);
}

}  // namespace dpbk
