// Integer PID remap shared by the host entry point and every kernel of the library.
//
// Round-robin dispatch puts hardware workgroup w on XCD x = w mod X (SwizzlePerf,
// Introduction; Appendix "Case Study: GEMM Swizzling").  The paper's closed form,
// (w mod X) * ceil(T/X) + w div X, renumbers workgroups so that every XCD owns a contiguous
// run of logical ids, but it leaves [0,T) whenever T is not a multiple of X.  The form below
// is the same map when X divides T and stays a bijection for every T >= 1, X >= 1:
//
//   q = T div X, r = T mod X.  XCD x receives n_x = q + [x < r] workgroups, the i-th of them
//   being w = i*X + x, so i ranges over [0, n_x).  Give XCD x the id interval starting at
//   s_x = x*q + min(x, r).  Then s_0 = 0, s_{x+1} = s_x + n_x and s_X = T, so the intervals
//   [s_x, s_x + n_x) tile [0, T) without gap or overlap and  w -> s_x + i  is a bijection.
//   (T < X gives q = 0, r = T: the identity.)
//
// The grouped-M raster decodes a logical id l into a tile: rows are cut into bands of
// group_m tile rows (the last band may be shorter, gsz rows); within a band l walks column
// by column, top to bottom inside a column.  (k mod gsz, k div gsz) is the mixed-radix
// decomposition of k in [0, gsz*grid_n), so each band, and hence the grid, is covered once.
//
// The skew (mode bit 4) moves the tile the raster produced down its own column by pn tile rows,
// cyclically: (pm, pn) -> ((pm + pn) mod grid_m, pn).  For every pn this is a rotation of that
// column, hence a bijection of the grid onto itself, and the composition with the raster stays a
// bijection.  A run of consecutive raster positions that stayed in one tile row now walks a
// diagonal.  It serves kernels whose tiles share no data but whose tile rows alias in the memory
// channels: a transpose of a matrix with a power-of-two row pitch writes every tile of a tile row
// into the same few channels, and tiles that run at the same time should therefore differ in
// their tile row as well as in their tile column.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define SWZ_HD __host__ __device__ __forceinline__
#else
#define SWZ_HD inline
#endif

enum : int { kModeRR = 0, kModeXcd = 1, kModeXcdGroupM = 2, kModeGroupM = 3, kModeSkew = 4, kModeCount = 8 };

// XCD renumbering of id w among `total` ids dealt round-robin to num_xcd XCDs (see the proof above).
// Requires 1 <= num_xcd, 0 <= w < total < 2^31.
SWZ_HD int swz_xcd_renumber(int w, int total, int num_xcd) {
  const int q = total / num_xcd;
  const int r = total - q * num_xcd;
  const int i = w / num_xcd;
  const int x = w - i * num_xcd;
  return x * q + (x < r ? x : r) + i;
}

// Tile (pm, pn) visited l-th by the raster.  Requires 1 <= group_m <= grid_m, 0 <= l < grid_m*grid_n.
SWZ_HD void swz_raster(int l, int grid_m, int grid_n, int group_m, bool grouped, int* pm, int* pn) {
  if (grouped) {
    const int width = group_m * grid_n;
    const int band = l / width;
    const int k = l - band * width;
    const int first = band * group_m;
    const int gsz = (grid_m - first < group_m) ? grid_m - first : group_m;
    const int c = k / gsz;
    *pm = first + (k - c * gsz);
    *pn = c;
  } else {
    const int row = l / grid_n;
    *pm = row;
    *pn = l - row * grid_n;
  }
}

SWZ_HD bool swz_mode_renumbers(int mode) { return (mode & 3) == kModeXcd || (mode & 3) == kModeXcdGroupM; }
SWZ_HD bool swz_mode_grouped(int mode) { return (mode & 3) == kModeXcdGroupM || (mode & 3) == kModeGroupM; }
SWZ_HD bool swz_mode_skewed(int mode) { return (mode & kModeSkew) != 0; }

// Tile at raster position l under `mode` (raster, then the skew if the mode asks for it).
// Requirements as swz_raster; pm + pn < 2^31 because grid_m*grid_n < 2^31.
SWZ_HD void swz_tile_at(int l, int grid_m, int grid_n, int group_m, int mode, int* pm, int* pn) {
  swz_raster(l, grid_m, grid_n, group_m, swz_mode_grouped(mode), pm, pn);
  if (swz_mode_skewed(mode)) *pm = (*pm + *pn) % grid_m;
}

// One workgroup per tile.  Requires: 1 <= grid_m, grid_n, num_xcd; 1 <= group_m <= grid_m;
// grid_m*grid_n < 2^31; 0 <= w < grid_m*grid_n.  All intermediate values are <= grid_m*grid_n.
SWZ_HD void swz_decode_tile(int w, int grid_m, int grid_n, int num_xcd, int group_m, int mode, int* pm, int* pn) {
  const int total = grid_m * grid_n;
  const int l = swz_mode_renumbers(mode) ? swz_xcd_renumber(w, total, num_xcd) : w;
  swz_tile_at(l, grid_m, grid_n, group_m, mode, pm, pn);
}

// Persistent grid (the launch style of the paper's own GEMM listing: num_blocks = number of
// compute units): num_wg workgroups stay resident and workgroup w computes, in round
// i = 0, 1, ..., the logical tile  p + i*num_wg,  where p is w renumbered among the num_wg
// workgroups (not among the tiles).  p ranges over [0, num_wg) bijectively, so p + i*num_wg
// visits every logical id in [0, T) exactly once.  Returns the logical id, or -1 once past T.
SWZ_HD int swz_persistent_logical(int w, int round, int num_wg, int total, int num_xcd, int mode) {
  const int p = swz_mode_renumbers(mode) ? swz_xcd_renumber(w, num_wg, num_xcd) : w;
  const int64_t l = (int64_t)p + (int64_t)round * num_wg;
  return l < total ? (int)l : -1;
}
