// Tiled 16-bit matrix transpose with a remapped program id:  out (N x M) = in (M x N)^T, both
// row-major (SwizzlePerf, Results and Appendix "Case Study: Other Swizzling Pattern Examples":
// the transpose kernel is the paper's largest win from XCD swizzling).
//
// One workgroup (256 threads) moves one TILE x TILE block: rows of `in` are read as 16-byte
// chunks into LDS, and read back with the transposing LDS read of gfx950 (ds_read_b64_tr_b16:
// inside a 16-lane group, lane s supplies 4 consecutive elements of row s/4 and lane i receives
// rows 0..3 of column i), so a lane ends up with 8 consecutive elements of one row of `out` and
// stores them as 16 bytes.  The kernel is bound by HBM: 4*M*N bytes per launch.
//
// TILE = 128: row segments of 256 bytes on both sides.
// TILE = 64: every row segment read or written is one whole 128-byte line, so tiles share no
//            lines and the mapping of tiles to XCDs cannot change the L2 hit rate.
// TILE = 32: row segments are half lines; horizontally adjacent tiles share the lines they read
//            and vertically adjacent tiles the lines they write.  This is the situation in which
//            co-locating neighbouring tiles on one XCD pays, and it is kept to show exactly that.
// With whole-line tiles what the order of the tiles decides is not the L2 but the memory channels:
// all tiles of one tile row write into the same TILE*2-byte wide column stripe of `out`, and when
// the row pitch of `out` is a power of two that stripe lives in a few channels only.  The skewed
// raster (pid_decode.h) makes tiles that run at the same time differ in their tile row as well as
// in their tile column; measured at 16384 x 16384 it takes the 64-wide tile from 3.9 to 5.2 TB/s
// (the 128-wide one from 4.3 to 4.7), and it costs 1-3 % where the pitch is no power of two.
//
// LDS layout: row r at byte r*(TILE*2), 16-byte chunk c in slot c ^ key(r) (same idea as the
// GEMM's B panel; TILE*2/16 slots per row).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pid_decode.h"

namespace swz {

typedef __attribute__((ext_vector_type(4))) short t_s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t t_u32x4;

template <int TILE>
__device__ __forceinline__ int tr_key(int row) {
  // the 16 lanes of a transposing read take 4 consecutive rows x 32 bytes (a chunk pair): give
  // those rows different chunk pairs where the row has room for it
  return TILE >= 64 ? (row & 3) << 1 : (row & 1) << 1;
}

// STREAM: the whole-line stores are streaming (non-temporal) stores.  That is the faster choice when the
// matrices are larger than the memory-side cache (6.1 against 5.4 TB/s at 16384 x 16384 with the skewed
// raster) and the slower one when `out` would have stayed in that cache (5.5 against 6.2 TB/s at
// 8192 x 8192), so the host decides.
template <int TILE, int MODE, bool STREAM>
__global__ __launch_bounds__(256) void transpose16_kernel(const uint16_t* __restrict__ in, uint16_t* __restrict__ out,
                                                          int M, int N, int grid_m, int grid_n, int num_xcd,
                                                          int group_m, int skew) {
  constexpr int ROW_BYTES = TILE * 2;
  constexpr int SLOTS = ROW_BYTES / 16;                  // 16-byte chunks per tile row
  constexpr int CHUNKS = TILE * SLOTS;                   // chunks per tile
  constexpr int PER_THREAD = CHUNKS / 256 > 0 ? CHUNKS / 256 : 1;
  __shared__ __attribute__((aligned(16))) unsigned char tile[TILE * ROW_BYTES];

  int pm, pn;
  swz_decode_tile((int)blockIdx.x, grid_m, grid_n, num_xcd, group_m, MODE | (skew ? kModeSkew : 0), &pm, &pn);
  const int m0 = pm * TILE, n0 = pn * TILE;
  const int tid = threadIdx.x;

  // ---- in -> LDS: row-contiguous 16-byte chunks (columns are whole chunks: N % 8 == 0) ----
#pragma unroll
  for (int i = 0; i < PER_THREAD; ++i) {
    const int q = tid + 256 * i;
    if (q < CHUNKS) {
      const int r = q / SLOTS, c = q % SLOTS;
      t_u32x4 v = {0u, 0u, 0u, 0u};
      if (m0 + r < M && n0 + c * 8 < N) {
        const t_u32x4* src = reinterpret_cast<const t_u32x4*>(in + (size_t)(m0 + r) * N + n0 + c * 8);
        // whole-line tiles read every line exactly once: streaming loads; half-line tiles rely on the L2 keeping
        // the line for the neighbouring tile
        if constexpr (TILE >= 64) v = __builtin_nontemporal_load(src);
        else v = *src;
      }
      *reinterpret_cast<t_u32x4*>(tile + r * ROW_BYTES + ((c ^ tr_key<TILE>(r)) << 4)) = v;
    }
  }
  __syncthreads();

  // ---- LDS -> out: a unit of work for a wave is 16 columns (rows of out) x 32 rows of the tile ----
  // lane: i = lane%16 -> column, g = lane/16 -> 8-row block; two transposing reads give rows 8g..8g+7
  const int lane = tid & 63, wave = tid >> 6;
  const int i = lane & 15, g = lane >> 4;
  constexpr int COL_BLOCKS = TILE / 16;                  // 16-column blocks
  constexpr int ROW_BLOCKS = TILE / 32;                  // 32-row blocks
  constexpr int UNITS = COL_BLOCKS * ROW_BLOCKS;         // wave-level units of work: 8 (TILE 64) or 2 (TILE 32)
  // what a lane holds after the two transposing reads of 32-row block rb of column block cb:
  // in[m0 + 32rb + 8g .. +7][n0 + 16cb + i]  =  out[n0 + 16cb + i][m0 + 32rb + 8g .. +7], 16 bytes
  auto read_unit = [&](int cb, int rb) __attribute__((always_inline)) {
    const int row = 32 * rb + 8 * g + (i >> 2);          // the row whose 4 elements this lane supplies (+4 for the second read)
    const int col = 16 * cb + 4 * (i & 3);
    const unsigned char* p0 = tile + row * ROW_BYTES + (((col >> 3) ^ tr_key<TILE>(row)) << 4) + (col & 7) * 2;
    const unsigned char* p1 = tile + (row + 4) * ROW_BYTES + (((col >> 3) ^ tr_key<TILE>(row + 4)) << 4) + (col & 7) * 2;
    const t_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) t_s16x4*)p0);
    const t_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) t_s16x4*)p1);
    t_u32x4 v;
    v[0] = (uint32_t)(uint16_t)lo[0] | ((uint32_t)(uint16_t)lo[1] << 16);
    v[1] = (uint32_t)(uint16_t)lo[2] | ((uint32_t)(uint16_t)lo[3] << 16);
    v[2] = (uint32_t)(uint16_t)hi[0] | ((uint32_t)(uint16_t)hi[1] << 16);
    v[3] = (uint32_t)(uint16_t)hi[2] | ((uint32_t)(uint16_t)hi[3] << 16);
    return v;
  };
  if constexpr (ROW_BLOCKS >= 2) {
    // Two 32-row blocks give the two 64-byte halves of 16 lines of `out`.  Lanes i and i + 8 trade one
    // half (a rotation by 8 inside the 16-lane row), after which one store instruction writes 8 whole
    // 128-byte lines (lanes i < 8 their left halves, lanes i >= 8 the right halves) and the next one the other 8.
    constexpr int PAIRS = COL_BLOCKS * (ROW_BLOCKS / 2);
#pragma unroll
    for (int u = wave; u < PAIRS; u += 4) {
      const int cb = u % COL_BLOCKS, rp = u / COL_BLOCKS;
      const t_u32x4 h0 = read_unit(cb, 2 * rp), h1 = read_unit(cb, 2 * rp + 1);
      const bool low = i < 8;
      t_u32x4 got, s0, s1;
#pragma unroll
      for (int e = 0; e < 4; ++e) got[e] = __builtin_amdgcn_mov_dpp(low ? h1[e] : h0[e], 0x128 /* row_ror:8 */, 0xf, 0xf, false);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s0[e] = low ? h0[e] : got[e];
        s1[e] = low ? got[e] : h1[e];
      }
      const int on = n0 + 16 * cb + (i & 7);
      const int om = m0 + 64 * rp + (low ? 0 : 32) + 8 * g;
      if (om < M) {                                        // M % 8 == 0: the 8 elements are in or out together
        t_u32x4* d0 = reinterpret_cast<t_u32x4*>(out + (size_t)on * M + om);
        t_u32x4* d1 = reinterpret_cast<t_u32x4*>(out + (size_t)(on + 8) * M + om);
        if constexpr (STREAM) {
          if (on < N) __builtin_nontemporal_store(s0, d0);
          if (on + 8 < N) __builtin_nontemporal_store(s1, d1);
        } else {
          if (on < N) *d0 = s0;
          if (on + 8 < N) *d1 = s1;
        }
      }
    }
  } else {
#pragma unroll
    for (int u = wave; u < UNITS; u += 4) {
      const int cb = u % COL_BLOCKS, rb = u / COL_BLOCKS;
      const t_u32x4 v = read_unit(cb, rb);
      const int on = n0 + 16 * cb + i;
      const int om = m0 + 32 * rb + 8 * g;
      if (on < N && om < M) *reinterpret_cast<t_u32x4*>(out + (size_t)on * M + om) = v;
    }
  }
}

// Four-byte elements: out (N x M) = in (M x N)^T, one 256-thread workgroup per 64 x 64 block (16 KiB of LDS).
// There is no transposing LDS read for 32-bit elements, so a lane gathers its four consecutive elements of a row
// of `out` with four 4-byte LDS reads from four consecutive tile rows.  A wave instruction covers 8 rows of
// `out` x 32 elements = 8 whole 128-byte lines: lane l takes column 8 jb + l/8 of the tile and tile rows
// 32 h + 4 (l%8) .. +3.  LDS layout: row r at byte r*256, 16-byte chunk c (4 columns) in slot
// c ^ (((r >> 2) & 7) << 1): the 64 lanes of one read (8 row groups x 8 columns = 2 chunks) then hit 64
// different banks.  Same mapping arguments, same streaming-store rule as the 16-bit kernel.
template <int MODE, bool STREAM>
__global__ __launch_bounds__(256) void transpose32_kernel(const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
                                                          int M, int N, int grid_m, int grid_n, int num_xcd,
                                                          int group_m, int skew) {
  constexpr int TILE = 64, SLOTS = TILE / 4, CHUNKS = TILE * SLOTS, ROW_BYTES = TILE * 4;
  __shared__ __attribute__((aligned(16))) unsigned char tile[TILE * ROW_BYTES];
  int pm, pn;
  swz_decode_tile((int)blockIdx.x, grid_m, grid_n, num_xcd, group_m, MODE | (skew ? kModeSkew : 0), &pm, &pn);
  const int m0 = pm * TILE, n0 = pn * TILE;
  const int tid = threadIdx.x;
  auto key = [](int r) { return ((r >> 2) & 7) << 1; };
#pragma unroll
  for (int i = 0; i < CHUNKS / 256; ++i) {
    const int q = tid + 256 * i;
    const int r = q / SLOTS, c = q % SLOTS;
    t_u32x4 v = {0u, 0u, 0u, 0u};
    if (m0 + r < M && n0 + c * 4 < N)               // N % 4 == 0: the 4 elements are in or out together
      v = __builtin_nontemporal_load(reinterpret_cast<const t_u32x4*>(in + (size_t)(m0 + r) * N + n0 + c * 4));
    *reinterpret_cast<t_u32x4*>(tile + r * ROW_BYTES + ((c ^ key(r)) << 4)) = v;
  }
  __syncthreads();
  const int lane = tid & 63, wave = tid >> 6;
  const int jj = lane >> 3, rg = lane & 7;
#pragma unroll
  for (int u = wave; u < 16; u += 4) {                 // 8 column blocks x 2 halves of the tile's rows
    const int jb = u >> 1, h = u & 1;
    const int col = 8 * jb + jj;                       // tile column = row of out
    const int row = 32 * h + 4 * rg;                   // first of this lane's 4 tile rows = column of out
    t_u32x4 v;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      v[k] = *reinterpret_cast<const uint32_t*>(tile + (row + k) * ROW_BYTES + (((col >> 2) ^ key(row + k)) << 4) + (col & 3) * 4);
    const int on = n0 + col, om = m0 + row;
    if (on < N && om < M) {                            // M % 4 == 0
      t_u32x4* dst = reinterpret_cast<t_u32x4*>(out + (size_t)on * M + om);
      if constexpr (STREAM) __builtin_nontemporal_store(v, dst);
      else *dst = v;
    }
  }
}

}  // namespace swz
