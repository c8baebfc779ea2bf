// Tiled bf16 GEMM for gfx950 with a remapped program id: C = A . B, A (M x K), B (K x N),
// C (M x N), all row-major (SwizzlePerf, Appendix "Case Study: GEMM Swizzling").
//
// One workgroup computes one BM x BN tile of C.  Its first scalar instructions turn the
// hardware workgroup id into a tile (pid_decode.h); nothing after that depends on the
// mapping mode, so every mode produces the same bits.
//
// Per K step of 64 the workgroup stages an A tile (BM x 64) and a B tile (64 x BN) in LDS,
// two stages deep: the global loads of step t+1 are in flight while the MFMAs of step t run.
//
// MFMA operand layout (v_mfma_f32_32x32x16_bf16, lane l of 64):
//   A operand: 8 bf16 = A[row = l%32][k = 8*(l/32) .. +7]   -> one 16-byte LDS read (A is k-contiguous)
//   B operand: 8 bf16 = B[k = 8*(l/32) .. +7][col = l%32]   -> B is n-contiguous in memory, so
//              the fragment is fetched with two transposing LDS reads (ds_read_b64_tr_b16):
//              inside each 16-lane group, lane s supplies the address of 4 consecutive
//              columns of row s/4, and lane i receives rows 0..3 of column i.
//   D: lane l, register v holds C[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32].
//
// LDS layouts (16-byte chunks, XOR-swizzled so that the read patterns above spread over banks):
//   A: row r at byte r*128, chunk c (8 k-values) stored at chunk slot c ^ ((r ^ (r>>3)) & 7)
//   B: row k at byte k*BN*2, chunk c (8 columns) stored at chunk slot c ^ ((k & 3) << 2)
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pid_decode.h"

namespace swz {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kBK = 64;

template <int BM_, int BN_, int WM_, int WN_>
struct GemmShape {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int NT = WM * WN * 64;          // threads per workgroup
  static constexpr int TM = BM / WM / 32;          // 32x32 blocks per wave, rows
  static constexpr int TN = BN / WN / 32;          // 32x32 blocks per wave, columns
  static constexpr int A_BYTES = BM * kBK * 2;
  static constexpr int B_BYTES = kBK * BN * 2;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static constexpr int B_ROW_CHUNKS = BN / 8;      // 16-byte chunks per B row
  static constexpr int A_LOADS = BM * 8 / NT;      // 16-byte chunks each thread moves per step
  static constexpr int B_LOADS = kBK * B_ROW_CHUNKS / NT;
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wave tiling");
  static_assert((BM * 8) % NT == 0 && (kBK * B_ROW_CHUNKS) % NT == 0, "load tiling");
};

__device__ __forceinline__ int a_lds_off(int row, int chunk) {
  return row * 128 + ((chunk ^ ((row ^ (row >> 3)) & 7)) << 4);
}

template <int BN>
__device__ __forceinline__ int b_lds_off(int krow, int chunk) {
  return krow * (BN * 2) + ((chunk ^ ((krow & 3) << 2)) << 4);
}

__device__ __forceinline__ s16x4 lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
}

template <class S>
__global__ __launch_bounds__(S::NT) void gemm_bf16_kernel(const uint16_t* __restrict__ A,
                                                          const uint16_t* __restrict__ B,
                                                          uint16_t* __restrict__ C, int M, int N, int K,
                                                          int grid_m, int grid_n, int num_xcd, int group_m,
                                                          int mode) {
  constexpr int BM = S::BM, BN = S::BN, TM = S::TM, TN = S::TN, NT = S::NT;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  int pm, pn;
  swz_decode_tile((int)blockIdx.x, grid_m, grid_n, num_xcd, group_m, mode, &pm, &pn);
  const int m0 = pm * BM;
  const int n0 = pn * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / S::WN;
  const int wn = wave % S::WN;

  // ---- global -> register staging (each thread owns fixed chunks of the A and B tiles) ----
  u32x4 ra[S::A_LOADS], rb[S::B_LOADS];
  auto load_tile = [&](int k0) {
#pragma unroll
    for (int i = 0; i < S::A_LOADS; ++i) {
      const int q = tid + NT * i;
      const int row = q >> 3, c = q & 7;
      const int gr = m0 + row, gk = k0 + c * 8;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (gr < M && gk < K) v = *reinterpret_cast<const u32x4*>(A + (size_t)gr * K + gk);
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < S::B_LOADS; ++i) {
      const int q = tid + NT * i;
      const int row = q / S::B_ROW_CHUNKS, c = q % S::B_ROW_CHUNKS;
      const int gk = k0 + row, gn = n0 + c * 8;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (gk < K && gn < N) v = *reinterpret_cast<const u32x4*>(B + (size_t)gk * N + gn);
      rb[i] = v;
    }
  };
  auto store_tile = [&](int stage) {
    unsigned char* sA = smem + stage * S::STAGE_BYTES;
    unsigned char* sB = sA + S::A_BYTES;
#pragma unroll
    for (int i = 0; i < S::A_LOADS; ++i) {
      const int q = tid + NT * i;
      *reinterpret_cast<u32x4*>(sA + a_lds_off(q >> 3, q & 7)) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < S::B_LOADS; ++i) {
      const int q = tid + NT * i;
      *reinterpret_cast<u32x4*>(sB + b_lds_off<BN>(q / S::B_ROW_CHUNKS, q % S::B_ROW_CHUNKS)) = rb[i];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // lane-constant parts of the fragment addresses
  const int a_row0 = wm * (TM * 32) + (lane & 31);          // + 32*bi
  const int a_kc0 = lane >> 5;                              // + 2*kk  (16-byte chunk index along k)
  const int b_krow0 = 8 * (lane >> 5) + ((lane & 15) >> 2); // + 16*kk (+4 for the upper half)
  const int b_col0 = wn * (TN * 32) + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);  // + 32*bj

  const int KT = (K + kBK - 1) / kBK;
  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int stage = kt & 1;
    if (kt + 1 < KT) load_tile((kt + 1) * kBK);

    const unsigned char* sA = smem + stage * S::STAGE_BYTES;
    const unsigned char* sB = sA + S::A_BYTES;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int bi = 0; bi < TM; ++bi) {
        const int row = a_row0 + 32 * bi;
        af[bi] = *reinterpret_cast<const bf16x8*>(sA + a_lds_off(row, a_kc0 + 2 * kk));
      }
#pragma unroll
      for (int bj = 0; bj < TN; ++bj) {
        const int col = b_col0 + 32 * bj;
        const int kr = b_krow0 + 16 * kk;
        const s16x4 lo = lds_read_tr16(sB + b_lds_off<BN>(kr, col >> 3) + (col & 7) * 2);
        const s16x4 hi = lds_read_tr16(sB + b_lds_off<BN>(kr + 4, col >> 3) + (col & 7) * 2);
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bfr[bj] = __builtin_bit_cast(bf16x8, both);
      }
#pragma unroll
      for (int bi = 0; bi < TM; ++bi)
#pragma unroll
        for (int bj = 0; bj < TN; ++bj)
          acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[bi], bfr[bj], acc[bi][bj], 0, 0, 0);
    }

    if (kt + 1 < KT) store_tile(stage ^ 1);
    __syncthreads();
  }

  // ---- epilogue: fp32 -> bf16 (nearest even), masked stores ----
#pragma unroll
  for (int bi = 0; bi < TM; ++bi) {
#pragma unroll
    for (int bj = 0; bj < TN; ++bj) {
      const int col = n0 + wn * (TN * 32) + 32 * bj + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * (TM * 32) + 32 * bi + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < M && col < N) {
          const __bf16 h = (__bf16)acc[bi][bj][v];
          C[(size_t)row * N + col] = __builtin_bit_cast(uint16_t, h);
        }
      }
    }
  }
}

// Runs only the device PID decode: one workgroup per tile, recording the tile it would
// compute and the XCD it actually landed on (hardware register XCC_ID, bits 3:0).
__global__ void pid_map_kernel(int grid_m, int grid_n, int num_xcd, int group_m, int mode,
                               int32_t* __restrict__ tile, int32_t* __restrict__ xcc) {
  if (threadIdx.x != 0) return;
  const int w = (int)blockIdx.x;
  int pm, pn;
  swz_decode_tile(w, grid_m, grid_n, num_xcd, group_m, mode, &pm, &pn);
  tile[w] = pm * grid_n + pn;
  if (xcc != nullptr) xcc[w] = (int32_t)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));
}

}  // namespace swz
