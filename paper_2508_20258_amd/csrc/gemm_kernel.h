// Tiled bf16 GEMM for gfx950 with a remapped program id: C = A . B, A (M x K), B (K x N),
// C (M x N), all row-major (SwizzlePerf, Appendix "Case Study: GEMM Swizzling").
//
// One workgroup computes one BM x BN tile of C.  Its first scalar instructions turn the
// hardware workgroup id into a tile (pid_decode.h); nothing after that depends on the
// mapping mode, so every mode produces the same bits.
//
// Staging.  Per K step of BK = 32 the workgroup needs an A tile (BM x BK) and a B tile
// (BK x BN).  They are copied global -> LDS by the memory pipeline itself
// (global_load_lds_dwordx4: each lane's 16 bytes land at  M0 base + lane*16, no VGPRs
// involved) into a ring of STAGES buffers, so the loads of steps t+1 .. t+STAGES-1 are in
// flight while the MFMAs of step t run.  A CU's vector memory path moves 64 bytes per clock,
// so a 256x256x64 step (64 KB) needs >= 1024 clocks of transfer on top of the L2/HBM latency,
// against 2048 clocks of MFMA work: one step of look-ahead is not enough, several shorter
// steps are.  A lane cannot choose where
// its bytes land, only what it fetches, so the XOR swizzle of the LDS layout is applied on the
// global-address side: the lane that owns slot p of a row fetches chunk p ^ key(row).
// Out-of-range chunks (rows >= M, columns >= N, k >= K) are fetched from a 16-byte block of
// zeros, which keeps every address valid and makes the K tail exact.
//
// MFMA (v_mfma_f32_16x16x32_bf16, lane l of 64).  Each operand register holds, for one row
// (or column) index l%16, the 8 consecutive k values 8*(l/16) .. +7 of a 32-wide k-block:
//   fragment of A: A[m = l%16][k..]   -> one 16-byte LDS read (A is k-contiguous)
//   fragment of B: B[k..][n = l%16]   -> B is n-contiguous, so it is fetched with two
//       transposing LDS reads (ds_read_b64_tr_b16): inside each 16-lane group, lane s
//       supplies the address of 4 consecutive columns of row s/4, and lane i receives
//       rows 0..3 of column i.
// The B fragment is passed as the instruction's first operand and the A fragment as its
// second, i.e. the instruction computes the 16x16 block of C transposed: lane l, register v
// then holds C[m = l%16][n = 4*(l/16) + v], four consecutive columns, one 8-byte store.
// The 16x16x32 shape is used rather than 32x32x16 because it draws less power for the same
// flops: with random operands held in registers and no memory traffic the chip sustains
// about 2.1 PFLOP/s with it against 1.9 PFLOP/s with 32x32x16 (the clock settles higher).
//
// Main loop.  While the MFMAs of K step t run, the LDS reads of step t+1 and the global loads
// of step t+STAGES-1 are issued, one memory instruction per MFMA slot.  One workgroup barrier
// per step, with no LDS-counter wait attached (the stage that is refilled after it was consumed
// a whole step earlier).  Steps past the end of K are fetched as zeros, which keeps the loop
// free of tail cases: before each barrier exactly STAGES-2 steps are outstanding and the wave
// waits until only STAGES-3 are.
//
// Epilogue.  Each wave converts its accumulators to bf16 (nearest even), writes them to a
// wave-private LDS patch and reads them back row-wise, so that global stores are 16 bytes
// per lane and cover whole 128-byte lines.
//
// LDS layouts (16-byte chunks, XOR-swizzled so that the read patterns spread over banks):
//   A: row r at byte r*64, chunk c (8 k-values) stored in slot c ^ ((r>>2) & 3): the 64 lanes of
//      a fragment read (16 rows x 4 chunks) then cover one contiguous KiB exactly once.
//   B: row k at byte k*BN*2, chunk c (8 columns) stored in slot c ^ (f(k) << 1) with
//      f(k) = (k & 3) | ((k>>3 & 1) << 2): the 8 rows a half-wave reads land in 8 different
//      32-byte bank groups.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "pid_decode.h"

namespace swz {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;


// Source of every out-of-range 16-byte chunk.
__device__ const u32x4 kZeroChunk = {0u, 0u, 0u, 0u};

template <int BM_, int BN_, int BK_, int STAGES_, int WM_, int WN_>
struct GemmShape {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, STAGES = STAGES_, WM = WM_, WN = WN_;
  static constexpr int KK = BK / 32;               // MFMA k-blocks (32 wide) per K step
  static constexpr int NW = WM * WN;               // waves per workgroup
  static constexpr int NT = NW * 64;               // threads per workgroup
  static constexpr int TM = BM / WM / 16;          // 16x16 blocks per wave, rows
  static constexpr int TN = BN / WN / 16;          // 16x16 blocks per wave, columns
  static constexpr int A_BYTES = BM * BK * 2;
  static constexpr int B_BYTES = BK * BN * 2;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int A_ROW_CHUNKS = BK / 8;      // 16-byte chunks per A row
  static constexpr int B_ROW_CHUNKS = BN / 8;      // 16-byte chunks per B row
  static constexpr int A_LOADS = BM * A_ROW_CHUNKS / NT;   // 16-byte chunks each thread moves per step
  static constexpr int B_LOADS = BK * B_ROW_CHUNKS / NT;
  static constexpr int LOADS = A_LOADS + B_LOADS;
  // epilogue patch of one wave: (TM*16) rows of (TN*16) bf16, row pitch padded by 16 bytes
  static constexpr int EPI_PITCH = TN * 16 * 2 + 16;
  static constexpr int EPI_WAVE_BYTES = TM * 16 * EPI_PITCH;
  static constexpr int EPI_BYTES = NW * EPI_WAVE_BYTES;
  static constexpr int LDS_BYTES = STAGES * STAGE_BYTES > EPI_BYTES ? STAGES * STAGE_BYTES : EPI_BYTES;
  static_assert(BK == 32, "K step");
  static_assert(STAGES >= 3 && (STAGES - 1) * LOADS < 64, "ring depth must fit the vmcnt counter");
  static_assert(BM % (WM * 16) == 0 && BN % (WN * 16) == 0, "wave tiling");
  static_assert((BM * A_ROW_CHUNKS) % NT == 0 && (BK * B_ROW_CHUNKS) % NT == 0, "load tiling");
  static_assert(TN * 16 * 2 / 16 <= 64 && 64 % (TN * 16 * 2 / 16) == 0, "epilogue row must divide a wave");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
};

template <int BK>
__device__ __forceinline__ int a_slot(int row, int chunk) {
  return chunk ^ ((row >> 2) & 3);
}

template <int BK>
__device__ __forceinline__ int a_lds_off(int row, int chunk) {
  return row * (BK * 2) + (a_slot<BK>(row, chunk) << 4);
}

// Workgroup barrier alone: no counter waits attached (the kernel states the ones it needs), and
// the memory clobber keeps the compiler from moving LDS accesses across it.
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }

// s_waitcnt that waits only for the vector-memory counter to drop to n.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | 0x0070 | 0x0F00 | ((N >> 4) << 14));
}

__device__ __forceinline__ int b_key(int krow) { return ((krow & 3) | (((krow >> 3) & 1) << 2)) << 1; }

template <int BN>
__device__ __forceinline__ int b_lds_off(int krow, int chunk) {
  return krow * (BN * 2) + ((chunk ^ b_key(krow)) << 4);
}

__device__ __forceinline__ s16x4 lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
}

// 16 bytes per lane, global -> LDS at (wave-uniform) LDS byte address lds_base + lane*16.
// Written as inline assembly on purpose: the compiler then keeps no book on these loads, so it
// does not guard later LDS reads of the *other* stage with a conservative vmcnt(0); the kernel
// waits for them itself (s_waitcnt vmcnt(0) before the barrier that publishes a stage).
__device__ __forceinline__ void load_to_lds(const void* gptr, uint32_t lds_base) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(lds_base);   // wave-uniform by construction
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(gptr) : "memory", "m0");
}

// Same, with the source given as a wave-uniform base (SGPR pair) plus a 32-bit per-lane byte offset.
__device__ __forceinline__ void load_to_lds_base_off(const void* base, uint32_t off, uint32_t lds_base) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(off), "s"(base) : "memory", "m0");
}

// One BM x BN tile of C, tile row pm, tile column pn, by the whole workgroup.  On return every
// wave has issued its stores; LDS may still be read by slower waves (callers that reuse it put a
// barrier first).
template <class S>
__device__ __forceinline__ void gemm_tile(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                          uint16_t* __restrict__ C, int M, int N, int K, int pm, int pn,
                                          unsigned char* smem) {
  constexpr int BM = S::BM, BN = S::BN, BK = S::BK, KK = S::KK, TM = S::TM, TN = S::TN, STAGES = S::STAGES;
  const int m0 = pm * BM;
  const int n0 = pn * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / S::WN;
  const int wn = wave % S::WN;

  // ---- global -> LDS staging: which chunk of the tile this lane fetches for each of its loads ----
  // Load i of wave w fills LDS bytes [(w*LOADS + i)*1024, +1024) of the A (resp. B) region.
  // A lane's source is  tile base (uniform, advances with the K step) + a 32-bit byte offset that
  // never changes.  Rows >= M and columns >= N are clamped to the last valid row / 8-column chunk:
  // whatever they bring in only reaches accumulators of C rows >= M or columns >= N, which are never
  // stored.  Only a K step that crosses the end of K needs zeros, and takes the predicated path.
  uint32_t a_off[S::A_LOADS], b_off[S::B_LOADS];
  int a_k[S::A_LOADS], b_k[S::B_LOADS];       // k offset of the chunk inside a K step
#pragma unroll
  for (int i = 0; i < S::A_LOADS; ++i) {
    const int q = (wave * S::A_LOADS + i) * 64 + lane;
    const int row = q / S::A_ROW_CHUNKS, slot = q % S::A_ROW_CHUNKS;
    const int c = a_slot<BK>(row, slot);       // XOR with a key is its own inverse
    const int r = (m0 + row < M) ? row : (M - 1 - m0);
    a_k[i] = c * 8;
    a_off[i] = (uint32_t)r * (uint32_t)K * 2u + (uint32_t)c * 16u;
  }
#pragma unroll
  for (int i = 0; i < S::B_LOADS; ++i) {
    const int q = (wave * S::B_LOADS + i) * 64 + lane;
    const int krow = q / S::B_ROW_CHUNKS, slot = q % S::B_ROW_CHUNKS;
    const int c = slot ^ b_key(krow);
    const int col = (n0 + c * 8 < N) ? c * 8 : (N - 8 - n0);
    b_k[i] = krow;
    b_off[i] = (uint32_t)krow * (uint32_t)N * 2u + (uint32_t)col * 2u;
  }
  const unsigned char* a_tile = reinterpret_cast<const unsigned char*>(A + (size_t)m0 * K);
  const unsigned char* b_tile = reinterpret_cast<const unsigned char*>(B + n0);
  const size_t a_step = (size_t)BK * 2;           // bytes per K step along a row of A
  const size_t b_step = (size_t)BK * N * 2;       // bytes per K step down the rows of B
  const unsigned char* zero = reinterpret_cast<const unsigned char*>(&kZeroChunk);
  const uint32_t smem_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;   // LDS byte address of the ring

  // Load number idx (0 .. LOADS-1) of K step kt into `stage`; A and B loads alternate.
  // full = the whole step lies inside K (uniform): no per-lane work at all.
  auto issue_load = [&](int kt, int stage, int idx, auto full) __attribute__((always_inline)) {
    const uint32_t sA = smem_addr + stage * S::STAGE_BYTES;
    const uint32_t sB = sA + S::A_BYTES;
    const int i = idx >> 1;
    const bool is_a = (idx & 1) == 0;
    const unsigned char* base = is_a ? a_tile + kt * a_step : b_tile + kt * b_step;
    const uint32_t off = is_a ? a_off[i] : b_off[i];
    const uint32_t dst = is_a ? sA + (wave * S::A_LOADS + i) * 1024 : sB + (wave * S::B_LOADS + i) * 1024;
    if constexpr (decltype(full)::value) {
      load_to_lds_base_off(base, off, dst);
    } else {
      const bool ok = kt * BK + (is_a ? a_k[i] : b_k[i]) < K;
      load_to_lds(ok ? base + off : zero, dst);
    }
  };
  constexpr std::true_type kFull{};
  constexpr std::false_type kTail{};

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

  // lane-constant parts of the fragment addresses
  const int a_row0 = wm * (TM * 16) + (lane & 15);          // + 16*bi
  const int a_kc0 = lane >> 4;                              // 16-byte chunk index along k
  const int b_krow0 = 8 * (lane >> 4) + ((lane & 15) >> 2); // (+4 for the upper half)
  const int b_col0 = wn * (TN * 16) + 4 * (lane & 3);       // + 16*bj

  // Fragment registers.  The MFMAs of a step run A-row-block by A-row-block (bi outer, bj
  // inner), so an A fragment is dead after its TN MFMAs and the same registers take the next
  // step's fragment right away; B fragments are needed by every row-block and are double
  // buffered.  A B fragment is two 8-byte halves.
  bf16x8 af[TM];
  s16x4 bq[2][TN][2];
  constexpr int NM = TM * TN;             // MFMAs per step
  auto read_a = [&](int stage, int bi) __attribute__((always_inline)) {
    const unsigned char* sA = smem + stage * S::STAGE_BYTES;
    af[bi] = *reinterpret_cast<const bf16x8*>(sA + a_lds_off<BK>(a_row0 + 16 * bi, a_kc0));
  };
  auto read_b = [&](int buf, int stage, int bj, int half) __attribute__((always_inline)) {
    const unsigned char* sB = smem + stage * S::STAGE_BYTES + S::A_BYTES;
    const int col = b_col0 + 16 * bj;
    const int kr = b_krow0 + 4 * half;
    bq[buf][bj][half] = lds_read_tr16(sB + b_lds_off<BN>(kr, col >> 3) + (col & 7) * 2);
  };
  auto mfma = [&](int buf, int bi, int bj) __attribute__((always_inline)) {
    const bf16x8 b = __builtin_bit_cast(bf16x8, __builtin_shufflevector(bq[buf][bj][0], bq[buf][bj][1], 0, 1, 2, 3, 4, 5, 6, 7));
    acc[bi][bj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, af[bi], acc[bi][bj], 0, 0, 0);
  };

  // One K step, issued as NM slots.  Slot i = MFMA (bi, bj) on the fragments of the current
  // step, then at most one LDS read for the next step (the B halves in the first 2*TN slots,
  // the A fragment of row-block bi after that block's last MFMA), then, in the middle of every
  // (NM/LOADS)-th run of slots, one global->LDS load of K step ld_kt.  Nothing moves across slot
  // boundaries, so memory instructions are fed to their queues at the pace of the MFMA pipe
  // instead of in bursts that would block the (in-order) wave.
  constexpr int SEG = NM / S::LOADS;
  static_assert(NM % S::LOADS == 0 && S::A_LOADS == S::B_LOADS && 2 * TN <= NM, "slot schedule");
  auto kblock = [&](int cur, int rd_stage, int ld_kt, int ld_stage, auto full) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      const int bi = i / TN, bj = i % TN;
      mfma(cur, bi, bj);
      if (i < 2 * TN) read_b(cur ^ 1, rd_stage, i / 2, i % 2);
      if (bj == TN - 1) read_a(rd_stage, bi);
      if (i % SEG == SEG / 2) issue_load(ld_kt, ld_stage, i / SEG, full);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // K step t lives in stage t%STAGES.  During step t a wave issues the MFMAs of step t, the LDS
  // reads of step t+1, and the global loads of step t+STAGES-1 into the stage of step t-1.
  //   * reads of step t+1 need that step landed for everybody: each wave waits for its own share
  //     (vmcnt) and then meets the others at the barrier that opens step t;
  //   * the refill overwrites the stage of step t-1: every wave consumed its fragments of step t-1
  //     in the MFMAs it issued before arriving at the same barrier, so those reads have completed
  //     and the barrier needs no wait on the LDS counter.
  // Two steps per loop trip keep the fragment-buffer index a compile-time constant; an odd step
  // count just processes one more step of zeros.
  static_assert(KK == 1, "one 32-wide k-block per K step");
  const int KT = (K + BK - 1) / BK;
#pragma unroll
  for (int t = 0; t < STAGES - 1; ++t)
#pragma unroll
    for (int l = 0; l < S::LOADS; ++l) issue_load(t, t, l, kTail);   // steps past K arrive as zeros
  wait_vmcnt<(STAGES - 2) * S::LOADS>();                         // step 0 has landed (this wave's part)
  __syncthreads();                                               // ... and everybody else's
#pragma unroll
  for (int bj = 0; bj < TN; ++bj) {
    read_b(0, 0, bj, 0);
    read_b(0, 0, bj, 1);
  }
#pragma unroll
  for (int bi = 0; bi < TM; ++bi) read_a(0, bi);

  int stage = 0;                       // stage of step kt
  int freed = STAGES - 1;              // stage of step kt-1, refilled during step kt
  auto step = [&](int kt, int cur, auto full) __attribute__((always_inline)) {
    wait_vmcnt<(STAGES - 3) * S::LOADS>();   // step kt+1 has landed (this wave's part)
    block_barrier();
    const int next = (stage + 1 == STAGES) ? 0 : stage + 1;
    kblock(cur, next, kt + STAGES - 1, freed, full);
    freed = stage;
    stage = next;
  };
  const int full_steps = K / BK;       // steps 0 .. full_steps-1 lie wholly inside K
  int kt = 0;
  for (; kt + STAGES < full_steps; kt += 2) {   // both refills of this trip fetch whole steps
    step(kt, 0, kFull);
    step(kt + 1, 1, kFull);
  }
  for (; kt < KT; kt += 2) {
    step(kt, 0, kTail);
    step(kt + 1, 1, kTail);
  }

  // ---- epilogue: fp32 -> bf16 (nearest even), transpose through a wave-private LDS patch ----
  wait_vmcnt<0>();   // the zero-filled look-ahead steps have landed too
  __syncthreads();   // all waves are done with the stage buffers the patches overlay
  unsigned char* patch = smem + wave * S::EPI_WAVE_BYTES;
#pragma unroll
  for (int bi = 0; bi < TM; ++bi) {
#pragma unroll
    for (int bj = 0; bj < TN; ++bj) {
      bf16x4 h;
#pragma unroll
      for (int e = 0; e < 4; ++e) h[e] = (__bf16)acc[bi][bj][e];
      const int r = 16 * bi + (lane & 15);
      const int ccol = 16 * bj + 4 * (lane >> 4);
      *reinterpret_cast<bf16x4*>(patch + r * S::EPI_PITCH + ccol * 2) = h;
    }
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this wave's patch is written (wave-private, no barrier)
  constexpr int ROW_CHUNKS = TN * 16 * 2 / 16;      // 16-byte chunks per patch row
  constexpr int ROWS_PER_PASS = 64 / ROW_CHUNKS;
  const int er = lane / ROW_CHUNKS, ec = lane % ROW_CHUNKS;
#pragma unroll
  for (int p = 0; p < TM * 16 / ROWS_PER_PASS; ++p) {
    const int r = p * ROWS_PER_PASS + er;
    const u32x4 v = *reinterpret_cast<const u32x4*>(patch + r * S::EPI_PITCH + ec * 16);
    const int row = m0 + wm * (TM * 16) + r;
    const int col = n0 + wn * (TN * 16) + ec * 8;
    if (row < M && col < N) *reinterpret_cast<u32x4*>(C + (size_t)row * N + col) = v;
  }
}

// One workgroup per tile.  MODE is a template parameter so that each mapping shows up under its
// own kernel name in profiler traces; only the decode depends on it.
template <class S, int MODE>
__global__ __launch_bounds__(S::NT) void gemm_bf16_kernel(const uint16_t* __restrict__ A,
                                                          const uint16_t* __restrict__ B,
                                                          uint16_t* __restrict__ C, int M, int N, int K,
                                                          int grid_m, int grid_n, int num_xcd, int group_m) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  int pm, pn;
  swz_decode_tile((int)blockIdx.x, grid_m, grid_n, num_xcd, group_m, MODE, &pm, &pn);
  gemm_tile<S>(A, B, C, M, N, K, pm, pn, smem);
}

// Persistent grid: gridDim.x workgroups (one per compute unit) stay resident; workgroup w is
// renumbered among the workgroups and walks the raster with stride gridDim.x, the launch style
// of the paper's GEMM case study (Appendix "Case Study: GEMM Swizzling", num_blocks = number of
// compute units).
template <class S, int MODE>
__global__ __launch_bounds__(S::NT) void gemm_bf16_persistent_kernel(const uint16_t* __restrict__ A,
                                                                     const uint16_t* __restrict__ B,
                                                                     uint16_t* __restrict__ C, int M, int N, int K,
                                                                     int grid_m, int grid_n, int num_xcd, int group_m) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int total = grid_m * grid_n;
  for (int round = 0;; ++round) {
    const int l = swz_persistent_logical((int)blockIdx.x, round, (int)gridDim.x, total, num_xcd, MODE);
    if (l < 0) break;                      // uniform: the whole workgroup leaves together
    int pm, pn;
    swz_raster(l, grid_m, grid_n, group_m, swz_mode_grouped(MODE), &pm, &pn);
    gemm_tile<S>(A, B, C, M, N, K, pm, pn, smem);
    __syncthreads();                       // the next tile's loads overwrite LDS the epilogue read
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

// Persistent flavour: gridDim.x workgroups; workgroup w records, for every round i, the tile it
// would compute (or -1) at tile[i*gridDim.x + w], and once the XCD it ran on at xcc[w].
__global__ void pid_map_persistent_kernel(int grid_m, int grid_n, int num_xcd, int group_m, int mode, int rounds,
                                          int32_t* __restrict__ tile, int32_t* __restrict__ xcc) {
  if (threadIdx.x != 0) return;
  const int w = (int)blockIdx.x, g = (int)gridDim.x;
  for (int round = 0; round < rounds; ++round) {
    const int l = swz_persistent_logical(w, round, g, grid_m * grid_n, num_xcd, mode);
    int t = -1;
    if (l >= 0) {
      int pm, pn;
      swz_raster(l, grid_m, grid_n, group_m, swz_mode_grouped(mode), &pm, &pn);
      t = pm * grid_n + pn;
    }
    tile[(size_t)round * g + w] = t;
  }
  if (xcc != nullptr) xcc[w] = (int32_t)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));
}

// Plain streaming copy of n 16-byte words (reads n*16 bytes, writes n*16 bytes): a kernel of
// known HBM traffic against which profiler byte counters are scaled.
__global__ __launch_bounds__(256) void copy16_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

}  // namespace swz
