// Tiled bf16 GEMM for gfx950 with a remapped program id: C = A . B, A (M x K), B (K x N),
// C (M x N), all row-major (SwizzlePerf, Appendix "Case Study: GEMM Swizzling").
//
// One workgroup computes one BM x BN tile of C.  Its first scalar instructions turn the
// hardware workgroup id into a tile (pid_decode.h); nothing after that depends on the
// mapping mode, so every mode produces the same bits.
//
// Staging.  The K loop advances in steps of 32.  Operands are copied global -> LDS by the
// memory pipeline itself (global_load_lds_dwordx4: each lane's 16 bytes land at
// M0 base + lane*16, no VGPRs involved) into two rings:
//   A ring: 3 slots, each a "double" BM x 64 (two K steps), so that a lane group fetches whole
//           128-byte lines of a row of A; a 32-wide slice would fetch every line as two
//           64-byte halves, i.e. twice the L2 requests for the same bytes (measured: +2.5 %
//           time).
//   B ring: 4 slots, each 32 x BN (rows of B are whole lines already).
// A CU's vector memory path moves 64 bytes per clock, so a 256x256x64 panel pair (64 KB) needs
// >= 1024 clocks of transfer on top of the L2/HBM latency against 2048 clocks of MFMA work: the
// loads run about three steps ahead of their use.  A lane cannot choose where its bytes land,
// only what it fetches, so the XOR swizzle of the LDS layout is applied on the global-address
// side: the lane that owns slot p of a row fetches chunk p ^ key(row).
// Rows >= M and columns >= N are fetched from clamped, valid addresses (what they bring in only
// reaches accumulators that are never stored); chunks with k >= K are fetched from a 16-byte
// block of zeros, which makes the K tail exact.
//
// MFMA (v_mfma_f32_16x16x32_bf16, lane l of 64).  Each operand register holds, for one row
// (or column) index l%16, the 8 consecutive k values 8*(l/16) .. +7 of a 32-wide K step:
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
// Main loop.  The eight waves form two groups of four; the two waves that share a SIMD are in
// different groups.  Time is cut into phases separated by workgroup barriers.  In a phase one
// group issues the 32 MFMAs of a K step back to back and nothing else, while the other group
// does the memory work of its next step (its share of the global->LDS loads, then all fragment
// reads from LDS) and waits for it; then the groups swap.  On each SIMD the MFMA pipe so sees
// one uninterrupted instruction stream at a time.  Measured on the same device against a loop
// in which every wave interleaves its own LDS reads and loads with its MFMAs: 1045-1070 clocks
// per K step instead of 1240 (1024 = MFMA pipe never idle).  The reasons, each measured:
//   * the SIMD issues MFMAs of the older wave first, so two waves that both have MFMAs ready do
//     not alternate; one starves and its memory instructions, queued behind its MFMAs (issue is
//     in order), come late;
//   * an LDS read in the middle of a wave's MFMA stream costs that stream about 13 clocks;
//   * in a memory phase nothing may be computed on the vector ALU per read: the 16 reads are one
//     of eight precomputed address registers plus an immediate, which needs the position of the
//     step in the ring cycle (12 steps: 4 B slots, 3 A doubles) at compile time, hence a main
//     loop body of 12 steps.  With address arithmetic in the phase it took longer than the 512
//     clocks of the other group's MFMAs and the MFMA pipe idled 10 % of the time.
// Steps past the end of K are fetched as zeros, which keeps the loop free of tail cases.
//
// Epilogue.  Each wave converts its accumulators to bf16 (nearest even) and rearranges them across
// lanes in registers (v_permlane16_swap between the registers of two neighbouring column blocks, then
// a rotation by 8 inside each 16-lane row), so that every lane holds 16 contiguous bytes and one
// store instruction covers whole 128-byte lines.  LDS is not involved, which lets a workgroup that
// has another tile to compute (persistent launch) start that tile's first loads before it converts
// and stores the current one.  Measured: neither the register epilogue (against a transposition
// through LDS patches) nor the overlap changes the rate by more than the noise, 0.5 %: what the
// chip delivers on this kernel is set by the power its arithmetic and its operand traffic draw, not
// by the few microseconds at either end of a tile.
//
// LDS layouts (16-byte chunks, XOR-swizzled so that the read patterns spread over banks):
//   A: row r at byte r*128, chunk c (8 k-values, c = 0..7 over the double) stored in slot
//      c ^ ((r>>1) & 7): the 16 lanes that read one chunk index of 16 consecutive rows hit 16
//      different 16-byte bank groups.
//   B: row k at byte k*BN*2, chunk c (8 columns) stored in slot c ^ (f(k) << 1) with
//      f(k) = (k & 3) | ((k>>3 & 1) << 2): the 8 rows a half-wave reads land in 8 different
//      32-byte bank groups.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "pid_decode.h"

namespace swz {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Source of every chunk that lies past the end of K.
__device__ const u32x4 kZeroChunk = {0u, 0u, 0u, 0u};

constexpr int kStepK = 32;     // K extent of one main-loop step (one 16x16x32 MFMA deep)
constexpr int kASlots = 3;     // A ring: doubles (two steps each)
constexpr int kBSlots = 4;     // B ring: single steps

template <int BM_, int BN_, int WM_, int WN_>
struct GemmShape {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int NW = WM * WN;               // waves per workgroup
  static constexpr int NT = NW * 64;               // threads per workgroup
  static constexpr int TM = BM / WM / 16;          // 16x16 blocks per wave, rows
  static constexpr int TN = BN / WN / 16;          // 16x16 blocks per wave, columns
  static constexpr int A_SLOT_BYTES = BM * 2 * kStepK * 2;   // BM rows x 64 k
  static constexpr int B_SLOT_BYTES = kStepK * BN * 2;       // 32 rows x BN
  static constexpr int A_RING_BYTES = kASlots * A_SLOT_BYTES;
  static constexpr int RING_BYTES = A_RING_BYTES + kBSlots * B_SLOT_BYTES;
  static constexpr int B_ROW_CHUNKS = BN / 8;      // 16-byte chunks per B row
  static constexpr int A_LOADS = BM * 8 / NT;      // 16-byte chunks each thread moves per A double
  static constexpr int B_LOADS = kStepK * B_ROW_CHUNKS / NT;   // ... per B step
  static constexpr int LOADS = A_LOADS / 2 + B_LOADS;          // loads each thread issues per step
  static constexpr int LDS_BYTES = RING_BYTES;
  static_assert(BM % (WM * 16) == 0 && BN % (WN * 16) == 0, "wave tiling");
  static_assert((BM * 8) % NT == 0 && (kStepK * B_ROW_CHUNKS) % NT == 0 && A_LOADS % 2 == 0, "load tiling");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
};

__device__ __forceinline__ int a_slot(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ int a_lds_off(int row, int chunk) { return row * 128 + (a_slot(row, chunk) << 4); }

__device__ __forceinline__ int b_key(int krow) { return ((krow & 3) | (((krow >> 3) & 1) << 2)) << 1; }

template <int BN>
__device__ __forceinline__ int b_lds_off(int krow, int chunk) {
  return krow * (BN * 2) + ((chunk ^ b_key(krow)) << 4);
}

__device__ __forceinline__ s16x4 lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
}

// Workgroup barrier alone: no counter waits attached (the kernel states the ones it needs), and
// the memory clobber keeps the compiler from moving LDS accesses across it.
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }

// s_waitcnt on the vector-memory counter (<= VM) and the LDS counter (<= LGKM) together.
template <int VM, int LGKM>
__device__ __forceinline__ void wait_vmcnt_lgkmcnt() {
  static_assert(VM >= 0 && VM < 64 && LGKM >= 0 && LGKM < 16, "counter ranges");
  __builtin_amdgcn_s_waitcnt((VM & 0xF) | 0x0070 | (LGKM << 8) | ((VM >> 4) << 14));
}

// s_waitcnt that waits only for the vector-memory counter to drop to n.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | 0x0070 | 0x0F00 | ((N >> 4) << 14));
}

// 16 bytes per lane, global -> LDS at (wave-uniform) LDS byte address lds_base + lane*16.
// Written as inline assembly on purpose: the compiler then keeps no book on these loads, so it
// does not guard later LDS reads of *other* ring slots with a conservative vmcnt(0); the kernel
// waits for them itself (s_waitcnt vmcnt before the barrier that publishes a slot).
// M0 is written by the scalar unit right before the load that reads it: on this generation such a
// write needs one wait state before an LDS-DMA instruction uses it, and the compiler inserts wait
// states only between instructions it emits itself, hence the s_nop inside the asm block.
__device__ __forceinline__ void load_to_lds(const void* gptr, uint32_t lds_base) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(lds_base);   // wave-uniform by construction
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(gptr) : "memory", "m0");
}

// Same, with the source given as a wave-uniform base (SGPR pair) plus a 32-bit per-lane byte offset.
__device__ __forceinline__ void load_to_lds_base_off(const void* base, uint32_t off, uint32_t lds_base) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(off), "s"(base) : "memory", "m0");
}

// f(integral_constant<int, 0>{}), f(integral_constant<int, 1>{}), ... in order.
template <class F, int... Is>
__device__ __forceinline__ void for_each_index(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}

// What the timing instantiation of the kernel records per workgroup (64-bit words): the shader clock
// counter and the constant 100 MHz counter at kernel entry, at the start and at the end of the K
// loop and after the last store was issued, then XCC_ID, HW_ID, the number of K steps, tile row,
// tile column.
constexpr int kProbeWords = 16;

// One BM x BN tile of C, tile row pm, tile column pn, by the whole workgroup.  On return every
// wave has issued its stores and LDS is no longer read.
//   staged   : the loads that open this tile's K loop (A doubles 0, 1, B steps 0..2) are already
//              under way: the previous call was given this tile as its next one;
//   has_next : another tile (npm, npn) follows in this workgroup: its opening loads are issued as
//              soon as the K loop has let go of LDS, before the accumulators are converted and
//              stored, so that their latency runs under the epilogue.
//   PROBE    : timing instantiation, see kProbeWords (probe = this workgroup's 16 words); the
//              stamps live in scalar registers until the tile is done, so the instruction stream
//              of the loop and every counter wait in it are those of the product kernel.
template <class S, bool PROBE = false>
__device__ __forceinline__ void gemm_tile(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                          uint16_t* __restrict__ C, int M, int N, int K, int pm, int pn,
                                          bool staged, bool has_next, int npm, int npn, unsigned char* smem,
                                          uint64_t* probe = nullptr) {
  constexpr int BM = S::BM, BN = S::BN, TM = S::TM, TN = S::TN;
  const int m0 = pm * BM;
  const int n0 = pn * BN;
  uint64_t stamp[8];
  auto take_stamp = [&](int i) __attribute__((always_inline)) {
    if constexpr (PROBE) {
      stamp[2 * i] = __builtin_readcyclecounter();
      stamp[2 * i + 1] = __builtin_amdgcn_s_memrealtime();
    }
  };
  take_stamp(0);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / S::WN;
  const int wn = wave % S::WN;

  // ---- global -> LDS staging: which chunk this lane fetches for each of its loads ----
  // A load i (0 .. A_LOADS-1) of wave w fills LDS bytes [(w*A_LOADS + i)*1024, +1024) of an A slot:
  // 8 rows x 128 bytes.  B load i fills [(w*B_LOADS + i)*1024, +1024) of a B slot: 2 rows x 512 bytes.
  // A lane's source is  tile base (uniform, advances with k) + a 32-bit byte offset that never changes
  // while a tile is being computed.
  uint32_t a_off[S::A_LOADS], b_off[S::B_LOADS];
  const unsigned char *a_tile, *b_tile;
  auto aim_at = [&](int tm0, int tn0) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < S::A_LOADS; ++i) {
      const int q = (wave * S::A_LOADS + i) * 64 + lane;
      const int row = q >> 3, slot = q & 7;
      const int c = a_slot(row, slot);           // XOR with a key is its own inverse
      const int r = (tm0 + row < M) ? row : (M - 1 - tm0);
      a_off[i] = (uint32_t)r * (uint32_t)K * 2u + (uint32_t)c * 16u;
    }
#pragma unroll
    for (int i = 0; i < S::B_LOADS; ++i) {
      const int q = (wave * S::B_LOADS + i) * 64 + lane;
      const int krow = q / S::B_ROW_CHUNKS, slot = q % S::B_ROW_CHUNKS;
      const int c = slot ^ b_key(krow);
      const int col = (tn0 + c * 8 < N) ? c * 8 : (N - 8 - tn0);
      b_off[i] = (uint32_t)krow * (uint32_t)N * 2u + (uint32_t)col * 2u;
    }
    a_tile = reinterpret_cast<const unsigned char*>(A + (size_t)tm0 * K);
    b_tile = reinterpret_cast<const unsigned char*>(B + tn0);
  };
  aim_at(m0, n0);
  const size_t a_dbl = (size_t)2 * kStepK * 2;        // bytes per A double along a row of A
  const size_t b_step = (size_t)kStepK * N * 2;       // bytes per K step down the rows of B
  const unsigned char* zero = reinterpret_cast<const unsigned char*>(&kZeroChunk);
  const uint32_t smem_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;   // LDS byte address of the rings

  // Load i of A double d into its ring slot.  full = the double lies wholly inside K (uniform).
  auto load_a = [&](int d, int slot, int i, auto full) __attribute__((always_inline)) {
    const unsigned char* base = a_tile + d * a_dbl;
    const uint32_t dst = smem_addr + slot * S::A_SLOT_BYTES + (wave * S::A_LOADS + i) * 1024;
    if constexpr (decltype(full)::value) {
      load_to_lds_base_off(base, a_off[i], dst);
    } else {
      const int q = (wave * S::A_LOADS + i) * 64 + lane;          // which chunk this is: only this (tail) path needs it
      const int ak = a_slot(q >> 3, q & 7) * 8;
      load_to_lds(d * 2 * kStepK + ak < K ? base + a_off[i] : zero, dst);
    }
  };
  // Load i of B step t into its ring slot.
  auto load_b = [&](int t, int slot, int i, auto full) __attribute__((always_inline)) {
    const unsigned char* base = b_tile + t * b_step;
    const uint32_t dst = smem_addr + S::A_RING_BYTES + slot * S::B_SLOT_BYTES + (wave * S::B_LOADS + i) * 1024;
    if constexpr (decltype(full)::value) {
      load_to_lds_base_off(base, b_off[i], dst);
    } else {
      const int bk = ((wave * S::B_LOADS + i) * 64 + lane) / S::B_ROW_CHUNKS;
      load_to_lds(t * kStepK + bk < K ? base + b_off[i] : zero, dst);
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
  const int a_kc0 = lane >> 4;                              // 16-byte chunk index along k (+4 for odd steps)
  const int b_krow0 = 8 * (lane >> 4) + ((lane & 15) >> 2); // (+4 for the upper half)
  const int b_col0 = wn * (TN * 16) + 4 * (lane & 3);       // + 16*bj

  // Fragment registers: one set per wave (a wave reads the fragments of a step, then issues that
  // step's MFMAs; nothing of the next step is touched in between).  A B fragment is two 8-byte halves.
  bf16x8 af[TM];
  s16x4 bq[TN][2];
  constexpr int NM = TM * TN;             // MFMAs per step
  // LDS byte addresses of this lane's part of the fragments, ring slot 0: computed once and
  // hidden from the optimiser, so that every read is "one of these registers + a constant" and
  // the constant (slot, row block, k half) goes into the instruction's 16-bit offset field.
  // A slots further than that field reaches get a second base, kAFar bytes up.
  typedef __attribute__((address_space(3))) const bf16x8* lds_a_ptr;
  typedef __attribute__((address_space(3))) s16x4* lds_b_ptr;
  constexpr uint32_t kAFar = 65536;
  auto opaque = [](uint32_t x) __attribute__((always_inline)) {
    asm volatile("" : "+v"(x));
    return x;
  };
  uint32_t a_rd[2][2], b_rd[TN];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    a_rd[h][0] = opaque(smem_addr + (uint32_t)a_lds_off(a_row0, a_kc0 + 4 * h));
    a_rd[h][1] = opaque(a_rd[h][0] + kAFar);
  }
#pragma unroll
  for (int bj = 0; bj < TN; ++bj) {
    const int col = b_col0 + 16 * bj;
    b_rd[bj] = opaque(smem_addr + (uint32_t)(S::A_RING_BYTES + b_lds_off<BN>(b_krow0, col >> 3) + (col & 7) * 2));
  }
  // A fragment bi of K step t (t = 2*double + half): row block bi is 16 rows = 2048 bytes further
  // (the swizzle key repeats every 16 rows).
  auto read_a = [&](int a_slot_idx, int half, int bi) __attribute__((always_inline)) {
    const uint32_t off = (uint32_t)a_slot_idx * S::A_SLOT_BYTES + (uint32_t)bi * 2048u;
    const bool far = __builtin_constant_p(off) && off >= kAFar;
    af[bi] = far ? *(lds_a_ptr)(uintptr_t)(a_rd[half][1] + (off - kAFar)) : *(lds_a_ptr)(uintptr_t)(a_rd[half][0] + off);
  };
  // B fragment bj, half hi: rows 4 further down = 4*BN*2 bytes (the key depends on k mod 4 and on
  // bit 3 of k only, and the lane's first row has k mod 8 < 4).
  auto read_b = [&](int b_slot_idx, int bj, int hi) __attribute__((always_inline)) {
    const uint32_t off = (uint32_t)b_slot_idx * S::B_SLOT_BYTES + (uint32_t)hi * (4u * BN * 2u);
    bq[bj][hi] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_b_ptr)(uintptr_t)(b_rd[bj] + off));
  };
  auto mfma = [&](int bi, int bj) __attribute__((always_inline)) {
    const bf16x8 b = __builtin_bit_cast(bf16x8, __builtin_shufflevector(bq[bj][0], bq[bj][1], 0, 1, 2, 3, 4, 5, 6, 7));
    acc[bi][bj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, af[bi], acc[bi][bj], 0, 0, 0);
  };

  // The eight waves form two groups of four (group = wave / 4; the two waves that share a SIMD
  // are in different groups).  Time is cut into phases; in every phase one group issues the 32
  // MFMAs of a K step back to back while the other group does the memory work of its next step
  // (fragment reads from LDS, its share of global->LDS loads), then the groups swap.  A barrier
  // separates the phases, so on each SIMD the MFMA pipe sees one uninterrupted stream and the
  // memory instructions of the other wave never queue behind an MFMA.
  //   group 0:  MEM(0) | CMP(0) | MEM(1) | CMP(1) | ...
  //   group 1:    -    | MEM(0) | CMP(0) | MEM(1) | ...
  // MEM(u) reads the fragments of step u (A double u/2, half u&1; B slot u%4) and issues half the
  // loads of A double u/2 + 2 and the loads of B step u + 3.
  //   * data: step u's data was issued by MEM(u-3) at the latest; every wave ends MEM(v) by waiting
  //     until only the loads of MEM(v) and MEM(v-1) are outstanding, so before the barrier that
  //     precedes group 0's MEM(u) everybody has waited for MEM(u-3)'s loads (group 0 at the end of
  //     MEM(u-1), group 1 at the end of MEM(u-1) too, one phase later but before the same barrier).
  //   * slots: MEM(u) refills B slot (u-1)%4 and, for even u, starts on the A slot of double
  //     u/2 - 1; their last readers were group 1's MEM(u-1), which ended with an LDS-counter wait
  //     before the barrier that precedes group 0's MEM(u).
  static_assert(S::NW == 8, "two groups of four waves");
  const int grp = wave >> 2;
  // rd_as / rd_bs: ring slots MEM(u) reads; ld_as / ld_bs: ring slots its loads fill
  auto mem_phase = [&](auto half_tag, int u, int rd_as, int rd_bs, int ld_as, int ld_bs, auto full) __attribute__((always_inline)) {
    constexpr int HALF = decltype(half_tag)::value;
    const int d = u >> 1;
#pragma unroll
    for (int i = 0; i < S::A_LOADS / 2; ++i) load_a(d + 2, ld_as, HALF * (S::A_LOADS / 2) + i, full);
#pragma unroll
    for (int i = 0; i < S::B_LOADS; ++i) load_b(u + 3, ld_bs, i, full);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int bj = 0; bj < TN; ++bj) {
      read_b(rd_bs, bj, 0);
      read_b(rd_bs, bj, 1);
    }
#pragma unroll
    for (int bi = 0; bi < TM; ++bi) read_a(rd_as, HALF, bi);
    wait_vmcnt_lgkmcnt<2 * S::LOADS, 0>();
    __builtin_amdgcn_sched_barrier(0);
  };
  // Row block by row block, the column blocks alternately left to right and right to left: from
  // one MFMA to the next exactly one of the two fragment operands changes (measured +1.3 to
  // +1.6 % against an order in which both change at the end of a row block: the chip is power
  // bound, and an operand that stays costs less).
  auto compute_phase = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NM; ++i) mfma(i / TN, ((i / TN) & 1) ? TN - 1 - i % TN : i % TN);
    __builtin_amdgcn_sched_barrier(0);
    block_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  auto phase_barrier = [&]() __attribute__((always_inline)) {
    block_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };

  const int KT = (K + kStepK - 1) / kStepK;
  // the loads that open a tile: A doubles 0 and 1, B steps 0 .. 2 (what MEM(0) and MEM(1) do not fetch themselves)
  static_assert(kBSlots == 4 && kASlots == 3, "the opening order is written for these ring depths");
  auto open_tile = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < S::A_LOADS; ++i) load_a(0, 0, i, kTail);
#pragma unroll
    for (int i = 0; i < S::B_LOADS; ++i) load_b(0, 0, i, kTail);
#pragma unroll
    for (int i = 0; i < S::B_LOADS; ++i) load_b(1, 1, i, kTail);
#pragma unroll
    for (int i = 0; i < S::A_LOADS; ++i) load_a(1, 1, i, kTail);
#pragma unroll
    for (int i = 0; i < S::B_LOADS; ++i) load_b(2, 2, i, kTail);
  };
  if (!staged) {
    open_tile();
    wait_vmcnt<S::A_LOADS + (kBSlots - 2) * S::B_LOADS>();        // A double 0 and B step 0 have landed (this wave's part)
  } else {
    // issued during the previous tile's epilogue, whose stores share the counter and may complete out of
    // order with loads: wait for everything
    wait_vmcnt<0>();
  }
  __syncthreads();                                               // ... and everybody else's
  take_stamp(1);
  if (grp == 1) phase_barrier();                                 // group 1 starts one phase later

  // one step whose position in the slot cycle (B: 4 steps, A: 3 doubles = 6 steps, together 12)
  // is a compile-time constant, so that every LDS address in it is a register plus an immediate
  auto step_at = [&](auto pos_tag, int u, auto full) __attribute__((always_inline)) {
    constexpr int P = decltype(pos_tag)::value;
    mem_phase(std::integral_constant<int, P & 1>{}, u, (P / 2) % kASlots, P % kBSlots, (P / 2 + 2) % kASlots,
              (P + 3) % kBSlots, full);
    phase_barrier();
    compute_phase();
  };
  auto step_pair = [&](int t, auto full) __attribute__((always_inline)) {   // t even; slots from t at run time
    const int d = t >> 1;
    mem_phase(std::integral_constant<int, 0>{}, t, d % kASlots, t % kBSlots, (d + 2) % kASlots, (t + 3) % kBSlots, full);
    phase_barrier();
    compute_phase();
    mem_phase(std::integral_constant<int, 1>{}, t + 1, d % kASlots, (t + 1) % kBSlots, (d + 2) % kASlots, (t + 4) % kBSlots, full);
    phase_barrier();
    compute_phase();
  };
  // steps 0 .. full_steps-1 lie wholly inside K; a step is fetched unpredicated if everything the
  // block it belongs to fetches lies inside K (step u fetches A double u/2+2 and B step u+3)
  const int full_steps = K / kStepK;
  constexpr int CYCLE = 2 * kASlots * kBSlots / 2;               // lcm(2*kASlots, kBSlots) = 12 for rings of 3 and 4
  static_assert(CYCLE % (2 * kASlots) == 0 && CYCLE % kBSlots == 0, "slot cycle");
  int t = 0;
  for (; t + CYCLE + 4 <= full_steps; t += CYCLE)
    for_each_index([&](auto pos) __attribute__((always_inline)) { step_at(pos, t + decltype(pos)::value, kFull); },
                   std::make_integer_sequence<int, CYCLE>{});
  for (; t + 6 <= full_steps; t += 2) step_pair(t, kFull);
  for (; t < KT; t += 2) step_pair(t, kTail);
  if (grp == 0) phase_barrier();                                 // group 1's last compute phase

  // ---- epilogue: fp32 -> bf16 (nearest even), rearranged across lanes in registers, 16-byte stores ----
  wait_vmcnt<0>();   // the zero-filled look-ahead steps have landed too
  __syncthreads();   // nobody reads the rings any more, and nothing is on its way into them
  take_stamp(2);
  if (has_next) {    // uniform: open the next tile now, its loads run under the conversion and the stores
    aim_at(npm * BM, npn * BN);
    open_tile();
  }
  // Lane (r = lane % 16, g = lane / 16) holds, for every block (bi, bj), C[16 bi + r][16 bj + 4 g + 0..3]:
  // 8 bytes once converted.  v_permlane16_swap exchanges the odd 16-lane rows of one register with the
  // even rows of another; applied to the registers of blocks bj = 2p and 2p + 1 it leaves every lane with
  // 16 contiguous bytes: lanes g = 0, 2 hold columns 0..7, 8..15 of block 2p, lanes g = 1, 3 those of block
  // 2p + 1, so the four lanes of a row cover 64 contiguous bytes.
  const int er = lane & 15, eg = lane >> 4;
  const int ecol = n0 + wn * (TN * 16) + ((eg & 1) ? 16 + 4 * (eg - 1) : 4 * eg);     // + 32 p
  static_assert(TN == 2 || TN == 4, "the register epilogue pairs up column blocks");
#pragma unroll
  for (int bi = 0; bi < TM; ++bi) {
    u32x4 chunk[TN / 2];
#pragma unroll
    for (int p = 0; p < TN / 2; ++p) {
      uint32_t d[2][2];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        bf16x4 c4;
#pragma unroll
        for (int e = 0; e < 4; ++e) c4[e] = (__bf16)acc[bi][2 * p + h][e];
        const auto two = __builtin_bit_cast(__attribute__((ext_vector_type(2))) uint32_t, c4);
        d[h][0] = two[0];
        d[h][1] = two[1];
      }
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const auto sw = __builtin_amdgcn_permlane16_swap(d[0][w], d[1][w], false, false);
        d[0][w] = sw[0];
        d[1][w] = sw[1];
      }
      chunk[p] = u32x4{d[0][0], d[0][1], d[1][0], d[1][1]};
    }
    const int row0 = m0 + wm * (TM * 16) + 16 * bi;
    if constexpr (TN == 4) {
      // Whole 128-byte lines per store instruction: lanes r and r + 8 trade one chunk (a rotation by 8 inside
      // the 16-lane row), after which the first instruction writes rows 0..7 of the block (lanes r < 8 the
      // left 64 bytes, lanes r >= 8 the right 64 bytes) and the second one rows 8..15.
      const bool low = er < 8;
      u32x4 give, got, s0, s1;
#pragma unroll
      for (int e = 0; e < 4; ++e) give[e] = low ? chunk[1][e] : chunk[0][e];
#pragma unroll
      for (int e = 0; e < 4; ++e) got[e] = __builtin_amdgcn_mov_dpp(give[e], 0x128 /* row_ror:8 */, 0xf, 0xf, false);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s0[e] = low ? chunk[0][e] : got[e];
        s1[e] = low ? got[e] : chunk[1][e];
      }
      const int col = ecol + (low ? 0 : 32);
      const int row = row0 + (er & 7);
      // C is written once and not read again by this kernel: streaming (non-temporal) stores
      if (row < M && col < N) __builtin_nontemporal_store(s0, reinterpret_cast<u32x4*>(C + (size_t)row * N + col));
      if (row + 8 < M && col < N) __builtin_nontemporal_store(s1, reinterpret_cast<u32x4*>(C + (size_t)(row + 8) * N + col));
    } else {
      const int row = row0 + er;
      if (row < M && ecol < N) __builtin_nontemporal_store(chunk[0], reinterpret_cast<u32x4*>(C + (size_t)row * N + ecol));
    }
  }
  take_stamp(3);
  if constexpr (PROBE) {
    if (tid == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) probe[i] = stamp[i];
      probe[8] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));      // XCC_ID
      probe[9] = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));      // HW_ID
      probe[10] = (uint64_t)KT;
      probe[11] = (uint64_t)pm;
      probe[12] = (uint64_t)pn;
      probe[13] = probe[14] = probe[15] = 0;
    }
  }
}

// One workgroup per tile.  MODE (one of the four renumbering / raster combinations) is a template
// parameter so that each mapping shows up under its own kernel name in profiler traces; the skew
// comes as an argument; only the decode depends on either.
template <class S, int MODE>
__global__ __launch_bounds__(S::NT) void gemm_bf16_kernel(const uint16_t* __restrict__ A,
                                                          const uint16_t* __restrict__ B,
                                                          uint16_t* __restrict__ C, int M, int N, int K,
                                                          int grid_m, int grid_n, int num_xcd, int group_m, int skew) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  int pm, pn;
  swz_decode_tile((int)blockIdx.x, grid_m, grid_n, num_xcd, group_m, MODE | (skew ? kModeSkew : 0), &pm, &pn);
  gemm_tile<S>(A, B, C, M, N, K, pm, pn, false, false, 0, 0, smem);
}

// The same kernel with time stamps (measurement aid): workgroup w also writes kProbeWords 64-bit words
// at probe + w*kProbeWords.
template <class S, int MODE>
__global__ __launch_bounds__(S::NT) void gemm_bf16_probe_kernel(const uint16_t* __restrict__ A,
                                                                const uint16_t* __restrict__ B,
                                                                uint16_t* __restrict__ C, int M, int N, int K,
                                                                int grid_m, int grid_n, int num_xcd, int group_m,
                                                                int skew, uint64_t* __restrict__ probe) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  int pm, pn;
  swz_decode_tile((int)blockIdx.x, grid_m, grid_n, num_xcd, group_m, MODE | (skew ? kModeSkew : 0), &pm, &pn);
  gemm_tile<S, true>(A, B, C, M, N, K, pm, pn, false, false, 0, 0, smem, probe + (size_t)blockIdx.x * kProbeWords);
}

// Persistent grid: gridDim.x workgroups (one per compute unit) stay resident; workgroup w is
// renumbered among the workgroups and walks the raster with stride gridDim.x, the launch style
// of the paper's GEMM case study (Appendix "Case Study: GEMM Swizzling", num_blocks = number of
// compute units).  A workgroup knows its next tile while it computes the current one, so the next
// tile's opening loads are in flight while the current tile is converted and stored.
template <class S, int MODE>
__global__ __launch_bounds__(S::NT) void gemm_bf16_persistent_kernel(const uint16_t* __restrict__ A,
                                                                     const uint16_t* __restrict__ B,
                                                                     uint16_t* __restrict__ C, int M, int N, int K,
                                                                     int grid_m, int grid_n, int num_xcd, int group_m,
                                                                     int skew) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int total = grid_m * grid_n;
  const int mode = MODE | (skew ? kModeSkew : 0);
  int l = swz_persistent_logical((int)blockIdx.x, 0, (int)gridDim.x, total, num_xcd, MODE);
  if (l < 0) return;                       // uniform: the whole workgroup leaves together
  int pm, pn;
  swz_tile_at(l, grid_m, grid_n, group_m, mode, &pm, &pn);
  bool staged = false;
  for (int round = 1;; ++round) {
    const int ln = swz_persistent_logical((int)blockIdx.x, round, (int)gridDim.x, total, num_xcd, MODE);
    int npm = 0, npn = 0;
    if (ln >= 0) swz_tile_at(ln, grid_m, grid_n, group_m, mode, &npm, &npn);
    gemm_tile<S>(A, B, C, M, N, K, pm, pn, staged, ln >= 0, npm, npn, smem);
    if (ln < 0) break;
    pm = npm;
    pn = npn;
    staged = true;
  }
}

}  // namespace swz
