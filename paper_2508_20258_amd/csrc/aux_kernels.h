// Small kernels beside the GEMM: the decode-only kernels that record what the device PID remap
// computes (and the XCD every workgroup really ran on), and the plain copy of known traffic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pid_decode.h"

namespace swz {

typedef __attribute__((ext_vector_type(4))) uint32_t aux_u32x4;

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
      swz_tile_at(l, grid_m, grid_n, group_m, mode, &pm, &pn);
      t = pm * grid_n + pn;
    }
    tile[(size_t)round * g + w] = t;
  }
  if (xcc != nullptr) xcc[w] = (int32_t)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));
}

// Plain streaming copy of n 16-byte words (reads n*16 bytes, writes n*16 bytes): a kernel of
// known HBM traffic against which profiler byte counters are scaled, and the rate of which the
// bandwidth-bound kernels are compared with.  Four loads are in flight per thread before the first
// store; a workgroup moves 16 KiB of consecutive addresses per round.
__global__ __launch_bounds__(256) void copy16_kernel(const aux_u32x4* __restrict__ src, aux_u32x4* __restrict__ dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * 1024;
  for (int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x; base < n; base += stride) {
    aux_u32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (base + 256 * j < n) v[j] = __builtin_nontemporal_load(src + base + 256 * j);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (base + 256 * j < n) __builtin_nontemporal_store(v[j], dst + base + 256 * j);
  }
}

}  // namespace swz
