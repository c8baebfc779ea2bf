// Measurement aid: sustained matrix-core rate of the device (see swz_mfma_peak).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swz {

typedef __attribute__((ext_vector_type(8))) __bf16 pk_bf16x8;
typedef __attribute__((ext_vector_type(4))) float pk_f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t pk_u32x4;

// Measurement aid: the MFMA rate the device sustains when nothing else happens.  Every wave
// issues iters x 64 independent v_mfma_f32_16x16x32_bf16 (the GEMM's instruction, 16384 flop
// each) on operands that stay in registers: pseudo-random bf16 values of magnitude ~2^-6, or
// zeros.  Launched with one 512-thread workgroup per CU (2 waves per SIMD).  out gets one float
// per thread so that the accumulators are live.
__global__ __launch_bounds__(512) void mfma_peak_kernel(float* __restrict__ out, int iters, int random_operands) {
  const uint32_t tid = threadIdx.x + blockIdx.x * 512u;
  pk_bf16x8 a[4], b[2];
#pragma unroll
  for (int f = 0; f < 6; ++f) {
    pk_u32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t x = (tid * 16u + f) * 2654435761u + i * 40503u;
      x ^= x >> 15;
      x *= 2246822519u;
      x ^= x >> 13;
      // two bf16: random sign and mantissa, exponent 2^-6 .. 2^-9
      const uint32_t lo = (x & 0x807fu) | (0x3c80u - ((x >> 20) & 0x180u));
      const uint32_t hi = ((x >> 16) & 0x807fu) | (0x3c80u - ((x >> 24) & 0x180u));
      v[i] = random_operands ? (lo | (hi << 16)) : 0u;
    }
    if (f < 4) a[f] = __builtin_bit_cast(pk_bf16x8, v);
    else b[f - 4] = __builtin_bit_cast(pk_bf16x8, v);
  }
  pk_f32x4 acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j & 1], a[i & 3], acc[i][j], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) sum += acc[i][j][e];
  out[tid] = sum;
}

}  // namespace swz
