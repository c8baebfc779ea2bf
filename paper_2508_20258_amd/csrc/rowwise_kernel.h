// Row softmax and layer normalisation over bf16 rows with a remapped program id (SwizzlePerf,
// Results and Appendix "Case Study: Other Swizzling Pattern Examples": the swizzle found for
// both kernels puts all column chunks of one row on one XCD).
//
// Decomposition (the one the paper's remap is about): a row of N elements is cut into `chunks`
// column chunks and one workgroup produces one chunk.  A chunk needs the statistics of its whole
// row (maximum and sum of exponentials; mean and variance), so every workgroup reads the whole
// row and then re-reads and writes its own chunk; nothing is exchanged between workgroups.  The
// redundant row reads are what the mapping acts on: the grid is M x chunks, hardware id w is
// decoded exactly like a GEMM tile id (row = logical id div chunks), and under the XCD
// renumbering the workgroups of one row run back to back on one XCD and find the row in its L2.
// With chunks = 1 a workgroup owns a whole row and the mapping is irrelevant; that is the form
// to use whenever M alone fills the chip.  In that form a row of up to 256*8*KEEP elements
// (KEEP <= 16 vectors per thread) stays in registers between the two phases, so HBM is read once;
// and rows of at most 2048 elements are handled one per wave, four rows per workgroup, with no
// LDS and no barrier (the grid is then ceil(M/4) x 1 groups of four consecutive rows).
//
// All arithmetic is fp32 on values widened exactly from bf16; results are rounded once to bf16
// (nearest even).  The statistics are computed over the same thread partition of the row in
// every workgroup of a launch, so the output bits never depend on the mode, and with 256 threads
// per row (N > 2048, or chunks > 1) not on `chunks` either.
#pragma once

#include <float.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pid_decode.h"

namespace swz {

typedef __attribute__((ext_vector_type(4))) uint32_t rw_u32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 rw_bf16x2;

constexpr int kRowThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ void rw_unpack(const rw_u32x4& v, float (&x)[8]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    x[2 * e] = __uint_as_float(v[e] << 16);
    x[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u);
  }
}

__device__ __forceinline__ rw_u32x4 rw_pack(const float (&y)[8]) {
  rw_u32x4 v;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    rw_bf16x2 h;
    h[0] = (__bf16)y[2 * e];
    h[1] = (__bf16)y[2 * e + 1];
    v[e] = __builtin_bit_cast(uint32_t, h);
  }
  return v;
}

__device__ __forceinline__ float rw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// (m, s): running maximum (in the log2 domain) and sum of 2^(t - m).  Identity: (-FLT_MAX, 0).
__device__ __forceinline__ void soft_merge(float& m, float& s, float m2, float s2) {
  const float mn = fmaxf(m, m2);
  s = s * rw_exp2(m - mn) + s2 * rw_exp2(m2 - mn);
  m = mn;
}

__device__ __forceinline__ void soft_update(float& m, float& s, const rw_u32x4& v) {
  float t[8];
  rw_unpack(v, t);
#pragma unroll
  for (int e = 0; e < 8; ++e) t[e] *= kLog2e;
  const float vmax = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])), fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
  if (vmax > m) {                                          // rare once the running maximum has settled
    s *= rw_exp2(m - vmax);
    m = vmax;
  }
  float add = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) add += rw_exp2(t[e] - m);
  s += add;
}

// (n, mean, m2): count, mean and sum of squared deviations; merged with the pairwise update of
// Chan, Golub and LeVeque, which is stable whatever the mean.  Identity: (0, 0, 0).
__device__ __forceinline__ void moments_merge(float& n, float& mean, float& m2, float n2, float mean2, float m22) {
  const float nn = n + n2;
  const float inv = nn > 0.f ? 1.0f / nn : 0.f;
  const float d = mean2 - mean;
  mean += d * (n2 * inv);
  m2 += m22 + d * d * (n * n2 * inv);
  n = nn;
}

__device__ __forceinline__ void moments_update(float& n, float& mean, float& m2, const rw_u32x4& v) {
  float x[8];
  rw_unpack(v, x);
  const float vmean = (((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]))) * 0.125f;
  float vm2 = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) vm2 += (x[e] - vmean) * (x[e] - vmean);
  moments_merge(n, mean, m2, 8.f, vmean, vm2);
}

// Applies `update` to every 16-byte vector of the row, vectors dealt to threads round-robin,
// four loads in flight per thread.
template <typename F>
__device__ __forceinline__ void for_each_row_vector(const rw_u32x4* __restrict__ rowp, int nv, int tid, F update) {
  int v = tid;
  for (; v + 3 * kRowThreads < nv; v += 4 * kRowThreads) {
    const rw_u32x4 a = rowp[v], b = rowp[v + kRowThreads], c = rowp[v + 2 * kRowThreads], d = rowp[v + 3 * kRowThreads];
    update(a);
    update(b);
    update(c);
    update(d);
  }
  for (; v < nv; v += kRowThreads) update(rowp[v]);
}

// Where a workgroup finds its work.  TPR = threads per row: 256 (one row or row chunk per
// workgroup) or 64 (one row per wave, chunks == 1).  KEEP > 0 (chunks == 1 only): the row is held
// in KEEP vector registers per thread, N <= TPR*8*KEEP.
template <int MODE, int TPR>
struct RowJob {
  int row, nv, v0, v1, tid;
  bool live;
  __device__ __forceinline__ RowJob(int M, int N, int chunks, int chunk_vecs, int num_xcd, int group_m) {
    constexpr int ROWS = kRowThreads / TPR;
    int group, chunk;
    swz_decode_tile((int)blockIdx.x, (M + ROWS - 1) / ROWS, chunks, num_xcd, group_m, MODE, &group, &chunk);
    row = group * ROWS + (int)threadIdx.x / TPR;
    tid = (int)threadIdx.x % TPR;
    nv = N >> 3;
    v0 = chunk * chunk_vecs;
    v1 = v0 + chunk_vecs < nv ? v0 + chunk_vecs : nv;
    live = row < M && v0 < nv;                             // uniform per workgroup when TPR == 256, per wave when TPR == 64
  }
};

template <int MODE, int KEEP, int TPR>
__global__ __launch_bounds__(kRowThreads) void softmax_rows_kernel(const uint16_t* __restrict__ in,
                                                                   uint16_t* __restrict__ out, int M, int N, int chunks,
                                                                   int chunk_vecs, int num_xcd, int group_m) {
  static_assert(TPR == kRowThreads || (TPR == 64 && KEEP > 0), "a wave-sized row group keeps its row in registers");
  const RowJob<MODE, TPR> job(M, N, chunks, chunk_vecs, num_xcd, group_m);
  if (!job.live) return;                                   // an empty trailing chunk or row: nothing to produce
  const int nv = job.nv, tid = job.tid;
  const rw_u32x4* rowp = reinterpret_cast<const rw_u32x4*>(in + (size_t)job.row * N);

  float m = -FLT_MAX, s = 0.f;
  rw_u32x4 held[KEEP > 0 ? KEEP : 1];
  if constexpr (KEEP > 0) {
#pragma unroll
    for (int i = 0; i < KEEP; ++i)
      if (tid + i * TPR < nv) held[i] = rowp[tid + i * TPR];
#pragma unroll
    for (int i = 0; i < KEEP; ++i)                          // same vectors, same order as the streaming form
      if (tid + i * TPR < nv) soft_update(m, s, held[i]);
  } else {
    for_each_row_vector(rowp, nv, tid, [&](const rw_u32x4& v) __attribute__((always_inline)) { soft_update(m, s, v); });
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) soft_merge(m, s, __shfl_xor(m, off, 64), __shfl_xor(s, off, 64));
  if constexpr (TPR == kRowThreads) {
    __shared__ float red[2 * (kRowThreads / 64)];
    if ((tid & 63) == 0) {
      red[2 * (tid >> 6)] = m;
      red[2 * (tid >> 6) + 1] = s;
    }
    __syncthreads();
    m = red[0];
    s = red[1];
#pragma unroll
    for (int w = 1; w < kRowThreads / 64; ++w) soft_merge(m, s, red[2 * w], red[2 * w + 1]);
  }
  const float inv = 1.0f / s;

  rw_u32x4* outp = reinterpret_cast<rw_u32x4*>(out + (size_t)job.row * N);
  auto emit = [&](const rw_u32x4& xv, int v) __attribute__((always_inline)) {
    float t[8], y[8];
    rw_unpack(xv, t);
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = rw_exp2(t[e] * kLog2e - m) * inv;
    __builtin_nontemporal_store(rw_pack(y), outp + v);
  };
  if constexpr (KEEP > 0) {
#pragma unroll
    for (int i = 0; i < KEEP; ++i)
      if (tid + i * TPR < nv) emit(held[i], tid + i * TPR);
  } else {
    for (int v = job.v0 + tid; v < job.v1; v += kRowThreads) emit(rowp[v], v);
  }
}

template <int MODE, int KEEP, int TPR>
__global__ __launch_bounds__(kRowThreads) void layernorm_rows_kernel(const uint16_t* __restrict__ in,
                                                                     const uint16_t* __restrict__ gamma,
                                                                     const uint16_t* __restrict__ beta,
                                                                     uint16_t* __restrict__ out, int M, int N, float eps,
                                                                     int chunks, int chunk_vecs, int num_xcd, int group_m) {
  static_assert(TPR == kRowThreads || (TPR == 64 && KEEP > 0), "a wave-sized row group keeps its row in registers");
  const RowJob<MODE, TPR> job(M, N, chunks, chunk_vecs, num_xcd, group_m);
  if (!job.live) return;
  const int nv = job.nv, tid = job.tid;
  const rw_u32x4* rowp = reinterpret_cast<const rw_u32x4*>(in + (size_t)job.row * N);

  float n = 0.f, mean = 0.f, m2 = 0.f;
  rw_u32x4 held[KEEP > 0 ? KEEP : 1];
  if constexpr (KEEP > 0) {
#pragma unroll
    for (int i = 0; i < KEEP; ++i)
      if (tid + i * TPR < nv) held[i] = rowp[tid + i * TPR];
#pragma unroll
    for (int i = 0; i < KEEP; ++i)
      if (tid + i * TPR < nv) moments_update(n, mean, m2, held[i]);
  } else {
    for_each_row_vector(rowp, nv, tid, [&](const rw_u32x4& v) __attribute__((always_inline)) { moments_update(n, mean, m2, v); });
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1)
    moments_merge(n, mean, m2, __shfl_xor(n, off, 64), __shfl_xor(mean, off, 64), __shfl_xor(m2, off, 64));
  if constexpr (TPR == kRowThreads) {
    __shared__ float red[3 * (kRowThreads / 64)];
    if ((tid & 63) == 0) {
      red[3 * (tid >> 6)] = n;
      red[3 * (tid >> 6) + 1] = mean;
      red[3 * (tid >> 6) + 2] = m2;
    }
    __syncthreads();
    n = red[0];
    mean = red[1];
    m2 = red[2];
#pragma unroll
    for (int w = 1; w < kRowThreads / 64; ++w) moments_merge(n, mean, m2, red[3 * w], red[3 * w + 1], red[3 * w + 2]);
  }
  const float rstd = 1.0f / sqrtf(m2 / n + eps);

  const rw_u32x4* gp = reinterpret_cast<const rw_u32x4*>(gamma);
  const rw_u32x4* bp = reinterpret_cast<const rw_u32x4*>(beta);
  rw_u32x4* outp = reinterpret_cast<rw_u32x4*>(out + (size_t)job.row * N);
  auto emit = [&](const rw_u32x4& xv, int v) __attribute__((always_inline)) {
    float x[8], g[8], b[8], y[8];
    rw_unpack(xv, x);
    rw_unpack(gp[v], g);
    rw_unpack(bp[v], b);
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = (x[e] - mean) * rstd * g[e] + b[e];
    __builtin_nontemporal_store(rw_pack(y), outp + v);
  };
  if constexpr (KEEP > 0) {
#pragma unroll
    for (int i = 0; i < KEEP; ++i)
      if (tid + i * TPR < nv) emit(held[i], tid + i * TPR);
  } else {
    for (int v = job.v0 + tid; v < job.v1; v += kRowThreads) emit(rowp[v], v);
  }
}

}  // namespace swz
