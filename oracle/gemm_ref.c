/* Reference GEMM for the tests (test infrastructure only; not part of the library).
 *
 * C = A . B as the paper's GEMM case study states it: A is M x K, B is K x N, C is M x N
 * (SwizzlePerf, Appendix "Case Study: GEMM Swizzling").  Inputs are bfloat16 bit patterns,
 * row-major and dense; each is widened exactly to double and the sum over k is accumulated
 * in double, k ascending.  No tiling, no reordering of the sum, no BLAS.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC oracle/gemm_ref.c -o oracle/libgemm_ref.so
 */
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen_bf16(uint16_t h) {
  uint32_t u = (uint32_t)h << 16; /* bf16 is the upper half of an IEEE binary32 */
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* Threads the full-matrix routine will use (1 when built without OpenMP). */
int ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Full product.  threads <= 0 keeps the OpenMP default; threads == 1 is the serial loop. */
void ref_gemm_bf16_f64(const uint16_t* A, const uint16_t* B, double* C, int64_t M, int64_t N, int64_t K,
                       int threads) {
#ifdef _OPENMP
  if (threads > 0) omp_set_num_threads(threads);
#else
  (void)threads;
#endif
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i) {
    double* c = C + i * N;
    for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
    for (int64_t k = 0; k < K; ++k) {       /* for every j the sum still runs k = 0,1,2,... */
      const double a = widen_bf16(A[i * K + k]);
      const uint16_t* b = B + k * N;
      for (int64_t j = 0; j < N; ++j) c[j] += a * widen_bf16(b[j]);
    }
  }
}

/* Selected elements: out[e] = sum_k A[ii[e]][k] * B[k][jj[e]]. */
void ref_gemm_bf16_f64_elems(const uint16_t* A, const uint16_t* B, int64_t M, int64_t N, int64_t K,
                             const int64_t* ii, const int64_t* jj, int64_t n, double* out) {
  (void)M;
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < n; ++e) {
    const uint16_t* a = A + ii[e] * K;
    const uint16_t* b = B + jj[e];
    double s = 0.0;
    for (int64_t k = 0; k < K; ++k) s += widen_bf16(a[k]) * widen_bf16(b[k * N]);
    out[e] = s;
  }
}
