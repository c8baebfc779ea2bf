/* libswz — XCD-aware swizzled bf16 GEMM for AMD Instinct MI355X (gfx950).
 *
 * C ABI.  No exception crosses it; every function that can fail returns a swz_status
 * (0 = success, negative = error) and, on error, leaves its output buffers untouched.
 *
 * Background (SwizzlePerf, Introduction and Appendix "Case Study: GEMM Swizzling"): on a
 * chiplet GPU the workgroups of a launch are handed to the XCDs round-robin, workgroup w to
 * XCD (w mod X), and every XCD has a private L2.  Output tiles in one row of C read the same
 * rows of A and tiles in one column read the same columns of B, so a kernel gains L2 reuse
 * when it recomputes its program id such that the tiles an XCD works on are neighbours.
 * "Hardware workgroup id" below is w (blockIdx.x of a 1-D launch); the "tile" is the
 * (pm, pn) block of C that workgroup computes.
 */
#ifndef SWZ_H
#define SWZ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Same declaration the HIP runtime headers make; repeating it keeps this header free of
 * any HIP include.  Python callers pass the stream handle as a pointer-sized integer. */
typedef struct ihipStream_t* hipStream_t;

typedef enum {
  SWZ_OK = 0,
  SWZ_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, unknown mode                */
  SWZ_ERR_UNSUPPORTED = -2, /* valid request the library cannot serve (dtype, alignment, tile) */
  SWZ_ERR_OVERFLOW = -3,    /* a count does not fit the 32-bit index arithmetic              */
  SWZ_ERR_HIP = -4          /* the HIP runtime reported an error (launch, attribute query)   */
} swz_status;

/* How hardware workgroup ids are turned into tiles. */
typedef enum {
  SWZ_MODE_RR = 0,         /* no renumbering, row-major raster: what round-robin dispatch gives by default */
  SWZ_MODE_XCD = 1,        /* XCD renumbering (each XCD owns one contiguous run of the raster), row-major   */
  SWZ_MODE_XCD_GROUPM = 2, /* XCD renumbering, grouped-M raster                                            */
  SWZ_MODE_GROUPM = 3,     /* no renumbering, grouped-M raster                                             */
  SWZ_MODE_SKEW = 4        /* flag, may be added to any of the four: skewed raster, modes 4..7 (see swz_pid_map) */
} swz_mode;

typedef enum { SWZ_DTYPE_BF16 = 0 } swz_dtype; /* A, B, C bfloat16; accumulation in fp32 */

/* Optional knobs for swz_gemm_ex / swz_gemm_plan.  A field equal to 0 means "library default". */
typedef struct {
  int32_t bm;      /* tile rows:    128 or 256 */
  int32_t bn;      /* tile columns: 128 or 256 (all four combinations; one of bm, bn given: the other takes its value) */
  int32_t bk;      /* K panel per tile step: 64 (the kernel streams it as two 32-wide halves) */
  int32_t group_m; /* tile rows per band of the grouped raster (default 4) */
  int32_t num_xcd; /* XCD count assumed by the renumbering (default: detected; 8 on an unpartitioned MI355X) */
  int32_t persistent; /* 0: one workgroup per tile (default); 1: persistent grid, see swz_pid_map_persistent */
  int32_t num_wg;  /* persistent grid size (default: one workgroup per compute unit, at most one per tile) */
} swz_params;

/* Human-readable name of a swz_status (the pass/fail reporting of the paper's validation step,
 * Methodology step 3, needs one).  Returns a static string, never null; unknown codes included. */
const char* swz_status_string(int status);

/* Facts about the current device that the remap depends on (the paper's "hardware context" of
 * Methodology step 2: XCD count, CUs, L2 size, taken from HIP device attributes).  Any pointer may
 * be null.
 *   num_xcd       : CU count / 32 (gfx950: 32 CUs per XCD; a partitioned device exposes fewer
 *                   XCDs), or the value of the environment variable SWZ_NUM_XCD (an integer in
 *                   1..1024, read once per process) when it is set; 0 if the CU count is not a
 *                   whole number of XCDs and no override is given.  Entry points that default
 *                   num_xcd then return SWZ_ERR_UNSUPPORTED until the caller names it.
 *   compute_units : hipDeviceAttributeMultiprocessorCount.
 *   l2_bytes      : hipDeviceAttributeL2CacheSize as the runtime reports it, unchanged (on an
 *                   MI355X that is 4 MiB, the private L2 of ONE XCD, not the sum over XCDs).
 *   lds_bytes     : hipDeviceAttributeMaxSharedMemoryPerBlock (LDS one workgroup may use). */
int swz_device_info(int* num_xcd, int* compute_units, int* l2_bytes, int* lds_bytes);

/* The PID map, computed on the host (GEMM swizzle of the paper's appendix, extended so that
 * it is a bijection for every launch size, including sizes that are not a multiple of
 * num_xcd, plus the grouped-M raster).
 *   out : caller-owned HOST buffer of grid_m*grid_n int32; out[w] = pm*grid_n + pn.
 *   mode 0/1 ignore group_m, mode 0/3 ignore num_xcd, but both must still be >= 1.
 *   Renumbering: XCD x = w mod num_xcd receives n_x = q + [x < r] workgroups (q = T div X,
 *   r = T mod X); its i-th workgroup (i = w div X) gets logical id  x*q + min(x,r) + i.
 *   Grouped raster of logical id l: bands of group_m tile rows (last band shorter), inside a
 *   band column by column, inside a column top to bottom.
 *   Skew (mode + SWZ_MODE_SKEW; not one of the paper's patterns, but judged by its criterion for
 *   a remap, bijectivity): the tile (pm, pn) the raster gives becomes ((pm + pn) mod grid_m, pn),
 *   i.e. column pn of the grid is rotated down by pn tile rows, so consecutive raster positions
 *   walk a diagonal.  For kernels whose tiles share nothing but whose tile rows collide in the
 *   memory channels (swz_transpose on power-of-two pitches).  swz_softmax / swz_layernorm return
 *   UNSUPPORTED for skewed modes; every other entry point that takes a mode accepts them.
 * Errors: INVALID_ARG (null out, any argument < 1, unknown mode), OVERFLOW (grid_m*grid_n >= 2^31). */
int swz_pid_map(int grid_m, int grid_n, int num_xcd, int group_m, int mode, int32_t* out);

/* The same map (paper: GEMM appendix; the claim "workgroups are dealt round-robin to the XCDs" of
 * the Introduction is what d_xcc lets a caller verify) evaluated by the DEVICE integer code the
 * GEMM kernel uses: launches
 * grid_m*grid_n workgroups; workgroup w writes d_tile[w] = pm*grid_n + pn and, if d_xcc is
 * not null, d_xcc[w] = id of the XCD it actually ran on (hardware register XCC_ID).
 *   d_tile, d_xcc : caller-owned DEVICE buffers of grid_m*grid_n int32.
 * Asynchronous on `stream`; never allocates or synchronises.  Errors as swz_pid_map, plus HIP. */
int swz_pid_map_device(int grid_m, int grid_n, int num_xcd, int group_m, int mode, int32_t* d_tile,
                       int32_t* d_xcc, hipStream_t stream);

/* The PID map of the persistent launch style (the one the paper's GEMM listing uses: the number
 * of workgroups equals the number of compute units and each workgroup loops over tiles).
 * num_wg workgroups; workgroup w is renumbered among the WORKGROUPS (p = XCD renumbering of w
 * over num_wg ids in modes 1/2, p = w otherwise) and computes in round i the tile the raster
 * visits (p + i*num_wg)-th.
 *   out : caller-owned HOST buffer of rounds*num_wg int32, rounds = ceil(grid_m*grid_n / num_wg);
 *         out[i*num_wg + w] = pm*grid_n + pn, or -1 where workgroup w has no tile in round i.
 * Every tile appears exactly once.  Errors as swz_pid_map; num_wg < 1 is INVALID_ARG. */
int swz_pid_map_persistent(int grid_m, int grid_n, int num_xcd, int group_m, int mode, int num_wg, int32_t* out);

/* Same map from the DEVICE code of the persistent GEMM kernel (num_wg workgroups are launched).
 *   d_tile : DEVICE buffer of rounds*num_wg int32, laid out as above;
 *   d_xcc  : optional DEVICE buffer of num_wg int32, the XCD each workgroup ran on.
 * Asynchronous on `stream`; never allocates or synchronises. */
int swz_pid_map_persistent_device(int grid_m, int grid_n, int num_xcd, int group_m, int mode, int num_wg,
                                  int32_t* d_tile, int32_t* d_xcc, hipStream_t stream);

/* C = A . B  (paper's GEMM case study: A is M x K, B is K x N, C is M x N), one workgroup per
 * output tile, workgroup ids remapped according to `mode`.
 *   A, B, C : caller-owned DEVICE pointers, row-major, densely packed (lda = K, ldb = N,
 *             ldc = N), 16-byte aligned, bfloat16.  C is written completely (every element of
 *             every tile, edge tiles masked); A and B are only read.  C must not alias A or B.
 *   dtype   : SWZ_DTYPE_BF16.   mode : a swz_mode.
 *   Products are accumulated in fp32 in ascending-k order per tile and rounded once to
 *   bfloat16 (nearest even); the result bits do not depend on `mode`.
 *   Defaults: num_xcd detected, group_m = 4, tile 256x256x64; when the 256x256 tile grid would have at
 *   most half as many tiles as the device has compute units, 128x256x64, and at most a quarter, 128x128x64
 *   (the chip is then better filled by more and smaller tiles; the result bits do not depend on the tile shape).
 * Asynchronous on `stream`; never allocates or synchronises.
 * Errors: INVALID_ARG (null pointer, M/N/K < 1, unknown mode), UNSUPPORTED (other dtype,
 * K or N not a multiple of 8, misaligned pointer), OVERFLOW (tile count >= 2^31 or a
 * dimension >= 2^31), HIP. */
int swz_gemm(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int dtype, int mode,
             hipStream_t stream);

/* swz_gemm (paper: Appendix "Case Study: GEMM Swizzling") with explicit tile shape / group_m /
 * num_xcd / launch style (null params = all defaults); persistent = 1 is the launch style of the
 * paper's own listing (as many workgroups as compute units, each looping over tiles).
 * UNSUPPORTED for tile rows or columns other than 128 or 256, or bk other than 64.  The persistent launch computes
 * every tile with the same instruction sequence, so its C is bit-identical to the default launch. */
int swz_gemm_ex(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int dtype, int mode,
                const swz_params* params, hipStream_t stream);

/* What swz_gemm_ex would launch for this problem: the resolved parameters and tile grid, i.e. the
 * arguments with which swz_pid_map reproduces the launch's map (the paper validates a remap by
 * its map being a bijection: Results, "broken remappings").
 * Pure host arithmetic apart from the device query that resolves num_xcd = 0.
 * Any output pointer may be null. */
int swz_gemm_plan(int64_t M, int64_t N, int64_t K, const swz_params* params, swz_params* resolved,
                  int* grid_m, int* grid_n);

/* out (N x M) = transpose of in (M x N), elements of 2 or 4 bytes moved verbatim, both row-major and dense
 * (the paper's transpose case study, its largest win from XCD swizzling: Results; Appendix "Case
 * Study: Other Swizzling Pattern Examples").  One workgroup per tile x tile block of `in`; the tile
 * grid is ceil(M/tile) x ceil(N/tile) and hardware workgroup ids are turned into tiles exactly as
 * swz_pid_map does for that grid (`mode`, params->group_m, params->num_xcd; other fields ignored).
 *   in, out : caller-owned DEVICE pointers, 16-byte aligned, must not overlap.
 *   elem_bytes : 2 (M and N multiples of 8) or 4 (M and N multiples of 4, tile 64 only).
 *   tile    : 64 (whole 128-byte lines; the fastest together with mode SWZ_MODE_XCD_GROUPM +
 *             SWZ_MODE_SKEW), 128 (row segments of 256 bytes) or 32 (half lines, shared between
 *             neighbouring tiles: the case where the mapping decides the L2 hit rate).
 *   Once input plus output exceed the 256 MB memory-side cache the stores of tiles 64 and 128 are
 *   streaming stores (the faster choice there, the slower one below it).
 * Asynchronous on `stream`; never allocates or synchronises.
 * Errors: INVALID_ARG (null, M/N < 1, unknown mode), UNSUPPORTED (elem_bytes not 2 or 4, tile not 32/64/128
 * (not 64 for 4-byte elements), M or N not a multiple of 8 (4 for 4-byte elements), misaligned pointer),
 * OVERFLOW, HIP. */
int swz_transpose(const void* in, void* out, int64_t M, int64_t N, int elem_bytes, int tile, int mode,
                  const swz_params* params, hipStream_t stream);

/* Row softmax, y[i][j] = exp(x[i][j] - max_i) / sum_k exp(x[i][k] - max_i), over a row-major dense
 * M x N bfloat16 matrix (the paper's softmax kernel: Results; Appendix "Case Study: Other Swizzling
 * Pattern Examples", whose swizzle routes all column chunks of a row to one XCD).  Each row is cut
 * into `chunks` column chunks of ceil(N/8/chunks) 16-byte vectors (trailing chunks may be empty);
 * one workgroup reads the whole row for the row statistics and writes one chunk.  The grid is
 * M x chunks and hardware workgroup ids are decoded exactly as swz_pid_map does for that grid
 * (tile row = matrix row, tile column = chunk; `mode`, params->group_m, params->num_xcd; other
 * fields ignored).  chunks = 1 gives one workgroup per row, except that rows of at most 2048
 * elements are then handled one per wave: the grid is ceil(M/4) x 1 groups of four consecutive rows.
 *   in, out : caller-owned DEVICE pointers, 16-byte aligned, must not overlap.  -inf entries are
 *             allowed (they get probability 0); a row of only -inf gives NaN.
 *   fp32 arithmetic, one rounding to bfloat16 (nearest even); the result bits never depend on
 *   `mode`, and for N > 2048 not on `chunks` either.
 * Asynchronous on `stream`; never allocates or synchronises.
 * Errors: INVALID_ARG (null, M/N/chunks < 1, chunks > N/8, unknown mode), UNSUPPORTED (N not a
 * multiple of 8 or above 2^24, misaligned pointer), OVERFLOW (M*chunks or a dimension >= 2^31), HIP. */
int swz_softmax(const void* in, void* out, int64_t M, int64_t N, int chunks, int mode, const swz_params* params,
                hipStream_t stream);

/* Layer normalisation of every row, y[i][j] = (x[i][j] - mean_i) / sqrt(var_i + eps) * gamma[j] + beta[j]
 * with the biased variance (the paper's layer normalisation kernel, same appendix: all column chunks
 * of a row on one XCD).  Same decomposition, grid, mapping, layout and error behaviour as swz_softmax.
 *   gamma, beta : DEVICE pointers to N bfloat16 each, 16-byte aligned.   eps >= 0.
 *   Mean and variance are accumulated in fp32 with pairwise (count, mean, M2) merges. */
int swz_layernorm(const void* in, const void* gamma, const void* beta, void* out, int64_t M, int64_t N, float eps,
                  int chunks, int mode, const swz_params* params, hipStream_t stream);

/* Measurement aid: swz_gemm_ex (one workgroup per tile only; persistent = 1 is UNSUPPORTED) run by
 * an instantiation of the same kernel that also takes time stamps, so that what bounds the kernel
 * (clock under load, cycles per K step, when each XCD finishes) can be read per workgroup.  The
 * stamps are kept in scalar registers while the tile is computed and written once at its end: the
 * loop's instruction stream is the product kernel's.  C is computed as by swz_gemm_ex.
 *   probe       : DEVICE buffer, 8-byte aligned, of probe_words >= 16 * grid_m * grid_n 64-bit words;
 *                 workgroup w (hardware id) writes words 16w .. 16w+15:
 *                 0,1  shader clock counter / constant 100 MHz counter at kernel entry
 *                 2,3  the same pair when the K loop starts (first operands have landed)
 *                 4,5  when the K loop has ended        6,7  when the last store has been issued
 *                 8    XCC_ID (the XCD it ran on)       9    HW_ID register
 *                 10   K steps of 32 the loop made      11, 12  tile row, tile column      13..15  zero
 * Asynchronous on `stream`; never allocates or synchronises.  Errors as swz_gemm_ex, plus INVALID_ARG
 * (null or too small probe buffer). */
int swz_gemm_probe(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int dtype, int mode,
                   const swz_params* params, uint64_t* probe, int64_t probe_words, hipStream_t stream);

/* Measurement aid, not part of the GEMM path: a plain streaming copy of `bytes` bytes
 * (reads `bytes`, writes `bytes`; both DEVICE pointers 16-byte aligned, bytes a multiple of
 * 16, buffers must not overlap).  The profiling harness scales the profiler's HBM byte
 * counters by what they read for this kernel of known traffic.
 * Asynchronous on `stream`.  Errors: INVALID_ARG (null, bytes < 16), UNSUPPORTED (alignment), HIP. */
int swz_copy_bytes(const void* src, void* dst, int64_t bytes, hipStream_t stream);

/* Measurement aid, not part of the GEMM path: the matrix-core rate the device sustains with nothing
 * else going on, against which the GEMM's TFLOP/s can be read beside the data-sheet peak.  Launches
 * one 512-thread workgroup per compute unit; every wave issues iters x 64 independent
 * v_mfma_f32_16x16x32_bf16 (16384 flop each) on register operands: pseudo-random bfloat16 values if
 * random_operands != 0, zeros otherwise (the clock the chip sustains depends on the data).
 * Flop per launch = *workgroups x 8 x iters x 64 x 16384.
 *   out : DEVICE buffer of out_floats >= 512 x (number of compute units) floats; receives one
 *         value per thread (the kernel's only memory traffic).   workgroups : HOST, may be null.
 * Asynchronous on `stream`.  Errors: INVALID_ARG (null, iters < 1, buffer too small), HIP. */
int swz_mfma_peak(float* out, int64_t out_floats, int iters, int random_operands, int* workgroups, hipStream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* SWZ_H */
