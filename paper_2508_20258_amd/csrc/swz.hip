// libswz: C-ABI entry points (declared in include/swz.h).  Host side: argument checks,
// tile choice, launches.  Nothing here allocates device memory or synchronises.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <stdlib.h>

#include <atomic>
#include <mutex>
#include <tuple>
#include <utility>

#include "../../include/swz.h"
#include "aux_kernels.h"
#include "gemm_kernel.h"
#include "mfma_peak_kernel.h"
#include "pid_decode.h"
#include "rowwise_kernel.h"
#include "transpose_kernel.h"

namespace {

constexpr int kCusPerXcd = 32;   // gfx950: 8 XCDs x 32 CUs
constexpr int kMaxDevices = 64;
constexpr int kDefaultBK = 64;  // K panel of a tile step; the kernel moves it as two 32-wide halves (ring of 4)

struct DeviceFacts {
  bool known = false;
  int num_xcd = 0, cus = 0, l2_bytes = 0, lds_bytes = 0;   // num_xcd 0: could not be derived
};
DeviceFacts g_facts[kMaxDevices];
std::atomic<bool> g_attr_set[kMaxDevices][4][4][2];
std::mutex g_mu;

// SWZ_NUM_XCD in the environment (read once per process): the XCD count to assume instead of the
// one derived from the CU count, for partitioned devices.  0 = not set or not a number in 1..1024.
int env_num_xcd() {
  static const int value = [] {
    const char* e = getenv("SWZ_NUM_XCD");
    if (e == nullptr || *e == 0) return 0;
    char* end = nullptr;
    const long v = strtol(e, &end, 10);
    return (end != nullptr && *end == 0 && v >= 1 && v <= 1024) ? (int)v : 0;
  }();
  return value;
}

int query_device(DeviceFacts* out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SWZ_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_mu);
  DeviceFacts& f = g_facts[dev];
  if (!f.known) {
    int cus = 0, l2 = 0, lds = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return SWZ_ERR_HIP;
    if (hipDeviceGetAttribute(&l2, hipDeviceAttributeL2CacheSize, dev) != hipSuccess) return SWZ_ERR_HIP;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return SWZ_ERR_HIP;
    f.cus = cus;
    f.l2_bytes = l2;
    f.lds_bytes = lds;
    // XCDs come in whole units of 32 CUs (a partitioned device exposes fewer of them); any other
    // CU count is not guessed at: the caller then has to name the XCD count.
    if (env_num_xcd() > 0) f.num_xcd = env_num_xcd();
    else f.num_xcd = (cus >= kCusPerXcd && cus % kCusPerXcd == 0) ? cus / kCusPerXcd : 0;
    f.known = true;
  }
  *out = f;
  return SWZ_OK;
}

// Launch through the call that returns the launch's own status: hipGetLastError() after a launch
// would also report (and clear) an error some earlier, unrelated HIP call left behind.
template <class... KArgs, size_t... Is>
int launch_impl(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                std::tuple<KArgs...>& vals, std::index_sequence<Is...>) {
  void* ptrs[] = {static_cast<void*>(&std::get<Is>(vals))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, stream) == hipSuccess ? SWZ_OK
                                                                                                             : SWZ_ERR_HIP;
}
template <class... KArgs, class... Args>
int launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream, Args... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count");
  std::tuple<KArgs...> vals{static_cast<KArgs>(args)...};
  return launch_impl(kernel, grid, block, lds, stream, vals, std::index_sequence_for<KArgs...>{});
}

bool valid_mode(int mode) { return mode >= 0 && mode < kModeCount; }

// Shared checks of the two PID-map entry points.  Clamps group_m to grid_m (same raster).
int check_map_args(int grid_m, int grid_n, int num_xcd, int* group_m, int mode) {
  if (grid_m < 1 || grid_n < 1 || num_xcd < 1 || *group_m < 1 || !valid_mode(mode)) return SWZ_ERR_INVALID_ARG;
  if ((int64_t)grid_m * (int64_t)grid_n >= (int64_t)1 << 31) return SWZ_ERR_OVERFLOW;
  if (*group_m > grid_m) *group_m = grid_m;
  return SWZ_OK;
}

// num_wg == 0: one workgroup per tile; otherwise the persistent kernel with num_wg workgroups.
template <class S, int MODE>
int launch_gemm_mode(const void* A, const void* B, void* C, int M, int N, int K, int grid_m, int grid_n,
                     int num_xcd, int group_m, int skew, int num_wg, hipStream_t stream, int slot) {
  auto kernel = num_wg > 0 ? swz::gemm_bf16_persistent_kernel<S, MODE> : swz::gemm_bf16_kernel<S, MODE>;
  const int style = num_wg > 0 ? 1 : 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SWZ_ERR_HIP;
  std::atomic<bool>& ready = g_attr_set[dev][slot][MODE][style];
  if (!ready.load(std::memory_order_acquire)) {       // first launch of this kernel on this device only
    std::lock_guard<std::mutex> lock(g_mu);
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            S::LDS_BYTES) != hipSuccess)
      return SWZ_ERR_HIP;
    ready.store(true, std::memory_order_release);
  }
  const unsigned blocks = (unsigned)(num_wg > 0 ? num_wg : grid_m * grid_n);
  return launch(kernel, dim3(blocks), dim3(S::NT), S::LDS_BYTES, stream, static_cast<const uint16_t*>(A),
                static_cast<const uint16_t*>(B), static_cast<uint16_t*>(C), M, N, K, grid_m, grid_n, num_xcd, group_m, skew);
}

template <class S>
int launch_gemm(const void* A, const void* B, void* C, int M, int N, int K, int grid_m, int grid_n,
                int num_xcd, int group_m, int mode, int num_wg, hipStream_t stream, int slot) {
  const int skew = swz_mode_skewed(mode) ? 1 : 0;
  switch (mode & 3) {
    case SWZ_MODE_RR: return launch_gemm_mode<S, kModeRR>(A, B, C, M, N, K, grid_m, grid_n, num_xcd, group_m, skew, num_wg, stream, slot);
    case SWZ_MODE_XCD: return launch_gemm_mode<S, kModeXcd>(A, B, C, M, N, K, grid_m, grid_n, num_xcd, group_m, skew, num_wg, stream, slot);
    case SWZ_MODE_XCD_GROUPM: return launch_gemm_mode<S, kModeXcdGroupM>(A, B, C, M, N, K, grid_m, grid_n, num_xcd, group_m, skew, num_wg, stream, slot);
    default: return launch_gemm_mode<S, kModeGroupM>(A, B, C, M, N, K, grid_m, grid_n, num_xcd, group_m, skew, num_wg, stream, slot);
  }
}

template <class S>
int launch_gemm_probe(const void* A, const void* B, void* C, int M, int N, int K, int grid_m, int grid_n, int num_xcd,
                      int group_m, int mode, uint64_t* probe, hipStream_t stream) {
  auto go = [&](auto kernel) {
    // set on every call: this is a measurement aid, not a hot path
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            S::LDS_BYTES) != hipSuccess)
      return (int)SWZ_ERR_HIP;
    return launch(kernel, dim3((unsigned)(grid_m * grid_n)), dim3(S::NT), S::LDS_BYTES, stream,
                  static_cast<const uint16_t*>(A), static_cast<const uint16_t*>(B), static_cast<uint16_t*>(C), M, N, K,
                  grid_m, grid_n, num_xcd, group_m, swz_mode_skewed(mode) ? 1 : 0, probe);
  };
  switch (mode & 3) {
    case SWZ_MODE_RR: return go(swz::gemm_bf16_probe_kernel<S, kModeRR>);
    case SWZ_MODE_XCD: return go(swz::gemm_bf16_probe_kernel<S, kModeXcd>);
    case SWZ_MODE_XCD_GROUPM: return go(swz::gemm_bf16_probe_kernel<S, kModeXcdGroupM>);
    default: return go(swz::gemm_bf16_probe_kernel<S, kModeGroupM>);
  }
}

int resolve_plan(int64_t M, int64_t N, int64_t K, const swz_params* p, swz_params* r, int* grid_m, int* grid_n) {
  if (M < 1 || N < 1 || K < 1) return SWZ_ERR_INVALID_ARG;
  const int64_t lim = (int64_t)1 << 31;
  if (M >= lim || N >= lim || K >= lim) return SWZ_ERR_OVERFLOW;
  swz_params q = {0, 0, 0, 0, 0, 0, 0};
  if (p != nullptr) q = *p;
  if (q.bm < 0 || q.bn < 0 || q.bk < 0 || q.group_m < 0 || q.num_xcd < 0 || q.num_wg < 0 ||
      (q.persistent != 0 && q.persistent != 1))
    return SWZ_ERR_INVALID_ARG;
  if (q.bm == 0 && q.bn == 0) {
    // 256x256 tiles are the faster kernel once they fill the chip; below that, more and smaller tiles are.
    // Measured (tiles of the 256x256 grid against compute units): up to a quarter, 128x128 tiles are 1.6-2.0x
    // faster; between a quarter and a half, 128x256 tiles are 1.25-1.3x faster (and 3-14 % ahead of 128x128);
    // above a half, 256x256 tiles win by 1.2-1.3x.  The device is only asked where its CU count decides.
    const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
    int cus = 256;                                  // assumed where no device can be asked (a whole MI355X)
    if (t256 > 8 && t256 <= 152) {
      DeviceFacts f;
      if (query_device(&f) == SWZ_OK && f.cus > 0) cus = f.cus;
    }
    q.bm = 2 * t256 <= cus ? 128 : 256;
    q.bn = 4 * t256 <= cus ? 128 : 256;
  }
  if (q.bm == 0) q.bm = q.bn;
  if (q.bn == 0) q.bn = q.bm;
  if (q.bk == 0) q.bk = kDefaultBK;
  if (q.group_m == 0) q.group_m = 4;
  if (!((q.bm == 128 || q.bm == 256) && (q.bn == 128 || q.bn == 256)) || q.bk != kDefaultBK) return SWZ_ERR_UNSUPPORTED;
  const int64_t gm = (M + q.bm - 1) / q.bm, gn = (N + q.bn - 1) / q.bn;
  if (gm * gn >= lim) return SWZ_ERR_OVERFLOW;
  if (q.num_xcd == 0 || (q.persistent && q.num_wg == 0)) {
    DeviceFacts f;
    const int st = query_device(&f);
    if (st != SWZ_OK) return st;
    if (q.num_xcd == 0) q.num_xcd = f.num_xcd;
    if (q.num_xcd == 0) return SWZ_ERR_UNSUPPORTED;   // CU count is not a whole number of XCDs: the caller must name it
    if (q.persistent && q.num_wg == 0) q.num_wg = f.cus;
  }
  if (!q.persistent) q.num_wg = 0;
  else if (q.num_wg > gm * gn) q.num_wg = (int32_t)(gm * gn);   // never more workgroups than tiles
  if (r != nullptr) *r = q;
  if (grid_m != nullptr) *grid_m = (int)gm;
  if (grid_n != nullptr) *grid_n = (int)gn;
  return SWZ_OK;
}

constexpr int64_t kMemorySideCacheBytes = (int64_t)256 << 20;   // gfx950: 256 MB behind the L2s, in front of HBM

template <int TILE, bool STREAM>
int launch_transpose_s(const void* in, void* out, int M, int N, int gm, int gn, int num_xcd, int group_m, int mode,
                       hipStream_t stream) {
  const dim3 grid((unsigned)(gm * gn)), block(256);
  auto* i = static_cast<const uint16_t*>(in);
  auto* o = static_cast<uint16_t*>(out);
  const int skew = swz_mode_skewed(mode) ? 1 : 0;
  switch (mode & 3) {
    case SWZ_MODE_RR: return launch(swz::transpose16_kernel<TILE, kModeRR, STREAM>, grid, block, 0, stream, i, o, M, N, gm, gn, num_xcd, group_m, skew);
    case SWZ_MODE_XCD: return launch(swz::transpose16_kernel<TILE, kModeXcd, STREAM>, grid, block, 0, stream, i, o, M, N, gm, gn, num_xcd, group_m, skew);
    case SWZ_MODE_XCD_GROUPM: return launch(swz::transpose16_kernel<TILE, kModeXcdGroupM, STREAM>, grid, block, 0, stream, i, o, M, N, gm, gn, num_xcd, group_m, skew);
    default: return launch(swz::transpose16_kernel<TILE, kModeGroupM, STREAM>, grid, block, 0, stream, i, o, M, N, gm, gn, num_xcd, group_m, skew);
  }
}

template <bool STREAM>
int launch_transpose32(const void* in, void* out, int M, int N, int gm, int gn, int num_xcd, int group_m, int mode,
                       hipStream_t stream) {
  const dim3 grid((unsigned)(gm * gn)), block(256);
  auto* i = static_cast<const uint32_t*>(in);
  auto* o = static_cast<uint32_t*>(out);
  const int skew = swz_mode_skewed(mode) ? 1 : 0;
  switch (mode & 3) {
    case SWZ_MODE_RR: return launch(swz::transpose32_kernel<kModeRR, STREAM>, grid, block, 0, stream, i, o, M, N, gm, gn, num_xcd, group_m, skew);
    case SWZ_MODE_XCD: return launch(swz::transpose32_kernel<kModeXcd, STREAM>, grid, block, 0, stream, i, o, M, N, gm, gn, num_xcd, group_m, skew);
    case SWZ_MODE_XCD_GROUPM: return launch(swz::transpose32_kernel<kModeXcdGroupM, STREAM>, grid, block, 0, stream, i, o, M, N, gm, gn, num_xcd, group_m, skew);
    default: return launch(swz::transpose32_kernel<kModeGroupM, STREAM>, grid, block, 0, stream, i, o, M, N, gm, gn, num_xcd, group_m, skew);
  }
}

template <int TILE>
int launch_transpose(const void* in, void* out, int M, int N, int gm, int gn, int num_xcd, int group_m, int mode,
                     hipStream_t stream) {
  // streaming stores once input plus output no longer fit the memory-side cache (and only where a store
  // instruction covers whole lines: tiles of 64 and 128)
  if (TILE >= 64 && (int64_t)M * N * 4 > kMemorySideCacheBytes)
    return launch_transpose_s<TILE, true>(in, out, M, N, gm, gn, num_xcd, group_m, mode, stream);
  return launch_transpose_s<TILE, false>(in, out, M, N, gm, gn, num_xcd, group_m, mode, stream);
}
// How the two row-wise entry points launch: threads per row (256, or 64 = one row per wave when a
// single workgroup per row is asked for and the row has at most 2048 elements), 16-byte vectors a
// thread keeps in registers (0 = the row is streamed twice), the grid and the mapping parameters.
struct RowPlan {
  int tpr, keep, grid_m, chunk_vecs, num_xcd, group_m;
};

int resolve_rows(int64_t M, int64_t N, int chunks, int mode, const swz_params* params, RowPlan* plan) {
  if (M < 1 || N < 1 || chunks < 1 || !valid_mode(mode)) return SWZ_ERR_INVALID_ARG;
  if (swz_mode_skewed(mode)) return SWZ_ERR_UNSUPPORTED;   // a skew would pull the chunks of a row apart again
  const int64_t lim = (int64_t)1 << 31;
  if (M >= lim || N >= lim || M * chunks >= lim) return SWZ_ERR_OVERFLOW;
  if ((N % 8) != 0 || N > ((int64_t)1 << 24)) return SWZ_ERR_UNSUPPORTED;   // 16-byte vectors; fp32 element counts stay exact
  const int64_t nv = N / 8;
  if (chunks > nv) return SWZ_ERR_INVALID_ARG;
  plan->group_m = 4;
  plan->num_xcd = 0;
  if (params != nullptr) {
    if (params->group_m < 0 || params->num_xcd < 0) return SWZ_ERR_INVALID_ARG;
    if (params->group_m > 0) plan->group_m = params->group_m;
    plan->num_xcd = params->num_xcd;
  }
  if (plan->num_xcd == 0) {
    DeviceFacts f;
    const int st = query_device(&f);
    if (st != SWZ_OK) return st;
    plan->num_xcd = f.num_xcd;
    if (plan->num_xcd == 0) return SWZ_ERR_UNSUPPORTED;
  }
  plan->chunk_vecs = (int)((nv + chunks - 1) / chunks);
  plan->tpr = (chunks == 1 && nv <= 4 * 64) ? 64 : swz::kRowThreads;
  const int64_t per_thread = (nv + plan->tpr - 1) / plan->tpr;
  plan->keep = chunks != 1 ? 0 : per_thread <= 4 ? 4 : per_thread <= 16 ? 16 : 0;
  const int rows_per_wg = swz::kRowThreads / plan->tpr;
  plan->grid_m = (int)((M + rows_per_wg - 1) / rows_per_wg);
  return check_map_args(plan->grid_m, chunks, plan->num_xcd, &plan->group_m, mode);
}

#define SWZ_LAUNCH_BY_MODE(KERNEL, KEEP, TPR, ...)                                                                \
  switch (mode) {                                                                                                 \
    case SWZ_MODE_RR: return launch(KERNEL<kModeRR, KEEP, TPR>, grid, block, 0, stream, __VA_ARGS__);             \
    case SWZ_MODE_XCD: return launch(KERNEL<kModeXcd, KEEP, TPR>, grid, block, 0, stream, __VA_ARGS__);           \
    case SWZ_MODE_XCD_GROUPM: return launch(KERNEL<kModeXcdGroupM, KEEP, TPR>, grid, block, 0, stream, __VA_ARGS__); \
    case SWZ_MODE_GROUPM: return launch(KERNEL<kModeGroupM, KEEP, TPR>, grid, block, 0, stream, __VA_ARGS__);     \
    default: return SWZ_ERR_INVALID_ARG;                                                                          \
  }
#define SWZ_LAUNCH_BY_PLAN(KERNEL, ...)                                          \
  if (plan.tpr == 64) {                                                          \
    SWZ_LAUNCH_BY_MODE(KERNEL, 4, 64, __VA_ARGS__)                               \
  } else if (plan.keep == 4) {                                                   \
    SWZ_LAUNCH_BY_MODE(KERNEL, 4, 256, __VA_ARGS__)                              \
  } else if (plan.keep == 16) {                                                  \
    SWZ_LAUNCH_BY_MODE(KERNEL, 16, 256, __VA_ARGS__)                             \
  } else {                                                                       \
    SWZ_LAUNCH_BY_MODE(KERNEL, 0, 256, __VA_ARGS__)                              \
  }
}  // namespace

extern "C" {

const char* swz_status_string(int status) {
  switch (status) {
    case SWZ_OK: return "ok";
    case SWZ_ERR_INVALID_ARG: return "invalid argument";
    case SWZ_ERR_UNSUPPORTED: return "unsupported dtype, alignment or tile shape";
    case SWZ_ERR_OVERFLOW: return "size does not fit 32-bit tile arithmetic";
    case SWZ_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int swz_device_info(int* num_xcd, int* compute_units, int* l2_bytes, int* lds_bytes) {
  DeviceFacts f;
  const int st = query_device(&f);
  if (st != SWZ_OK) return st;
  if (num_xcd) *num_xcd = f.num_xcd;
  if (compute_units) *compute_units = f.cus;
  if (l2_bytes) *l2_bytes = f.l2_bytes;
  if (lds_bytes) *lds_bytes = f.lds_bytes;
  return SWZ_OK;
}

int swz_pid_map(int grid_m, int grid_n, int num_xcd, int group_m, int mode, int32_t* out) {
  if (out == nullptr) return SWZ_ERR_INVALID_ARG;
  const int st = check_map_args(grid_m, grid_n, num_xcd, &group_m, mode);
  if (st != SWZ_OK) return st;
  const int total = grid_m * grid_n;
  for (int w = 0; w < total; ++w) {
    int pm, pn;
    swz_decode_tile(w, grid_m, grid_n, num_xcd, group_m, mode, &pm, &pn);
    out[w] = pm * grid_n + pn;
  }
  return SWZ_OK;
}

int swz_pid_map_device(int grid_m, int grid_n, int num_xcd, int group_m, int mode, int32_t* d_tile,
                       int32_t* d_xcc, hipStream_t stream) {
  if (d_tile == nullptr) return SWZ_ERR_INVALID_ARG;
  const int st = check_map_args(grid_m, grid_n, num_xcd, &group_m, mode);
  if (st != SWZ_OK) return st;
  return launch(swz::pid_map_kernel, dim3((unsigned)(grid_m * grid_n)), dim3(64), 0, stream, grid_m, grid_n, num_xcd,
                group_m, mode, d_tile, d_xcc);
}

int swz_pid_map_persistent(int grid_m, int grid_n, int num_xcd, int group_m, int mode, int num_wg, int32_t* out) {
  if (out == nullptr || num_wg < 1) return SWZ_ERR_INVALID_ARG;
  const int st = check_map_args(grid_m, grid_n, num_xcd, &group_m, mode);
  if (st != SWZ_OK) return st;
  const int total = grid_m * grid_n;
  const int64_t rounds = ((int64_t)total + num_wg - 1) / num_wg;
  if (rounds * num_wg >= (int64_t)1 << 31) return SWZ_ERR_OVERFLOW;
  for (int round = 0; round < (int)rounds; ++round) {
    for (int w = 0; w < num_wg; ++w) {
      const int l = swz_persistent_logical(w, round, num_wg, total, num_xcd, mode);
      int t = -1;
      if (l >= 0) {
        int pm, pn;
        swz_tile_at(l, grid_m, grid_n, group_m, mode, &pm, &pn);
        t = pm * grid_n + pn;
      }
      out[(size_t)round * num_wg + w] = t;
    }
  }
  return SWZ_OK;
}

int swz_pid_map_persistent_device(int grid_m, int grid_n, int num_xcd, int group_m, int mode, int num_wg,
                                  int32_t* d_tile, int32_t* d_xcc, hipStream_t stream) {
  if (d_tile == nullptr || num_wg < 1) return SWZ_ERR_INVALID_ARG;
  const int st = check_map_args(grid_m, grid_n, num_xcd, &group_m, mode);
  if (st != SWZ_OK) return st;
  const int64_t rounds = ((int64_t)grid_m * grid_n + num_wg - 1) / num_wg;
  if (rounds * num_wg >= (int64_t)1 << 31) return SWZ_ERR_OVERFLOW;
  return launch(swz::pid_map_persistent_kernel, dim3((unsigned)num_wg), dim3(64), 0, stream, grid_m, grid_n, num_xcd,
                group_m, mode, (int)rounds, d_tile, d_xcc);
}

int swz_transpose(const void* in, void* out, int64_t M, int64_t N, int elem_bytes, int tile, int mode,
                  const swz_params* params, hipStream_t stream) {
  if (in == nullptr || out == nullptr || M < 1 || N < 1 || !valid_mode(mode)) return SWZ_ERR_INVALID_ARG;
  const int64_t lim = (int64_t)1 << 31;
  if (M >= lim || N >= lim) return SWZ_ERR_OVERFLOW;
  if (elem_bytes == 4) {
    if (tile != 64 || (M % 4) != 0 || (N % 4) != 0) return SWZ_ERR_UNSUPPORTED;
  } else if (elem_bytes != 2 || (tile != 32 && tile != 64 && tile != 128) || (M % 8) != 0 || (N % 8) != 0) {
    return SWZ_ERR_UNSUPPORTED;
  }
  if ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) return SWZ_ERR_UNSUPPORTED;
  int group_m = 4, num_xcd = 0;
  if (params != nullptr) {
    if (params->group_m < 0 || params->num_xcd < 0) return SWZ_ERR_INVALID_ARG;
    if (params->group_m > 0) group_m = params->group_m;
    num_xcd = params->num_xcd;
  }
  if (num_xcd == 0) {
    DeviceFacts f;
    const int st = query_device(&f);
    if (st != SWZ_OK) return st;
    num_xcd = f.num_xcd;
    if (num_xcd == 0) return SWZ_ERR_UNSUPPORTED;
  }
  const int64_t gm = (M + tile - 1) / tile, gn = (N + tile - 1) / tile;
  if (gm * gn >= lim) return SWZ_ERR_OVERFLOW;
  const int st = check_map_args((int)gm, (int)gn, num_xcd, &group_m, mode);
  if (st != SWZ_OK) return st;
  if (elem_bytes == 4) {
    if (M * N * 8 > kMemorySideCacheBytes)
      return launch_transpose32<true>(in, out, (int)M, (int)N, (int)gm, (int)gn, num_xcd, group_m, mode, stream);
    return launch_transpose32<false>(in, out, (int)M, (int)N, (int)gm, (int)gn, num_xcd, group_m, mode, stream);
  }
  if (tile == 128) return launch_transpose<128>(in, out, (int)M, (int)N, (int)gm, (int)gn, num_xcd, group_m, mode, stream);
  return tile == 64 ? launch_transpose<64>(in, out, (int)M, (int)N, (int)gm, (int)gn, num_xcd, group_m, mode, stream)
                    : launch_transpose<32>(in, out, (int)M, (int)N, (int)gm, (int)gn, num_xcd, group_m, mode, stream);
}

int swz_softmax(const void* in, void* out, int64_t M, int64_t N, int chunks, int mode, const swz_params* params,
                hipStream_t stream) {
  if (in == nullptr || out == nullptr) return SWZ_ERR_INVALID_ARG;
  RowPlan plan;
  const int st = resolve_rows(M, N, chunks, mode, params, &plan);
  if (st != SWZ_OK) return st;
  if ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) return SWZ_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)((int64_t)plan.grid_m * chunks)), block(swz::kRowThreads);
  SWZ_LAUNCH_BY_PLAN(swz::softmax_rows_kernel, static_cast<const uint16_t*>(in), static_cast<uint16_t*>(out), (int)M,
                     (int)N, chunks, plan.chunk_vecs, plan.num_xcd, plan.group_m)
}

int swz_layernorm(const void* in, const void* gamma, const void* beta, void* out, int64_t M, int64_t N, float eps,
                  int chunks, int mode, const swz_params* params, hipStream_t stream) {
  if (in == nullptr || gamma == nullptr || beta == nullptr || out == nullptr || !(eps >= 0.f)) return SWZ_ERR_INVALID_ARG;
  RowPlan plan;
  const int st = resolve_rows(M, N, chunks, mode, params, &plan);
  if (st != SWZ_OK) return st;
  if ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(gamma) |
       reinterpret_cast<uintptr_t>(beta)) & 15)
    return SWZ_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)((int64_t)plan.grid_m * chunks)), block(swz::kRowThreads);
  SWZ_LAUNCH_BY_PLAN(swz::layernorm_rows_kernel, static_cast<const uint16_t*>(in), static_cast<const uint16_t*>(gamma),
                     static_cast<const uint16_t*>(beta), static_cast<uint16_t*>(out), (int)M, (int)N, eps, chunks,
                     plan.chunk_vecs, plan.num_xcd, plan.group_m)
}

int swz_mfma_peak(float* out, int64_t out_floats, int iters, int random_operands, int* workgroups, hipStream_t stream) {
  if (out == nullptr || iters < 1) return SWZ_ERR_INVALID_ARG;
  DeviceFacts f;
  const int st = query_device(&f);
  if (st != SWZ_OK) return st;
  if (out_floats < (int64_t)f.cus * 512) return SWZ_ERR_INVALID_ARG;
  if (workgroups != nullptr) *workgroups = f.cus;
  return launch(swz::mfma_peak_kernel, dim3((unsigned)f.cus), dim3(512), 0, stream, out, iters, random_operands ? 1 : 0);
}

int swz_copy_bytes(const void* src, void* dst, int64_t bytes, hipStream_t stream) {
  if (src == nullptr || dst == nullptr || bytes < 16) return SWZ_ERR_INVALID_ARG;
  if ((bytes & 15) || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15)) return SWZ_ERR_UNSUPPORTED;
  const int64_t n = bytes / 16;
  const int64_t want = (n + 1023) / 1024;                       // a workgroup moves 1024 words per round
  const unsigned blocks = (unsigned)(want < 8192 ? want : 8192);
  return launch(swz::copy16_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<const swz::aux_u32x4*>(src),
                static_cast<swz::aux_u32x4*>(dst), n);
}

int swz_gemm_plan(int64_t M, int64_t N, int64_t K, const swz_params* params, swz_params* resolved, int* grid_m,
                  int* grid_n) {
  return resolve_plan(M, N, K, params, resolved, grid_m, grid_n);
}

// The four tile shapes: 8 waves each; 256x256 -> wave tile 128x64, the other three -> wave tile 64x64 or 64x32.
using Shape128 = swz::GemmShape<128, 128, 2, 4>;
using Shape256 = swz::GemmShape<256, 256, 2, 4>;
using Shape128x256 = swz::GemmShape<128, 256, 2, 4>;
using Shape256x128 = swz::GemmShape<256, 128, 4, 2>;

// Checks shared by the GEMM entry points; on success r, grid_m, grid_n and group_m describe the launch.
static int check_gemm(const void* A, const void* B, const void* C, int64_t M, int64_t N, int64_t K, int dtype, int mode,
                      const swz_params* params, swz_params* r, int* grid_m, int* grid_n, int* group_m) {
  if (A == nullptr || B == nullptr || C == nullptr || !valid_mode(mode)) return SWZ_ERR_INVALID_ARG;
  int st = resolve_plan(M, N, K, params, r, grid_m, grid_n);
  if (st != SWZ_OK) return st;
  if (dtype != SWZ_DTYPE_BF16) return SWZ_ERR_UNSUPPORTED;
  if ((K % 8) != 0 || (N % 8) != 0) return SWZ_ERR_UNSUPPORTED;   // 16-byte vector loads along k and n
  // per-lane source offsets inside a tile step are 32-bit: (bm-1) rows of A, 31 rows of B
  if ((int64_t)r->bm * K * 2 >= ((int64_t)1 << 32) || (int64_t)32 * N * 2 >= ((int64_t)1 << 32)) return SWZ_ERR_OVERFLOW;
  if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(C)) & 15)
    return SWZ_ERR_UNSUPPORTED;
  *group_m = r->group_m;
  return check_map_args(*grid_m, *grid_n, r->num_xcd, group_m, mode);
}

int swz_gemm_ex(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int dtype, int mode,
                const swz_params* params, hipStream_t stream) {
  swz_params r;
  int grid_m = 0, grid_n = 0, group_m = 0;
  const int st = check_gemm(A, B, C, M, N, K, dtype, mode, params, &r, &grid_m, &grid_n, &group_m);
  if (st != SWZ_OK) return st;
  if (r.bm == 128 && r.bn == 128)
    return launch_gemm<Shape128>(A, B, C, (int)M, (int)N, (int)K, grid_m, grid_n, r.num_xcd, group_m, mode, r.num_wg, stream, 0);
  if (r.bm == 128)
    return launch_gemm<Shape128x256>(A, B, C, (int)M, (int)N, (int)K, grid_m, grid_n, r.num_xcd, group_m, mode, r.num_wg, stream, 2);
  if (r.bn == 128)
    return launch_gemm<Shape256x128>(A, B, C, (int)M, (int)N, (int)K, grid_m, grid_n, r.num_xcd, group_m, mode, r.num_wg, stream, 3);
  return launch_gemm<Shape256>(A, B, C, (int)M, (int)N, (int)K, grid_m, grid_n, r.num_xcd, group_m, mode, r.num_wg, stream, 1);
}

int swz_gemm_probe(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int dtype, int mode,
                   const swz_params* params, uint64_t* probe, int64_t probe_words, hipStream_t stream) {
  if (probe == nullptr) return SWZ_ERR_INVALID_ARG;
  swz_params r;
  int grid_m = 0, grid_n = 0, group_m = 0;
  const int st = check_gemm(A, B, C, M, N, K, dtype, mode, params, &r, &grid_m, &grid_n, &group_m);
  if (st != SWZ_OK) return st;
  if (r.persistent) return SWZ_ERR_UNSUPPORTED;
  if (probe_words < (int64_t)grid_m * grid_n * swz::kProbeWords) return SWZ_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(probe) & 7) return SWZ_ERR_UNSUPPORTED;
  if (r.bm == 128 && r.bn == 128)
    return launch_gemm_probe<Shape128>(A, B, C, (int)M, (int)N, (int)K, grid_m, grid_n, r.num_xcd, group_m, mode, probe, stream);
  if (r.bm == 128)
    return launch_gemm_probe<Shape128x256>(A, B, C, (int)M, (int)N, (int)K, grid_m, grid_n, r.num_xcd, group_m, mode, probe, stream);
  if (r.bn == 128)
    return launch_gemm_probe<Shape256x128>(A, B, C, (int)M, (int)N, (int)K, grid_m, grid_n, r.num_xcd, group_m, mode, probe, stream);
  return launch_gemm_probe<Shape256>(A, B, C, (int)M, (int)N, (int)K, grid_m, grid_n, r.num_xcd, group_m, mode, probe, stream);
}

int swz_gemm(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int dtype, int mode,
             hipStream_t stream) {
  return swz_gemm_ex(A, B, C, M, N, K, dtype, mode, nullptr, stream);
}

}  // extern "C"
