// Internal declarations shared by the HIP translation units of librtc.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>
#include <tuple>
#include <utility>

#include "rtc.h"

namespace rtc {

// Element size of a dtype, 0 when unknown.
inline size_t elem_size(int dt) {
  return dt == RTC_I32 ? 4 : (dt == RTC_I64 || dt == RTC_F64) ? 8 : 0;
}

// Tropical product launchers (tropical.hip).  `op` is RTC_OP_CONV, _DECONV, _MAXCONV or _MINDECONV.
// `cap` (optional, dense [batch][n]) fuses out = min(out, cap) into the store, which is how
// the greedy-processing-component step applies its final min with beta^u.
// With `census` (device, RTC_CENSUS_COUNTS words) the call classifies and prepares the rows exactly
// as the product would and then, instead of computing it, adds to census[] how much of the
// iteration space each arithmetic flavour would take (rtc_product_census); `out` is not touched.
int launch_tropical(int op, const void* f, const void* g, void* out, int64_t batch, int64_t n,
                    int64_t stride_f, int64_t stride_g, int dt, const void* cap, void* ws,
                    size_t ws_bytes, int32_t* dev_flags, hipStream_t stream,
                    unsigned long long* census = nullptr);
size_t tropical_workspace_bytes(int64_t batch, int64_t n, int dt);
// Per-row selector codes of the products' convexity test (RTC_STRUCTURE_*), see rtc_product_structure.
int launch_structure_probe(int op, const void* f, const void* g, int32_t* codes, int32_t* periods, int64_t batch,
                           int64_t n, int64_t stride_f, int64_t stride_g, int dt, hipStream_t stream);
int launch_selftest_half_minmax(uint32_t* mismatches, hipStream_t stream);
// Planner knobs: process-wide, atomic so that a call in one host thread may read them while
// another thread sets them (each launch decision reads them once).
extern std::atomic<double> g_packed_min_work;  // see rtc_set_packed_min_work
extern std::atomic<int64_t> g_packed_small_n;  // see rtc_set_packed_small_n
extern std::atomic<bool> g_structure_paths;    // see rtc_set_structure_paths
extern std::atomic<int64_t> g_small_items;     // see rtc_set_small_problem_items
extern std::atomic<int> g_rebase_wide;         // see rtc_set_rebase_wide

// HBM-bound curve kernels (curve_ops.hip).
int launch_pseudo_inverse(const void* f, int64_t n, const void* x, int64_t m, int32_t* out,
                          int64_t batch, int mode, int dt, hipStream_t stream);
int launch_compose(const void* outer, int64_t n_outer, const int32_t* inner, int64_t n, void* out,
                   int64_t batch, int dt, int32_t* dev_flags, hipStream_t stream);
// Remaining service of a component and, with gamma and at least one of ev_lo / ev_up, its
// event-domain images (lower / upper pseudo-inverse of gamma at the result) in the same kernel.
// scratch (optional): batch * ceil(n / 4096) elements of dtype dt for the segment totals of rows
// that are cut over several workgroups; without it every row is one workgroup's.
int launch_residual_service(const void* beta, const void* alpha, void* out, int64_t batch,
                            int64_t n, int dt, bool suffix_min, hipStream_t stream, void* scratch,
                            const void* gamma = nullptr, int64_t n_gamma = 0, int32_t* ev_lo = nullptr,
                            int32_t* ev_up = nullptr);
int launch_closure_init(const void* f, void* out, int64_t batch, int64_t n, int dt, bool super,
                        int32_t* dev_flags, hipStream_t stream);
int launch_copy(const void* src, void* dst, int64_t count, int dt, hipStream_t stream);
// out_v (optional, [batch] of dtype dt): the maximal vertical deviation from the same pass
int launch_max_hdev(const void* alpha, const void* beta, int32_t* out, int64_t batch, int64_t n,
                    int dt, int32_t* dev_flags, hipStream_t stream, void* out_v = nullptr);
int launch_validate_monotone(const void* f, int64_t batch, int64_t n, int64_t stride, int dt, int32_t* first_bad,
                             int32_t* dev_flags, hipStream_t stream);
int launch_max_vdev(const void* alpha, const void* beta, void* out, int64_t batch, int64_t n, int dt,
                    hipStream_t stream);

// Optional kernel timing (profile.hip).  kind = RTC_PROFILE_KIND(dtype, packed, product).
// `gated`: the launch sits behind a per-row selector and may find no row of its kind; such
// launches are recorded only by rtc_profile_enable(2) (the two event records cost about 10 us of
// idle stream each, which a benchmark step should not pay for kernels that do nothing).
void prof_begin(int kind, hipStream_t stream, bool gated = false);
void prof_end(hipStream_t stream);

// Kernel launches go through launch_checked, which takes the launch's OWN return code (the
// thread's sticky "last error" may belong to some other library's earlier call, and reading it
// would both blame a good launch and swallow that error).  A failed launch is remembered per host
// thread until hip_ok() reports it.  Arguments are converted to the kernel's parameter types
// here, as a direct call would convert them.
// An entry point first walks its whole launch sequence in a dry run (validated(), below): nothing
// is launched, every launch's grid is checked against what the runtime accepts, and a grid that
// does not fit turns into RTC_ERR_SHAPE before the first kernel of the call is enqueued.  HIP
// takes grid x block as a 32-bit number of threads: a product of 2^32 is refused and a larger one
// wraps around silently, so the limit is grid * block < 2^32 (67 108 863 workgroups of 64
// threads, 4 194 303 of 1024).
extern thread_local bool t_launch_failed;
extern thread_local bool t_dry_run;
extern thread_local bool t_dry_bad;

inline bool grid_fits(dim3 grid, dim3 block) {
  return grid.x >= 1 && grid.y == 1 && grid.z == 1 && (uint64_t)grid.x * block.x * block.y * block.z < (1ull << 32);
}
// Guard for host code that computes a grid in 64 bits before narrowing it.
inline bool blocks_fit(int64_t blocks, int threads) { return blocks >= 1 && blocks * threads < (1ll << 32); }

template <typename... P, typename... A, size_t... I>
inline hipError_t launch_with_tuple(void (*kernel)(P...), dim3 grid, dim3 block, size_t shmem, hipStream_t stream,
                                    std::index_sequence<I...>, A&&... a) {
  std::tuple<P...> params{static_cast<P>(std::forward<A>(a))...};
  void* ptrs[] = {static_cast<void*>(&std::get<I>(params))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, shmem, stream);
}

template <typename... P, typename... A>
inline void launch_checked(void (*kernel)(P...), dim3 grid, dim3 block, size_t shmem, hipStream_t stream, A&&... a) {
  static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
  if (!grid_fits(grid, block)) {          // never hand the runtime a grid it would wrap around
    (t_dry_run ? t_dry_bad : t_launch_failed) = true;
    return;
  }
  if (t_dry_run) return;
  if (launch_with_tuple(kernel, grid, block, shmem, stream, std::index_sequence_for<P...>{}, std::forward<A>(a)...) !=
      hipSuccess)
    t_launch_failed = true;
}
#define RTC_LAUNCH(kernel, grid, block, shmem, stream, ...) ::rtc::launch_checked(kernel, grid, block, shmem, stream, __VA_ARGS__)

// RTC_OK, or RTC_ERR_HIP when a launch of this thread failed since the last call (which clears it).
inline int hip_ok() {
  if (t_dry_run) return RTC_OK;
  const bool failed = t_launch_failed;
  t_launch_failed = false;
  return failed ? RTC_ERR_HIP : RTC_OK;
}

// Runs `sequence` (a callable that enqueues the kernels of one call and returns a status) twice:
// dry first, then for real when every grid of the dry run fitted and it returned RTC_OK.
template <typename F>
inline int validated(F&& sequence) {
  t_dry_run = true;
  t_dry_bad = false;
  const int rc = sequence();
  t_dry_run = false;
  if (rc != RTC_OK) return rc;
  if (t_dry_bad) return RTC_ERR_SHAPE;
  t_launch_failed = false;
  return sequence();
}

}  // namespace rtc
