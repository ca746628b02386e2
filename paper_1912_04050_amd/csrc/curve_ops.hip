// HBM-bound curve kernels: pseudo-inverse (search), composition (gather), residual
// service (subtract + prefix-max scan + clamp), horizontal / vertical deviation (search or
// subtract + max-reduce).  One pass over the data each; none of them is arithmetic-bound.
#include <hip/hip_runtime.h>

#include <limits>

#include "rtc_internal.h"

namespace rtc {
namespace {

template <typename T> __device__ __forceinline__ T vmax(T a, T b) { return b > a ? b : a; }

template <typename T> __device__ __forceinline__ T lowest() {
  if constexpr (std::numeric_limits<T>::has_infinity) return -__builtin_huge_val();
  else return std::numeric_limits<T>::lowest();
}

// Lower pseudo-inverse: first index with f[k] >= x (n if none).  f nondecreasing.
template <typename T>
__device__ __forceinline__ int lower_index(const T* __restrict__ f, int n, T x) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (f[mid] >= x) hi = mid; else lo = mid + 1;
  }
  return lo;
}

// Upper pseudo-inverse: last index with f[k] <= x (-1 if none).
template <typename T>
__device__ __forceinline__ int upper_index(const T* __restrict__ f, int n, T x) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (f[mid] <= x) lo = mid + 1; else hi = mid;
  }
  return lo - 1;
}

// ---- searches of a whole workgroup's queries through a window of the curve in LDS ----------
// A binary search in HBM / L2 is a chain of ~log2(n) dependent loads.  The queries of one
// workgroup (consecutive samples of another curve) mostly fall into a short stretch of f, so:
// the wavefronts 0 and 1 locate the answers of the smallest and of the largest query with a
// 64-ary search (three dependent loads for n = 65536), the stretch between them is staged in
// LDS, and every query is searched there.  A stretch longer than the window (queries that are
// not clustered) falls back to the plain search per thread.  Both give the answer of the plain
// search for every nondecreasing f.
constexpr int kSearchWindow = 2048;    // samples of f staged per workgroup
constexpr int kSearchPerThread = 4;    // queries per thread
constexpr int kSearchPerBlock = 256 * kSearchPerThread;

// Whether f[k] lies beyond the query: LOWER counts the samples < x (the first index with
// f[k] >= x is their number), UPPER the samples <= x (the last index with f[k] <= x is their
// number - 1).
template <typename T> __device__ __forceinline__ bool beyond(T fk, T x, bool upper) { return upper ? fk > x : fk >= x; }

// First index in [0, n) at which pred turns true (n if it never does); pred nondecreasing in
// the index.  All 64 lanes of the wavefront take part: each round probes 64 evenly spaced
// positions and keeps the stretch between the last false and the first true one.
template <typename Pred>
__device__ __forceinline__ int wave_first_true(int n, Pred pred) {
  const int lane = threadIdx.x & 63;
  int lo = 0, hi = n;
  while (hi > lo) {
    const int width = hi - lo, step = (width + 63) >> 6;
    const int p = lo + min((lane + 1) * step, width) - 1;
    const uint64_t b = __ballot(pred(p));
    if (b == 0) { lo = hi; break; }
    const int first = __builtin_ctzll(b);
    hi = lo + min((first + 1) * step, width) - 1;
    lo = lo + first * step;
  }
  return lo;
}

// Number of samples of fr[0, n) not beyond each of the calling workgroup's (256 threads)
// queries xv[0 .. kSearchPerThread), in cnt[]: for every thread, whether its queries are real
// or repeats of a real one.  s_win: kSearchWindow values of LDS.
template <typename T>
__device__ __forceinline__ void windowed_counts(const T* __restrict__ fr, int n, const T (&xv)[kSearchPerThread],
                                                bool upper, T* s_win, int (&cnt)[kSearchPerThread]) {
  __shared__ T s_mm[2][4];
  __shared__ int s_ab[2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  T xmin = xv[0], xmax = xv[0];
#pragma unroll
  for (int e = 1; e < kSearchPerThread; ++e) { xmin = xv[e] < xmin ? xv[e] : xmin; xmax = vmax(xmax, xv[e]); }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const T a = __shfl_xor(xmin, off), b = __shfl_xor(xmax, off);
    xmin = a < xmin ? a : xmin; xmax = vmax(xmax, b);
  }
  if (lane == 0) { s_mm[0][wave] = xmin; s_mm[1][wave] = xmax; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < 4; ++w) { xmin = s_mm[0][w] < xmin ? s_mm[0][w] : xmin; xmax = vmax(xmax, s_mm[1][w]); }
  if (wave < 2) {
    const T q = wave == 0 ? xmin : xmax;
    const int at = wave_first_true(n, [&](int k) { return beyond(fr[k], q, upper); });
    if (lane == 0) s_ab[wave] = at;
  }
  __syncthreads();
  const int a = s_ab[0], len = s_ab[1] - a;
  if (len >= 0 && len <= kSearchWindow) {
#pragma unroll 4
    for (int i = threadIdx.x; i < len; i += 256) s_win[i] = fr[a + i];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kSearchPerThread; ++e) {
      int lo = 0, hi = len;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (beyond(s_win[mid], xv[e], upper)) hi = mid; else lo = mid + 1;
      }
      cnt[e] = a + lo;
    }
  } else {
#pragma unroll
    for (int e = 0; e < kSearchPerThread; ++e) cnt[e] = upper ? upper_index(fr, n, xv[e]) + 1 : lower_index(fr, n, xv[e]);
  }
}

// Both pseudo-inverses of a workgroup's queries from ONE staged window: with a = the number of
// samples below the smallest query and b = the number of samples not above the largest one, the
// stretch fr[a, b) holds every sample that lies inside the queries' range, so for each query
//   lower count (samples <  x) = a + (samples of the window <  x)
//   upper count (samples <= x) = a + (samples of the window <= x).
// THREADS threads (a multiple of 64, at most 1024), PER queries per thread, WINDOW samples of LDS
// in s_win; a longer stretch falls back to the plain searches per thread.
template <typename T, int THREADS, int PER, int WINDOW>
__device__ __forceinline__ void windowed_counts_both(const T* __restrict__ fr, int n, const T (&xv)[PER], T* s_win,
                                                     int (&cnt_lo)[PER], int (&cnt_up)[PER]) {
  constexpr int NW = THREADS / 64;
  __shared__ T s_mm[2][NW];
  __shared__ int s_ab[2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  T xmin = xv[0], xmax = xv[0];
#pragma unroll
  for (int e = 1; e < PER; ++e) { xmin = xv[e] < xmin ? xv[e] : xmin; xmax = vmax(xmax, xv[e]); }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const T a = __shfl_xor(xmin, off), b = __shfl_xor(xmax, off);
    xmin = a < xmin ? a : xmin; xmax = vmax(xmax, b);
  }
  if (lane == 0) { s_mm[0][wave] = xmin; s_mm[1][wave] = xmax; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < NW; ++w) { xmin = s_mm[0][w] < xmin ? s_mm[0][w] : xmin; xmax = vmax(xmax, s_mm[1][w]); }
  if (wave < 2) {
    const T q = wave == 0 ? xmin : xmax;
    const bool upper = wave == 1;
    const int at = wave_first_true(n, [&](int k) { return beyond(fr[k], q, upper); });
    if (lane == 0) s_ab[wave] = at;
  }
  __syncthreads();
  const int a = s_ab[0], len = s_ab[1] - a;
  if (len >= 0 && len <= WINDOW) {
#pragma unroll 4
    for (int i = threadIdx.x; i < len; i += THREADS) s_win[i] = fr[a + i];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      int lo = 0, hi = len;
      while (lo < hi) {                       // samples < x
        const int mid = (lo + hi) >> 1;
        if (s_win[mid] >= xv[e]) hi = mid; else lo = mid + 1;
      }
      cnt_lo[e] = a + lo;
      hi = len;                               // samples <= x: from the first one >= x on
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (s_win[mid] > xv[e]) hi = mid; else lo = mid + 1;
      }
      cnt_up[e] = a + lo;
    }
  } else {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      cnt_lo[e] = lower_index(fr, n, xv[e]);
      cnt_up[e] = upper_index(fr, n, xv[e]) + 1;
    }
  }
  __syncthreads();   // s_win and the small arrays may be reused by the caller's next pass
}

template <typename T>
__global__ __launch_bounds__(256) void pinv_kernel(const T* __restrict__ f, int n,
                                                   const T* __restrict__ x, int m,
                                                   int32_t* __restrict__ out, int blocks_per_row,
                                                   int mode) {
  __shared__ T s_win[kSearchWindow];
  const int row = blockIdx.x / blocks_per_row;
  const int base = (blockIdx.x % blocks_per_row) * kSearchPerBlock;
  const T* fr = f + (int64_t)row * n;
  const bool upper = mode != RTC_INV_LOWER;
  T xv[kSearchPerThread];
#pragma unroll
  for (int e = 0; e < kSearchPerThread; ++e)      // past the end: the last query again
    xv[e] = x[(int64_t)row * m + min(base + e * 256 + (int)threadIdx.x, m - 1)];
  int cnt[kSearchPerThread];
  windowed_counts(fr, n, xv, upper, s_win, cnt);
#pragma unroll
  for (int e = 0; e < kSearchPerThread; ++e) {
    const int j = base + e * 256 + threadIdx.x;
    if (j < m) out[(int64_t)row * m + j] = upper ? cnt[e] - 1 : cnt[e];
  }
}

template <typename T>
__global__ __launch_bounds__(256) void compose_kernel(const T* __restrict__ outer, int n_outer,
                                                      const int32_t* __restrict__ inner, int n,
                                                      T* __restrict__ out, int blocks_per_row,
                                                      int32_t* __restrict__ dev_flags) {
  const int row = blockIdx.x / blocks_per_row;
  const int d = (blockIdx.x % blocks_per_row) * 256 + threadIdx.x;
  bool clamped = false;
  if (d < n) {
    int k = inner[(int64_t)row * n + d];
    if (k < 0) { k = 0; clamped = true; }
    if (k > n_outer - 1) { k = n_outer - 1; clamped = true; }
    out[(int64_t)row * n + d] = outer[(int64_t)row * n_outer + k];
  }
  if (dev_flags != nullptr && __any(clamped)) {
    if ((threadIdx.x & 63) == 0) atomicOr(dev_flags, RTC_FLAG_DOMAIN);
  }
}

// ---- wave-level inclusive max-scan with DPP row shifts and row broadcasts ----------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int32_t dpp_move(int32_t identity, int32_t v) {
  return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int64_t dpp_move(int64_t identity, int64_t v) {
  const int32_t lo = __builtin_amdgcn_update_dpp((int32_t)identity, (int32_t)v, CTRL, ROW_MASK, 0xf, false);
  const int32_t hi = __builtin_amdgcn_update_dpp((int32_t)(identity >> 32), (int32_t)(v >> 32), CTRL, ROW_MASK, 0xf, false);
  return ((int64_t)hi << 32) | (uint32_t)lo;
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_move(double identity, double v) {
  return __longlong_as_double(dpp_move<CTRL, ROW_MASK>((int64_t)__double_as_longlong(identity),
                                                       (int64_t)__double_as_longlong(v)));
}

template <typename T> __device__ __forceinline__ T vmin(T a, T b) { return b < a ? b : a; }

template <typename T> __device__ __forceinline__ T highest() {
  if constexpr (std::numeric_limits<T>::has_infinity) return __builtin_huge_val();
  else return std::numeric_limits<T>::max();
}

// The two scans of a greedy processing component share one kernel:
//   MIN = false: running maximum over increasing index (identity: lowest)
//   MIN = true : running minimum (identity: highest); the kernel then walks the row backwards,
//                which turns it into the suffix minimum.
template <typename T, bool MIN> struct ScanOp {
  static __device__ __forceinline__ T id() { return MIN ? highest<T>() : lowest<T>(); }
  static __device__ __forceinline__ T op(T a, T b) { return MIN ? vmin(a, b) : vmax(a, b); }
};

template <typename T, bool MIN>
__device__ __forceinline__ T wave_scan(T v) {
  using S = ScanOp<T, MIN>;
  const T id = S::id();
  v = S::op(v, dpp_move<0x111, 0xf>(id, v));  // row_shr:1
  v = S::op(v, dpp_move<0x112, 0xf>(id, v));  // row_shr:2
  v = S::op(v, dpp_move<0x114, 0xf>(id, v));  // row_shr:4
  v = S::op(v, dpp_move<0x118, 0xf>(id, v));  // row_shr:8
  v = S::op(v, dpp_move<0x142, 0xa>(id, v));  // row_bcast:15 into rows 1 and 3
  v = S::op(v, dpp_move<0x143, 0xc>(id, v));  // row_bcast:31 into rows 2 and 3
  return v;
}

// Remaining service of a greedy processing component:
//   SUFFIX = false: out[D] = max(0, max_{l<=D} beta[l] - alpha[l])   (beta^l, alpha^u -> beta'^l)
//   SUFFIX = true : out[D] = max(0, min_{l>=D} beta[l] - alpha[l])   (beta^u, alpha^l -> beta'^u)
// `parts` workgroups per row (few rows would otherwise leave most CUs idle): each scans one segment
// of the row in scan order, after reducing everything before its segment itself (maximum and
// minimum are exact and order-free, so the extra reads cost time only, and no workgroup waits for
// another).  seg = segment length, a multiple of the 4096 positions one pass covers.
template <typename T, bool SUFFIX>
__global__ __launch_bounds__(1024) void residual_service_kernel(const T* __restrict__ beta,
                                                                const T* __restrict__ alpha,
                                                                T* __restrict__ out, int n, int parts, int seg) {
  using S = ScanOp<T, SUFFIX>;
  constexpr int kPer = 4;
  __shared__ T wave_tot[16];
  __shared__ T carry_s;
  const int row = blockIdx.x / parts, part = blockIdx.x % parts;
  const int start = part * seg;
  if (start >= n) return;
  const int end = min(n, start + seg);
  const T* bl = beta + (int64_t)row * n;
  const T* au = alpha + (int64_t)row * n;
  T* o = out + (int64_t)row * n;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  T carry = S::id();
  if (start > 0) {
    // everything before the segment; the loads of eight passes are independent and in flight together
    T acc = S::id();
#pragma unroll 8
    for (int p = threadIdx.x; p < start; p += 1024) {
      const int i = SUFFIX ? n - 1 - p : p;
      acc = S::op(acc, (T)(bl[i] - au[i]));
    }
    const T incl = wave_scan<T, SUFFIX>(acc);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 16; ++w) carry = S::op(carry, wave_tot[w]);
    __syncthreads();
  }
  // the differences of one pass, loaded one pass ahead of their use
  auto load = [&](int base, T (&d)[kPer]) {
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const int p = base + threadIdx.x * kPer + e;
      const int i = SUFFIX ? n - 1 - p : p;
      // the difference may be negative; inputs obey the no-overflow precondition
      d[e] = p < n ? (T)(bl[i] - au[i]) : S::id();
    }
  };
  T next[kPer];
  load(start, next);
  for (int base = start; base < end; base += 1024 * kPer) {
    const int p0 = base + threadIdx.x * kPer;   // position in scan order
    T v[kPer];
    T run = S::id();
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      run = S::op(run, next[e]);
      v[e] = run;
    }
    if (base + 1024 * kPer < end) load(base + 1024 * kPer, next);
    const T incl = wave_scan<T, SUFFIX>(run);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    T before = carry;
    for (int w = 0; w < wave; ++w) before = S::op(before, wave_tot[w]);
    // exclusive prefix inside the wave = inclusive value of the previous lane
    T prev = __shfl_up(incl, 1);
    if (lane == 0) prev = S::id();
    before = S::op(before, prev);
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const int p = p0 + e;
      if (p < n) {
        const T r = S::op(before, v[e]);
        o[SUFFIX ? n - 1 - p : p] = r > (T)0 ? r : (T)0;
      }
    }
    if (threadIdx.x == 1023) carry_s = S::op(before, run);
    __syncthreads();
    carry = carry_s;
  }
}

// The tail of a greedy processing component in one kernel: the remaining service as in
// residual_service_kernel, and the event-domain images of the values while they are still in
// registers -- ev_lo / ev_up (each optional) = lower / upper pseudo-inverse of gamma at out[D].
// The values of a pass are monotone in scan order, so their answers fall into one stretch of
// gamma, which windowed_counts_both stages once for both inverses: gamma and out are read resp.
// written once instead of twice and three times.
template <typename T> constexpr int tail_window() { return sizeof(T) == 8 ? 6144 : 8192; }

template <typename T, bool SUFFIX>
__global__ __launch_bounds__(1024) void gpc_tail_kernel(const T* __restrict__ beta, const T* __restrict__ alpha,
                                                        T* __restrict__ out, int n, int parts, int seg,
                                                        const T* __restrict__ gamma, int n_gamma,
                                                        int32_t* __restrict__ ev_lo, int32_t* __restrict__ ev_up) {
  using S = ScanOp<T, SUFFIX>;
  constexpr int kPer = 4;
  __shared__ T s_win[tail_window<T>()];
  __shared__ T wave_tot[16];
  __shared__ T carry_s;
  const int row = blockIdx.x / parts, part = blockIdx.x % parts;
  const int start = part * seg;
  if (start >= n) return;
  const int end = min(n, start + seg);
  const T* bl = beta + (int64_t)row * n;
  const T* au = alpha + (int64_t)row * n;
  const T* gr = gamma + (int64_t)row * n_gamma;
  T* o = out + (int64_t)row * n;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  T carry = S::id();
  if (start > 0) {
    T acc = S::id();
#pragma unroll 8
    for (int p = threadIdx.x; p < start; p += 1024) {
      const int i = SUFFIX ? n - 1 - p : p;
      acc = S::op(acc, (T)(bl[i] - au[i]));
    }
    const T incl = wave_scan<T, SUFFIX>(acc);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 16; ++w) carry = S::op(carry, wave_tot[w]);
    __syncthreads();
  }
  auto load = [&](int base, T (&d)[kPer]) {
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const int p = base + threadIdx.x * kPer + e;
      const int i = SUFFIX ? n - 1 - p : p;
      d[e] = p < n ? (T)(bl[i] - au[i]) : S::id();
    }
  };
  T next[kPer];
  load(start, next);
  for (int base = start; base < end; base += 1024 * kPer) {
    const int p0 = base + threadIdx.x * kPer;   // position in scan order
    T v[kPer];
    T run = S::id();
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      run = S::op(run, next[e]);
      v[e] = run;
    }
    if (base + 1024 * kPer < end) load(base + 1024 * kPer, next);
    const T incl = wave_scan<T, SUFFIX>(run);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    T before = carry;
    for (int w = 0; w < wave; ++w) before = S::op(before, wave_tot[w]);
    T prev = __shfl_up(incl, 1);
    if (lane == 0) prev = S::id();
    before = S::op(before, prev);
    // a position past the row's end repeats the value before it (its difference is the scan's
    // identity), i.e. a real query, which is what the windowed search asks for
    T q[kPer];
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const T r = S::op(before, v[e]);
      q[e] = r > (T)0 ? r : (T)0;
      const int p = p0 + e;
      if (p < n) o[SUFFIX ? n - 1 - p : p] = q[e];
    }
    if (threadIdx.x == 1023) carry_s = S::op(before, run);
    int cnt_lo[kPer], cnt_up[kPer];
    windowed_counts_both<T, 1024, kPer, tail_window<T>()>(gr, n_gamma, q, s_win, cnt_lo, cnt_up);   // (has barriers)
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const int p = p0 + e;
      if (p < n) {
        const int64_t at = (int64_t)row * n + (SUFFIX ? n - 1 - p : p);
        if (ev_lo != nullptr) ev_lo[at] = cnt_lo[e];
        if (ev_up != nullptr) ev_up[at] = cnt_up[e] - 1;
      }
    }
    carry = carry_s;
  }
}

__device__ __forceinline__ void atomic_max_any(int32_t* p, int32_t v) { atomicMax(p, v); }
__device__ __forceinline__ void atomic_max_any(int64_t* p, int64_t v) { atomicMax((long long*)p, (long long)v); }
__device__ __forceinline__ void atomic_max_any(double* p, double v) { atomicMax(p, v); }

template <typename T>
__global__ __launch_bounds__(256) void init_kernel(T* __restrict__ dst, int count, T value) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < count) dst[i] = value;
}

// h[i] = 0 and (v optional) v[i] = value for i < count: the starting values of the deviation kernels' atomic maxima
template <typename T>
__global__ __launch_bounds__(256) void init2_kernel(int32_t* __restrict__ h, T* __restrict__ v, int count, T value) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < count) {
    h[i] = 0;
    if (v != nullptr) v[i] = value;
  }
}

constexpr int kDevPerThread = 4;   // alpha samples per thread in the deviation kernels
constexpr int kDevPerBlock = 256 * kDevPerThread;

// Maximal horizontal deviation: each thread searches beta for a few alpha[D]; a workgroup
// covers kDevPerBlock consecutive D of one row and merges into out[row] (pre-set to 0) with
// an atomic max.
// With out_v (optional; pre-set to the lowest value) the same pass also takes the maximal vertical
// deviation of its samples, alpha[D] - beta[D]: delay and backlog bound from one read of alpha.
template <typename T>
__global__ __launch_bounds__(256) void hdev_kernel(const T* __restrict__ alpha,
                                                   const T* __restrict__ beta, int32_t* __restrict__ out,
                                                   int n, int blocks_per_row,
                                                   int32_t* __restrict__ dev_flags, T* __restrict__ out_v) {
  static_assert(kDevPerThread == kSearchPerThread, "the deviation kernels search kSearchPerThread samples per thread");
  __shared__ T s_win[kSearchWindow];
  __shared__ int32_t red[4];
  __shared__ int32_t unb[4];
  __shared__ T redv[4];
  const int row = blockIdx.x / blocks_per_row;
  const int base = (blockIdx.x % blocks_per_row) * kDevPerBlock;
  const T* a = alpha + (int64_t)row * n;
  const T* b = beta + (int64_t)row * n;
  T xv[kSearchPerThread];
#pragma unroll
  for (int e = 0; e < kDevPerThread; ++e) xv[e] = a[min(base + e * 256 + (int)threadIdx.x, n - 1)];   // past the end: the last sample again
  T vmaxdev = lowest<T>();
  if (out_v != nullptr) {
#pragma unroll
    for (int e = 0; e < kDevPerThread; ++e)     // (a repeated last sample changes no maximum)
      vmaxdev = vmax(vmaxdev, (T)(xv[e] - b[min(base + e * 256 + (int)threadIdx.x, n - 1)]));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) vmaxdev = vmax(vmaxdev, __shfl_xor(vmaxdev, off));
    if ((threadIdx.x & 63) == 0) redv[threadIdx.x >> 6] = vmaxdev;    // read after the barriers of the search below
  }
  int cnt[kSearchPerThread];
  windowed_counts(b, n, xv, false, s_win, cnt);
  int32_t h = 0;
  bool unbounded = false;
#pragma unroll
  for (int e = 0; e < kDevPerThread; ++e) {
    const int d = base + e * 256 + threadIdx.x;
    if (d < n) {
      const int k = cnt[e];
      unbounded |= (k == n);
      h = max(h, k - d);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) h = max(h, __shfl_xor(h, off));
  const bool any_unb = __any(unbounded);
  if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6] = h; unb[threadIdx.x >> 6] = any_unb; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int32_t m = max(max(red[0], red[1]), max(red[2], red[3]));
    if (m > 0) atomicMax(&out[row], m);
    if (dev_flags != nullptr && (unb[0] | unb[1] | unb[2] | unb[3])) atomicOr(dev_flags, RTC_FLAG_UNBOUNDED);
    if (out_v != nullptr) atomic_max_any(&out_v[row], vmax(vmax(redv[0], redv[1]), vmax(redv[2], redv[3])));
  }
}

// Maximal vertical deviation; same decomposition, out[row] pre-set to the lowest value.
template <typename T>
__global__ __launch_bounds__(256) void vdev_kernel(const T* __restrict__ alpha,
                                                   const T* __restrict__ beta, T* __restrict__ out, int n,
                                                   int blocks_per_row) {
  __shared__ T red[4];
  const int row = blockIdx.x / blocks_per_row;
  const int base = (blockIdx.x % blocks_per_row) * kDevPerBlock;
  const T* a = alpha + (int64_t)row * n;
  const T* b = beta + (int64_t)row * n;
  T m = lowest<T>();
#pragma unroll
  for (int e = 0; e < kDevPerThread; ++e) {
    const int d = base + e * 256 + threadIdx.x;
    if (d < n) m = vmax(m, (T)(a[d] - b[d]));
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = vmax(m, __shfl_xor(m, off));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) atomic_max_any(&out[row], vmax(vmax(red[0], red[1]), vmax(red[2], red[3])));
}

// Start of a closure iteration: out = f with out[0] forced to 0 (the value the unit element
// delta_0 contributes).  A row whose f[0] has the wrong sign (below 0 for the sub-additive,
// above 0 for the super-additive closure) has no finite closure: flag it.
template <typename T>
__global__ __launch_bounds__(256) void closure_init_kernel(const T* __restrict__ f, T* __restrict__ out, int n,
                                                           int blocks_per_row, bool super,
                                                           int32_t* __restrict__ dev_flags) {
  const int row = blockIdx.x / blocks_per_row;
  const int i = (blockIdx.x % blocks_per_row) * 256 + threadIdx.x;
  if (i >= n) return;
  T v = f[(int64_t)row * n + i];
  if (i == 0) {
    if (dev_flags != nullptr && (super ? v > (T)0 : v < (T)0)) atomicOr(dev_flags, RTC_FLAG_DOMAIN);
    v = (T)0;
  }
  out[(int64_t)row * n + i] = v;
}

template <typename T>
__global__ __launch_bounds__(256) void copy_kernel(const T* __restrict__ src, T* __restrict__ dst, int64_t count) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * 256;
  for (; i < count; i += step) dst[i] = src[i];
}

template <typename T>
int pinv_typed(const void* f, int64_t n, const void* x, int64_t m, int32_t* out, int64_t batch, int mode,
               hipStream_t stream) {
  const int64_t bpr = (m + kSearchPerBlock - 1) / kSearchPerBlock;
  if (bpr * batch > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_LAUNCH(pinv_kernel<T>, dim3((uint32_t)(bpr * batch)), dim3(256), 0, stream,
                     static_cast<const T*>(f), (int)n, static_cast<const T*>(x), (int)m, out, (int)bpr, mode);
  return hip_ok();
}

template <typename T>
int compose_typed(const void* outer, int64_t n_outer, const int32_t* inner, int64_t n, void* out,
                  int64_t batch, int32_t* dev_flags, hipStream_t stream) {
  const int64_t bpr = (n + 255) / 256;
  if (bpr * batch > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_LAUNCH(compose_kernel<T>, dim3((uint32_t)(bpr * batch)), dim3(256), 0, stream,
                     static_cast<const T*>(outer), (int)n_outer, inner, (int)n, static_cast<T*>(out),
                     (int)bpr, dev_flags);
  return hip_ok();
}

}  // namespace

#define RTC_DISPATCH(dt, CALL)                    \
  switch (dt) {                                   \
    case RTC_I32: { using T = int32_t; CALL; }    \
    case RTC_I64: { using T = int64_t; CALL; }    \
    case RTC_F64: { using T = double; CALL; }     \
    default: return RTC_ERR_DTYPE;                \
  }

int launch_pseudo_inverse(const void* f, int64_t n, const void* x, int64_t m, int32_t* out,
                          int64_t batch, int mode, int dt, hipStream_t stream) {
  RTC_DISPATCH(dt, return pinv_typed<T>(f, n, x, m, out, batch, mode, stream));
}

int launch_compose(const void* outer, int64_t n_outer, const int32_t* inner, int64_t n, void* out,
                   int64_t batch, int dt, int32_t* dev_flags, hipStream_t stream) {
  RTC_DISPATCH(dt, return compose_typed<T>(outer, n_outer, inner, n, out, batch, dev_flags, stream));
}

int launch_residual_service(const void* beta, const void* alpha, void* out, int64_t batch,
                            int64_t n, int dt, bool suffix_min, hipStream_t stream, const void* gamma,
                            int64_t n_gamma, int32_t* ev_lo, int32_t* ev_up) {
  // Several workgroups per row when the rows alone would not fill the chip.  A workgroup's passes
  // over its segment are bound by latency (about 3.3 us each, measured), the whole launch by its
  // traffic: 3 arrays, plus (parts - 1) more for what the workgroups re-read before their segments
  // (at about 3.5 TB/s).  Take the power of two that minimises the larger of the two.
  const bool events = gamma != nullptr && (ev_lo != nullptr || ev_up != nullptr);
  int64_t parts = 1;
  {
    const double array_bytes = (double)batch * (double)n * (dt == RTC_I32 ? 4.0 : 8.0);
    double best = 1e300;
    for (int64_t p = 1; p <= 16 && (p == 1 || (batch * p <= 512 && n / p >= 8192)); p *= 2) {
      // with the event-domain images a pass also searches (two barriers and a staged window more)
      const double latency_us = (double)((n + p * 4096 - 1) / (p * 4096)) * (events ? 6.0 : 3.3);
      const double traffic_us = ((events ? 4.0 : 2.0) + (double)p) * array_bytes / 3.5e6;
      const double t = latency_us > traffic_us ? latency_us : traffic_us;
      if (t < best) { best = t; parts = p; }
    }
  }
  const int64_t seg = ((n + parts - 1) / parts + 4095) / 4096 * 4096;
  if (batch * parts > 0x7fffffffLL) return RTC_ERR_SHAPE;
  prof_begin(RTC_PROFILE_KIND_TAIL, stream);
  RTC_DISPATCH(dt, {
    if (events) {
      if (suffix_min)
        RTC_LAUNCH((gpc_tail_kernel<T, true>), dim3((uint32_t)(batch * parts)), dim3(1024), 0, stream,
                           static_cast<const T*>(beta), static_cast<const T*>(alpha), static_cast<T*>(out), (int)n,
                           (int)parts, (int)seg, static_cast<const T*>(gamma), (int)n_gamma, ev_lo, ev_up);
      else
        RTC_LAUNCH((gpc_tail_kernel<T, false>), dim3((uint32_t)(batch * parts)), dim3(1024), 0, stream,
                           static_cast<const T*>(beta), static_cast<const T*>(alpha), static_cast<T*>(out), (int)n,
                           (int)parts, (int)seg, static_cast<const T*>(gamma), (int)n_gamma, ev_lo, ev_up);
    } else if (suffix_min) {
      RTC_LAUNCH((residual_service_kernel<T, true>), dim3((uint32_t)(batch * parts)), dim3(1024), 0, stream,
                         static_cast<const T*>(beta), static_cast<const T*>(alpha), static_cast<T*>(out), (int)n,
                         (int)parts, (int)seg);
    } else {
      RTC_LAUNCH((residual_service_kernel<T, false>), dim3((uint32_t)(batch * parts)), dim3(1024), 0, stream,
                         static_cast<const T*>(beta), static_cast<const T*>(alpha), static_cast<T*>(out), (int)n,
                         (int)parts, (int)seg);
    }
    prof_end(stream);
    return hip_ok();
  });
}

int launch_closure_init(const void* f, void* out, int64_t batch, int64_t n, int dt, bool super,
                        int32_t* dev_flags, hipStream_t stream) {
  const int64_t bpr = (n + 255) / 256;
  if (bpr * batch > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_DISPATCH(dt, {
    RTC_LAUNCH(closure_init_kernel<T>, dim3((uint32_t)(bpr * batch)), dim3(256), 0, stream,
                       static_cast<const T*>(f), static_cast<T*>(out), (int)n, (int)bpr, super, dev_flags);
    return hip_ok();
  });
}

int launch_copy(const void* src, void* dst, int64_t count, int dt, hipStream_t stream) {
  const int64_t want = (count + 2047) / 2048;
  const int blocks = (int)(want < 65535 ? want : 65535);
  RTC_DISPATCH(dt, {
    RTC_LAUNCH(copy_kernel<T>, dim3(blocks), dim3(256), 0, stream, static_cast<const T*>(src),
                       static_cast<T*>(dst), count);
    return hip_ok();
  });
}

int launch_max_hdev(const void* alpha, const void* beta, int32_t* out, int64_t batch, int64_t n,
                    int dt, int32_t* dev_flags, hipStream_t stream, void* out_v) {
  const int64_t bpr = (n + kDevPerBlock - 1) / kDevPerBlock;
  if (bpr * batch > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_DISPATCH(dt, {
    RTC_LAUNCH(init2_kernel<T>, dim3((uint32_t)((batch + 255) / 256)), dim3(256), 0, stream, out,
                       static_cast<T*>(out_v), (int)batch, std::numeric_limits<T>::has_infinity
                           ? (T)-std::numeric_limits<T>::infinity() : std::numeric_limits<T>::lowest());
    RTC_LAUNCH(hdev_kernel<T>, dim3((uint32_t)(bpr * batch)), dim3(256), 0, stream,
                       static_cast<const T*>(alpha), static_cast<const T*>(beta), out, (int)n, (int)bpr,
                       dev_flags, static_cast<T*>(out_v));
    return hip_ok();
  });
}

namespace {
// One workgroup per row: smallest i with f[i+1] < f[i], or -1.
template <typename T>
__global__ __launch_bounds__(256) void validate_monotone_kernel(const T* __restrict__ f, int64_t stride, int n,
                                                                int32_t* __restrict__ first_bad,
                                                                int32_t* __restrict__ dev_flags) {
  __shared__ int red[4];
  const int row = blockIdx.x;
  const T* fr = f + (int64_t)row * stride;
  int bad = 0x7fffffff;
  for (int i = threadIdx.x; i + 1 < n; i += 256)
    if (fr[i + 1] < fr[i]) { bad = i; break; }       // ascending i per thread: its first one
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) bad = min(bad, __shfl_xor(bad, off));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = bad;
  __syncthreads();
  if (threadIdx.x == 0) {
    bad = min(min(red[0], red[1]), min(red[2], red[3]));
    if (first_bad != nullptr) first_bad[row] = bad == 0x7fffffff ? -1 : bad;
    if (bad != 0x7fffffff) atomicOr(dev_flags, RTC_FLAG_NOT_MONOTONE);
  }
}
}  // namespace

int launch_validate_monotone(const void* f, int64_t batch, int64_t n, int64_t stride, int dt, int32_t* first_bad,
                             int32_t* dev_flags, hipStream_t stream) {
  RTC_DISPATCH(dt, {
    RTC_LAUNCH(validate_monotone_kernel<T>, dim3((uint32_t)batch), dim3(256), 0, stream,
                       static_cast<const T*>(f), stride, (int)n, first_bad, dev_flags);
    return hip_ok();
  });
}

int launch_max_vdev(const void* alpha, const void* beta, void* out, int64_t batch, int64_t n, int dt,
                    hipStream_t stream) {
  const int64_t bpr = (n + kDevPerBlock - 1) / kDevPerBlock;
  if (bpr * batch > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_DISPATCH(dt, {
    RTC_LAUNCH(init_kernel<T>, dim3((uint32_t)((batch + 255) / 256)), dim3(256), 0, stream,
                       static_cast<T*>(out), (int)batch, std::numeric_limits<T>::has_infinity
                           ? (T)-std::numeric_limits<T>::infinity() : std::numeric_limits<T>::lowest());
    RTC_LAUNCH(vdev_kernel<T>, dim3((uint32_t)(bpr * batch)), dim3(256), 0, stream,
                       static_cast<const T*>(alpha), static_cast<const T*>(beta), static_cast<T*>(out),
                       (int)n, (int)bpr);
    return hip_ok();
  });
}

}  // namespace rtc
