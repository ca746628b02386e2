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
template <typename T> __device__ __forceinline__ T highest() {
  if constexpr (std::numeric_limits<T>::has_infinity) return __builtin_huge_val();
  else return std::numeric_limits<T>::max();
}

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

// Stages fr[a, a + len) into s_win (len <= WINDOW, uniform) with every load of a thread in flight
// before the first one is waited for.  A loop of "load, store to LDS" is compiled into one round
// trip per iteration: the store waits for its own load.  The barrier in the instruction stream
// between the two phases keeps the compiler from sinking the loads back into the stores' blocks.
// Entries [len, padded) of s_win (padded <= WINDOW, uniform) are set to the largest value of the type.
template <typename T, int THREADS, int WINDOW>
__device__ __forceinline__ void stage_window(const T* __restrict__ fr, int a, int len, T* s_win, int padded = 0) {
  constexpr int K = (WINDOW + THREADS - 1) / THREADS;
  T tmp[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if (k * THREADS < len) {                   // (uniform)
      const int i = k * THREADS + (int)threadIdx.x;
      tmp[k] = fr[a + (i < len ? i : len - 1)];
    }
  }
  asm volatile("" ::: "memory");
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int i = k * THREADS + (int)threadIdx.x;
    if (i < len) s_win[i] = tmp[k];
    else if (i < padded) s_win[i] = highest<T>();
  }
}

// The search of one kind of count (search_window, MODE 0 and 1) wants the window padded with the
// largest value up to one entry short of the power of two above its length: then no probe needs
// a bounds check.  padded_length(len) is that length; it fits the window for len < WINDOW.
__device__ __forceinline__ int pow2_above(int len) { return len > 0 ? 2 << (31 - __builtin_clz(len)) : 1; }
__device__ __forceinline__ int padded_length(int len) { return pow2_above(len) - 1; }

// ---- searching the staged window ---------------------------------------------------------------
// A binary search per query over the whole window is a chain of log2(len) dependent LDS reads,
// one query after the other.  Instead the searches of a thread's queries run side by side and
// without branches (the range is the same for all lanes, so all searches take the same steps),
// and when both kinds of count are asked for the wavefront first brackets its queries -- they are
// neighbours, consecutive samples of a curve, so their answers lie close together -- with two
// 64-ary searches for its smallest and largest one (each lane probes one position per round: two
// rounds for up to 4096 samples).  Nothing here assumes that the queries are sorted: the bracket
// comes from a minimum and a maximum.

// first index in [lo, hi) whose sample is > x (GT) or >= x, hi if there is none, for a wave-uniform x
// and a wave-uniform range, by all 64 lanes together
template <typename T, bool GT>
__device__ __forceinline__ int wave_first_beyond(const T* s_win, int lo, int hi, T x) {
  return lo + wave_first_true(hi - lo, [&](int k) { const T w = s_win[lo + k]; return GT ? w > x : w >= x; });
}

// Counts of the window's samples below (c_lo; MODE 0 and 2) and not above (c_up; MODE 1 and 2)
// each query; wmin / wmax: smallest and largest query of the calling wavefront (wave-uniform).
template <typename T, int PER, int MODE>
__device__ __forceinline__ void search_window(const T* s_win, int len, const T (&xv)[PER], T wmin, T wmax,
                                              int (&c_lo)[PER], int (&c_up)[PER]) {
  if constexpr (MODE != 2) {
    // One kind of count (the brackets cost about what they save there: measured on rows of 16384
    // and 65536 samples, 4- and 8-byte values).  The searches of a thread's queries run side by
    // side, without branches: the window's length is the same for all, so every search takes the
    // same steps -- largest count `at` with sample at - 1 not beyond the query, found one bit
    // of `at` at a time from the top -- and the LDS reads of the PER queries are in flight together.
    // The window is padded (padded_length) with the largest value, which is beyond every query
    // (or equal to it and counted, for a query that is that value: hence the min at the end), so
    // a step is an add, a read, a compare and a select; counts are kept as byte offsets.
    constexpr int kBytes = (int)sizeof(T);
    int at[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) at[e] = 0;
    for (int step = pow2_above(len) * (kBytes / 2); step >= kBytes; step >>= 1) {   // (uniform)
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const int probe = at[e] + step;
        const T w = *reinterpret_cast<const T*>(reinterpret_cast<const char*>(s_win) + probe - kBytes);
        const bool below = MODE == 0 ? w < xv[e] : !(w > xv[e]);
        at[e] = below ? probe : at[e];
      }
    }
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int c = min((int)((unsigned)at[e] / (unsigned)kBytes), len);
      if (MODE == 0) c_lo[e] = c; else c_up[e] = c;
    }
    return;
  }
  // both kinds: the wavefront's bracket first, then all 2 PER searches of a thread side by side
  // inside it, as above
  const int L = wave_first_beyond<T, false>(s_win, 0, len, wmin);     // samples below every query of the wave
  const int H = wave_first_beyond<T, true>(s_win, L, len, wmax);      // samples not above its largest query
  const int span = H - L;
  int lo[PER], up[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) { lo[e] = 0; up[e] = 0; }
  for (int step = span > 0 ? 1 << (31 - __builtin_clz(span)) : 0; step > 0; step >>= 1) {   // (wave-uniform)
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int pl = lo[e] + step, pu = up[e] + step;
      const T wl = s_win[L + min(pl, span) - 1], wu = s_win[L + min(pu, span) - 1];
      lo[e] = pl <= span && wl < xv[e] ? pl : lo[e];
      up[e] = pu <= span && !(wu > xv[e]) ? pu : up[e];
    }
  }
#pragma unroll
  for (int e = 0; e < PER; ++e) { c_lo[e] = L + lo[e]; c_up[e] = L + up[e]; }
}

// Smallest and largest query of the calling wavefront (in all its lanes) and, through s_mm and one
// barrier, of the workgroup.
template <typename T, int THREADS, int PER>
__device__ __forceinline__ void query_range(const T (&xv)[PER], T (*s_mm)[THREADS / 64], T& wmin, T& wmax, T& xmin, T& xmax) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  wmin = xv[0]; wmax = xv[0];
#pragma unroll
  for (int e = 1; e < PER; ++e) { wmin = xv[e] < wmin ? xv[e] : wmin; wmax = vmax(wmax, xv[e]); }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const T a = __shfl_xor(wmin, off), b = __shfl_xor(wmax, off);
    wmin = a < wmin ? a : wmin; wmax = vmax(wmax, b);
  }
  if (lane == 0) { s_mm[0][wave] = wmin; s_mm[1][wave] = wmax; }
  __syncthreads();
  xmin = wmin; xmax = wmax;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) { xmin = s_mm[0][w] < xmin ? s_mm[0][w] : xmin; xmax = vmax(xmax, s_mm[1][w]); }
}

// Counts of the samples of fr[0, n) below (cnt_lo; MODE 0 and 2) and not above (cnt_up; MODE 1 and
// 2) each of the calling workgroup's queries xv[], for every thread, whether its queries are real
// or repeats of a real one.  With a = the number of samples below the smallest query (not above
// it, when only the upper counts are asked for) and b = the number of samples not above the
// largest one (below it, when only the lower counts are), the stretch fr[a, b) holds every sample
// the counts depend on: count = a + (count inside the stretch).  Two wavefronts find a and b in
// three round trips each; a stretch longer than WINDOW (queries that are not clustered) falls back
// to the plain search per thread.  THREADS threads (a multiple of 64, at least 128), PER queries
// per thread; s_win: WINDOW values of LDS.  Ends with a barrier: the arrays may be reused at once.
// (a_out, b_out, xmax_out: a, b and the largest query, for callers that go on from there.)
template <typename T, int THREADS, int PER, int WINDOW, int MODE>
__device__ __forceinline__ void exact_windowed_counts(const T* __restrict__ fr, int n, const T (&xv)[PER], T* s_win,
                                                      int (&cnt_lo)[PER], int (&cnt_up)[PER], int& a_out, int& b_out,
                                                      T& xmax_out) {
  __shared__ T s_mm[2][THREADS / 64];
  __shared__ int s_ab[2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  T wmin, wmax, xmin, xmax;
  query_range<T, THREADS, PER>(xv, s_mm, wmin, wmax, xmin, xmax);
  xmax_out = xmax;
  if (wave < 2) {
    const T q = wave == 0 ? xmin : xmax;
    const bool upper = wave == 0 ? MODE == 1 : MODE != 0;
    const int at = wave_first_true(n, [&](int k) { return beyond(fr[k], q, upper); });
    if (lane == 0) s_ab[wave] = at;
  }
  __syncthreads();
  const int a = s_ab[0], len = s_ab[1] - a;
  a_out = a; b_out = s_ab[1];
  if (MODE == 2 ? len <= WINDOW : len < WINDOW) {   // (uniform; len >= 0: the predicates are nested)
    stage_window<T, THREADS, WINDOW>(fr, a, len, s_win, MODE == 2 ? 0 : padded_length(len));
    __syncthreads();
    search_window<T, PER, MODE>(s_win, len, xv, wmin, wmax, cnt_lo, cnt_up);
#pragma unroll
    for (int e = 0; e < PER; ++e) { cnt_lo[e] += a; cnt_up[e] += a; }
  } else {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (MODE != 1) cnt_lo[e] = lower_index(fr, n, xv[e]);
      if (MODE != 0) cnt_up[e] = upper_index(fr, n, xv[e]) + 1;
    }
  }
  __syncthreads();
}

template <typename T, int THREADS, int PER, int WINDOW, int MODE>
__device__ __forceinline__ void exact_windowed_counts(const T* __restrict__ fr, int n, const T (&xv)[PER], T* s_win,
                                                      int (&cnt_lo)[PER], int (&cnt_up)[PER]) {
  int a, b;
  T xmax;
  exact_windowed_counts<T, THREADS, PER, WINDOW, MODE>(fr, n, xv, s_win, cnt_lo, cnt_up, a, b, xmax);
}

// ---- a workgroup that takes one block of queries after the other -------------------------------
// Lower counts (samples of fr below each query) for a workgroup whose blocks of queries follow
// each other along a curve.  The block before left b = the number of samples below its largest
// query.  If no query of this block is smaller than that one, every sample before b lies below all of
// them, so the window may start at b without any search; how far it must reach is guessed from the
// length of the last one, and the guess is checked against the window's own last sample (nothing
// beyond a sample that is >= the largest query is counted by any of them).  The window's loads
// then travel together with the loads of the queries: one round trip per block instead of the
// three of the 64-ary searches and the one of the staging after them.  A block that does not fit
// (a smaller query, a window too short) takes the exact path, as does the first.
template <typename T> struct ChainState {
  int b = -1;        // samples below the largest query of the block before; < 0: nothing known yet
  int len = 0;       // length of its stretch
  T xmax = T();      // its largest query
};

template <typename T, int THREADS, int PER, int WINDOW>
__device__ __forceinline__ void chained_lower_counts(const T* __restrict__ fr, int n, const T (&xv)[PER], T* s_win,
                                                     int (&cnt)[PER], ChainState<T>& st) {
  __shared__ T s_mm[2][THREADS / 64];
  __shared__ int s_b;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int unused[PER];
  if (st.b >= 0) {                                                   // (uniform, as all of st)
    const int a = st.b;
    const int len = min(min(WINDOW - 1, n - a), max(THREADS, st.len + (st.len >> 1)));
    stage_window<T, THREADS, WINDOW>(fr, a, len, s_win, padded_length(len));
    T wmin, wmax, xmin, xmax;
    query_range<T, THREADS, PER>(xv, s_mm, wmin, wmax, xmin, xmax);   // (its barrier also puts the window's writes before the reads below)
    const bool fits = !(xmin < st.xmax) && (a + len >= n || !(s_win[len - 1] < xmax));
    if (fits) {
      search_window<T, PER, 0>(s_win, len, xv, wmin, wmax, cnt, unused);
#pragma unroll
      for (int e = 0; e < PER; ++e) cnt[e] += a;
      if (wave == 0) {
        const int b = a + wave_first_beyond<T, false>(s_win, 0, len, xmax);
        if (lane == 0) s_b = b;
      }
      __syncthreads();
      st.len = s_b - a; st.b = s_b; st.xmax = xmax;
      return;      // (s_b is written again only behind the next block's barrier)
    }
    __syncthreads();                                                 // the window is staged again below
  }
  exact_windowed_counts<T, THREADS, PER, WINDOW, 0>(fr, n, xv, s_win, cnt, unused, st.len, st.b, st.xmax);
  st.len = st.b - st.len;                                            // (a came back in st.len)
}

// ---- the same, with the window located in ONE round trip ------------------------------------
// The 64-ary searches above cost three dependent round trips before the window can be staged.
// Instead every thread fetches one sample of a coarse table of the row, the last sample of each of
// THREADS granules of G = ceil(n / THREADS) samples -- positions that do not depend on the queries,
// so the loads travel together with the loads of the queries themselves (and hit in L2: every
// workgroup of a row asks for the same ones; a caller that has the table as one contiguous piece
// passes its entry instead).  With glo = the first granule whose last sample is >= the smallest
// query (> it, for the upper counts alone) and ghi = the first granule whose last sample is > the
// largest query (>= it, for the lower counts alone), every sample before granule glo lies below
// all queries and every sample after granule ghi beyond all of them, so the stretch
// [glo G, (ghi + 1) G) holds all that the counts depend on: at most two granules more than the
// exact stretch.  A stretch longer than the window falls back to the exact searches.
template <int THREADS> __device__ __forceinline__ int coarse_granule(int n) { return (n + THREADS - 1) / THREADS; }

// Position in the row of entry e of its coarse table.
template <int THREADS> __device__ __forceinline__ int coarse_position(int n, int e) {
  const int64_t at = (int64_t)(e + 1) * coarse_granule<THREADS>(n);
  return (at < n ? (int)at : n) - 1;
}

// s_coarse: THREADS values of LDS.  Ends with a barrier.
template <typename T, int THREADS, int PER, int WINDOW, int MODE>
__device__ __forceinline__ void coarse_windowed_counts(const T* __restrict__ fr, int n, const T (&xv)[PER], T coarse,
                                                       T* s_win, T* s_coarse, int (&cnt_lo)[PER], int (&cnt_up)[PER]) {
  constexpr int NW = THREADS / 64;
  __shared__ T s_mm[2][NW];
  const int lane = threadIdx.x & 63;
  s_coarse[threadIdx.x] = coarse;
  T wmin, wmax, xmin, xmax;
  query_range<T, THREADS, PER>(xv, s_mm, wmin, wmax, xmin, xmax);      // (its barrier also covers s_coarse)
  // the table is nondecreasing: the first granule beyond a query is the number of granules that are not
  int glo = 0, ghi = 0;
#pragma unroll
  for (int e = 0; e < NW; ++e) {
    const T c = s_coarse[e * 64 + lane];
    glo += __builtin_popcountll(__ballot(MODE == 1 ? !(c > xmin) : !(c >= xmin)));
    ghi += __builtin_popcountll(__ballot(MODE == 0 ? !(c >= xmax) : !(c > xmax)));
  }
  const int G = coarse_granule<THREADS>(n);
  const int64_t a64 = (int64_t)glo * G, b64 = (int64_t)(ghi + 1) * G;
  const int a = a64 < n ? (int)a64 : n, len = (b64 < n ? (int)b64 : n) - a;
  if (MODE == 2 ? len <= WINDOW : len < WINDOW) {   // (uniform; len >= 0 because ghi >= glo)
    stage_window<T, THREADS, WINDOW>(fr, a, len, s_win, MODE == 2 ? 0 : padded_length(len));
    __syncthreads();
    search_window<T, PER, MODE>(s_win, len, xv, wmin, wmax, cnt_lo, cnt_up);
#pragma unroll
    for (int e = 0; e < PER; ++e) { cnt_lo[e] += a; cnt_up[e] += a; }
    __syncthreads();
  } else {
    exact_windowed_counts<T, THREADS, PER, WINDOW, MODE>(fr, n, xv, s_win, cnt_lo, cnt_up);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void pinv_kernel(const T* __restrict__ f, int n,
                                                   const T* __restrict__ x, int m,
                                                   int32_t* __restrict__ out, int blocks_per_row,
                                                   int mode) {
  __shared__ T s_buf[kSearchWindow + 1];       // (one entry in front: the search reads entry `count - 1` at a non-negative offset)
  T* s_win = s_buf + 1;
  const int row = blockIdx.x / blocks_per_row;
  const int base = (blockIdx.x % blocks_per_row) * kSearchPerBlock + (int)threadIdx.x;
  const T* fr = f + (int64_t)row * n;
  const bool upper = mode != RTC_INV_LOWER;
  T xv[kSearchPerThread];
#pragma unroll
  for (int e = 0; e < kSearchPerThread; ++e)      // past the end: the last query again
    xv[e] = x[(int64_t)row * m + min(base + e * 256, m - 1)];
  int cnt[kSearchPerThread], unused[kSearchPerThread];
  if (upper) exact_windowed_counts<T, 256, kSearchPerThread, kSearchWindow, 1>(fr, n, xv, s_win, unused, cnt);
  else exact_windowed_counts<T, 256, kSearchPerThread, kSearchWindow, 0>(fr, n, xv, s_win, cnt, unused);
#pragma unroll
  for (int e = 0; e < kSearchPerThread; ++e) {
    if (base + e * 256 < m) out[(int64_t)row * m + base + e * 256] = upper ? cnt[e] - 1 : cnt[e];
  }
}

// Four elements per thread, a block of 256 apart: the index loads of all four travel together,
// then the four gathers.
constexpr int kComposePerThread = 4;
constexpr int kComposePerBlock = 256 * kComposePerThread;

template <typename T>
__global__ __launch_bounds__(256) void compose_kernel(const T* __restrict__ outer, int n_outer,
                                                      const int32_t* __restrict__ inner, int n,
                                                      T* __restrict__ out, int blocks_per_row,
                                                      int32_t* __restrict__ dev_flags) {
  const int row = blockIdx.x / blocks_per_row;
  const int d0 = (blockIdx.x % blocks_per_row) * kComposePerBlock + threadIdx.x;
  const int32_t* in = inner + (int64_t)row * n;
  const T* o = outer + (int64_t)row * n_outer;
  int k[kComposePerThread];
#pragma unroll
  for (int e = 0; e < kComposePerThread; ++e) k[e] = in[min(d0 + e * 256, n - 1)];   // past the end: the last index again
  bool clamped = false;
  T v[kComposePerThread];
#pragma unroll
  for (int e = 0; e < kComposePerThread; ++e) {
    const bool real = d0 + e * 256 < n;
    if (k[e] < 0) { k[e] = 0; clamped |= real; }
    if (k[e] > n_outer - 1) { k[e] = n_outer - 1; clamped |= real; }
    v[e] = o[k[e]];
  }
#pragma unroll
  for (int e = 0; e < kComposePerThread; ++e)
    if (d0 + e * 256 < n) out[(int64_t)row * n + d0 + e * 256] = v[e];
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
// and, with EVENTS, the event-domain images of the values while they are still in registers:
//   ev_lo / ev_up (each optional) = lower / upper pseudo-inverse of gamma at out[D].
// A row is cut into `parts` segments of seg positions (in scan order; seg a multiple of the
// kScanPass positions one pass covers), one workgroup each.  What a segment needs from the ones
// before it is one number, the maximum (minimum) of their differences: segment_extrema_kernel
// reduces every segment but the last of each row first (a second read of the operands; no
// workgroup ever waits for another), and a scanning workgroup folds the totals before its own
// segment into its carry.  The values of a pass are monotone in scan order, so their answers fall
// into one stretch of gamma, which is staged once for both inverses.
constexpr int kScanThreads = 256;
constexpr int kScanPer = 4;                                  // consecutive positions per thread
constexpr int kScanPass = kScanThreads * kScanPer;           // positions per pass
constexpr int kExtremaPerThread = 8;
constexpr int kExtremaTrip = 256 * kExtremaPerThread;

// With gamma, the row's workgroups also gather the coarse table of gamma (see coarse_windowed_counts:
// kScanThreads samples, fetched here once per row so that the scanning workgroups read them as one
// contiguous piece) into coarse_tab[row][kScanThreads].
template <typename T, bool SUFFIX>
__global__ __launch_bounds__(256) void segment_extrema_kernel(const T* __restrict__ beta, const T* __restrict__ alpha,
                                                              T* __restrict__ seg_tot, int n, int parts, int seg,
                                                              const T* __restrict__ gamma, int n_gamma,
                                                              T* __restrict__ coarse_tab) {
  using S = ScanOp<T, SUFFIX>;
  __shared__ T red[4];
  const int row = blockIdx.x / (parts - 1), part = blockIdx.x % (parts - 1);
  if (gamma != nullptr) {
    const T* gr = gamma + (int64_t)row * n_gamma;
    for (int e = part * 256 + threadIdx.x; e < kScanThreads; e += (parts - 1) * 256)
      coarse_tab[(int64_t)row * kScanThreads + e] = gr[coarse_position<kScanThreads>(n_gamma, e)];
  }
  const int start = part * seg;                      // < n: the launcher's parts are all non-empty
  const int last = min(n, start + seg) - 1;
  const T* bl = beta + (int64_t)row * n;
  const T* au = alpha + (int64_t)row * n;
  T acc = S::id();
  for (int base = start + threadIdx.x; base <= last; base += kExtremaTrip) {
    T bv[kExtremaPerThread], av[kExtremaPerThread];
#pragma unroll
    for (int e = 0; e < kExtremaPerThread; ++e) {    // past the end: the last position again
      const int p = min(base + e * 256, last);
      const int i = SUFFIX ? n - 1 - p : p;
      bv[e] = bl[i];
      av[e] = au[i];
    }
#pragma unroll
    for (int e = 0; e < kExtremaPerThread; ++e) acc = S::op(acc, (T)(bv[e] - av[e]));
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc = S::op(acc, __shfl_xor(acc, off));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) seg_tot[(int64_t)row * parts + part] = S::op(S::op(red[0], red[1]), S::op(red[2], red[3]));
}

// Carry into segment `part` of a row: the totals of the segments before it, reduced by every
// wavefront for itself (no barrier; a handful of values unless the row has millions of samples).
template <typename T, bool SUFFIX>
__device__ __forceinline__ T carry_before(const T* __restrict__ seg_tot, int row, int parts, int part) {
  using S = ScanOp<T, SUFFIX>;
  T acc = S::id();
  const T* tot = seg_tot + (int64_t)row * parts;
  for (int j = threadIdx.x & 63; j < part; j += 64) acc = S::op(acc, tot[j]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc = S::op(acc, __shfl_xor(acc, off));
  return acc;
}

template <typename T, bool SUFFIX, bool EVENTS>
__global__ __launch_bounds__(kScanThreads) void residual_service_kernel(const T* __restrict__ beta, const T* __restrict__ alpha,
                                                                        T* __restrict__ out, int n, int parts, int seg,
                                                                        const T* __restrict__ seg_tot,
                                                                        const T* __restrict__ gamma, int n_gamma,
                                                                        int32_t* __restrict__ ev_lo, int32_t* __restrict__ ev_up,
                                                                        const T* __restrict__ coarse_tab) {
  using S = ScanOp<T, SUFFIX>;
  constexpr int NW = kScanThreads / 64;
  __shared__ T s_win[EVENTS ? kSearchWindow : 1];
  __shared__ T s_coarse[EVENTS ? kScanThreads : 1];
  __shared__ T wave_tot[NW];
  __shared__ T carry_s;
  const int row = blockIdx.x / parts, part = blockIdx.x % parts;
  const int start = part * seg;
  if (start >= n) return;
  const int end = min(n, start + seg);
  const T* bl = beta + (int64_t)row * n;
  const T* au = alpha + (int64_t)row * n;
  T* o = out + (int64_t)row * n;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // The differences of one pass, loaded one pass ahead of their use.  Every load is issued
  // whatever the position (one past the row's end reads the last sample), so that all loads of
  // a pass travel together: a load under its own condition is waited for on the spot.
  auto load = [&](int base, T (&d)[kScanPer]) {
    T bv[kScanPer], av[kScanPer];
#pragma unroll
    for (int e = 0; e < kScanPer; ++e) {
      const int p = min(base + (int)threadIdx.x * kScanPer + e, n - 1);
      const int i = SUFFIX ? n - 1 - p : p;
      bv[e] = bl[i];
      av[e] = au[i];
    }
#pragma unroll
    for (int e = 0; e < kScanPer; ++e) {
      // the difference may be negative; inputs obey the no-overflow precondition
      d[e] = base + (int)threadIdx.x * kScanPer + e < n ? (T)(bv[e] - av[e]) : S::id();
    }
  };
  T next[kScanPer];
  load(start, next);
  // the thread's entry of the row's coarse table of gamma (the same for every pass): from the table
  // that segment_extrema_kernel has gathered, else from the row itself
  T coarse = (T)0;
  const T* gr = nullptr;
  if constexpr (EVENTS) {
    gr = gamma + (int64_t)row * n_gamma;
    coarse = coarse_tab != nullptr ? coarse_tab[(int64_t)row * kScanThreads + threadIdx.x]
                                   : gr[coarse_position<kScanThreads>(n_gamma, threadIdx.x)];
  }
  T carry = part > 0 ? carry_before<T, SUFFIX>(seg_tot, row, parts, part) : S::id();
  for (int base = start; base < end; base += kScanPass) {
    const int p0 = base + threadIdx.x * kScanPer;   // position in scan order
    T v[kScanPer];
    T run = S::id();
#pragma unroll
    for (int e = 0; e < kScanPer; ++e) {
      run = S::op(run, next[e]);
      v[e] = run;
    }
    if (base + kScanPass < end) load(base + kScanPass, next);
    const T incl = wave_scan<T, SUFFIX>(run);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    T before = carry;
    for (int w = 0; w < wave; ++w) before = S::op(before, wave_tot[w]);
    // exclusive prefix inside the wave = inclusive value of the previous lane
    T prev = __shfl_up(incl, 1);
    if (lane == 0) prev = S::id();
    before = S::op(before, prev);
    // a position past the row's end repeats the value before it (its difference is the scan's
    // identity), i.e. a real query, which is what the windowed search asks for
    T q[kScanPer];
#pragma unroll
    for (int e = 0; e < kScanPer; ++e) {
      const T r = S::op(before, v[e]);
      q[e] = r > (T)0 ? r : (T)0;
      const int p = p0 + e;
      if (p < n) o[SUFFIX ? n - 1 - p : p] = q[e];
    }
    if (threadIdx.x == kScanThreads - 1) carry_s = S::op(before, run);
    if constexpr (EVENTS) {
      int cnt_lo[kScanPer], cnt_up[kScanPer];
      coarse_windowed_counts<T, kScanThreads, kScanPer, kSearchWindow, 2>(gr, n_gamma, q, coarse, s_win, s_coarse, cnt_lo,
                                                                           cnt_up);   // (has barriers)
#pragma unroll
      for (int e = 0; e < kScanPer; ++e) {
        const int p = p0 + e;
        if (p < n) {
          const int64_t at = (int64_t)row * n + (SUFFIX ? n - 1 - p : p);
          if (ev_lo != nullptr) ev_lo[at] = cnt_lo[e];
          if (ev_up != nullptr) ev_up[at] = cnt_up[e] - 1;
        }
      }
    } else {
      __syncthreads();
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

// Maximal horizontal deviation: each thread searches beta for a few alpha[D]; a workgroup takes
// `trips` consecutive blocks of kDevPerBlock samples of one row, one after the other, and merges
// into out[row] (pre-set to 0) with one atomic max at the end (atomics on one address are served
// one after the other, so a row should not see many more of them than it takes to fill the chip).
// With out_v (optional; pre-set to the lowest value) the same pass also takes the maximal vertical
// deviation of its samples, alpha[D] - beta[D]: delay and backlog bound from one read of alpha.
template <typename T>
__global__ __launch_bounds__(256) void hdev_kernel(const T* __restrict__ alpha,
                                                   const T* __restrict__ beta, int32_t* __restrict__ out,
                                                   int n, int parts, int trips,
                                                   int32_t* __restrict__ dev_flags, T* __restrict__ out_v) {
  static_assert(kDevPerThread == kSearchPerThread, "the deviation kernels search kSearchPerThread samples per thread");
  __shared__ T s_buf[kSearchWindow + 1];       // (one entry in front: the search reads entry `count - 1` at a non-negative offset)
  T* s_win = s_buf + 1;
  __shared__ int32_t red[4];
  __shared__ int32_t unb[4];
  __shared__ T redv[4];
  const int row = blockIdx.x / parts;
  const int first = (blockIdx.x % parts) * trips * kDevPerBlock;
  if (first >= n) return;
  const T* a = alpha + (int64_t)row * n;
  const T* b = beta + (int64_t)row * n;
  T vmaxdev = lowest<T>();
  int32_t h = 0;
  bool unbounded = false;
  ChainState<T> chain;
  for (int trip = 0; trip < trips; ++trip) {
    const int base = first + trip * kDevPerBlock + (int)threadIdx.x;
    if (first + trip * kDevPerBlock >= n) break;                                       // (uniform)
    T xv[kSearchPerThread];
#pragma unroll
    for (int e = 0; e < kDevPerThread; ++e) xv[e] = a[min(base + e * 256, n - 1)];   // past the end: the last sample again
    if (out_v != nullptr) {
      T bv[kDevPerThread];
#pragma unroll
      for (int e = 0; e < kDevPerThread; ++e) bv[e] = b[min(base + e * 256, n - 1)];
#pragma unroll
      for (int e = 0; e < kDevPerThread; ++e) vmaxdev = vmax(vmaxdev, (T)(xv[e] - bv[e]));   // (a repeated last sample changes no maximum)
    }
    int cnt[kSearchPerThread];
    chained_lower_counts<T, 256, kSearchPerThread, kSearchWindow>(b, n, xv, s_win, cnt, chain);   // (ends with a barrier)
#pragma unroll
    for (int e = 0; e < kDevPerThread; ++e) {
      const int d = base + e * 256;
      if (d < n) {
        const int k = cnt[e];
        unbounded |= (k == n);
        h = max(h, k - d);
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) h = max(h, __shfl_xor(h, off));
  if (out_v != nullptr) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) vmaxdev = vmax(vmaxdev, __shfl_xor(vmaxdev, off));
  }
  const bool any_unb = __any(unbounded);
  if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6] = h; unb[threadIdx.x >> 6] = any_unb; redv[threadIdx.x >> 6] = vmaxdev; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int32_t m = max(max(red[0], red[1]), max(red[2], red[3]));
    if (m > 0) atomicMax(&out[row], m);
    if (dev_flags != nullptr && (unb[0] | unb[1] | unb[2] | unb[3])) atomicOr(dev_flags, RTC_FLAG_UNBOUNDED);
    if (out_v != nullptr) atomic_max_any(&out_v[row], vmax(vmax(redv[0], redv[1]), vmax(redv[2], redv[3])));
  }
}

// Maximal vertical deviation, out[row] pre-set to the lowest value.  `parts` workgroups per row, each
// over a segment of seg samples (a multiple of the 2048 one trip covers): as many workgroups as keep
// every CU busy and no more, because each ends in one atomic on its row's result and atomics on one
// address are served one after the other.  Eight loads per operand and thread are in flight per trip
// (a position past the segment's end reads its last sample again, which changes no maximum).
constexpr int kVdevPerThread = 8;
constexpr int kVdevTrip = 256 * kVdevPerThread;

template <typename T>
__global__ __launch_bounds__(256) void vdev_kernel(const T* __restrict__ alpha,
                                                   const T* __restrict__ beta, T* __restrict__ out, int n,
                                                   int parts, int seg) {
  __shared__ T red[4];
  const int row = blockIdx.x / parts;
  const int start = (blockIdx.x % parts) * seg;
  if (start >= n) return;
  const int last = min(n, start + seg) - 1;
  const T* a = alpha + (int64_t)row * n;
  const T* b = beta + (int64_t)row * n;
  T m = lowest<T>();
  for (int base = start + threadIdx.x; base <= last; base += kVdevTrip) {
    T av[kVdevPerThread], bv[kVdevPerThread];
#pragma unroll
    for (int e = 0; e < kVdevPerThread; ++e) {
      const int d = min(base + e * 256, last);
      av[e] = a[d];
      bv[e] = b[d];
    }
#pragma unroll
    for (int e = 0; e < kVdevPerThread; ++e) m = vmax(m, (T)(av[e] - bv[e]));
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
  const int64_t bpr = (n + kComposePerBlock - 1) / kComposePerBlock;
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
                            int64_t n, int dt, bool suffix_min, hipStream_t stream, void* scratch, const void* gamma,
                            int64_t n_gamma, int32_t* ev_lo, int32_t* ev_up) {
  // One workgroup per row, passing over it 1024 positions at a time, moves the fewest bytes; but the
  // passes of a row are then taken one after the other.  Once the rows alone give every CU its
  // eight workgroups, that is the better trade; below that every segment of one pass gets its own
  // workgroup, which costs one more read of both operands (segment_extrema_kernel) and no waiting.
  const bool events = gamma != nullptr && (ev_lo != nullptr || ev_up != nullptr);
  const int64_t passes = (n + kScanPass - 1) / kScanPass;
  // (the scratch holds n elements per row; a row's totals and its coarse table of gamma must fit)
  const int64_t parts = (batch >= 2048 || scratch == nullptr || passes + kScanThreads > n) ? 1 : passes;
  const int64_t seg = parts == 1 ? passes * kScanPass : kScanPass;
  if (batch * parts > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_DISPATCH(dt, {
    T* tot = static_cast<T*>(scratch);              // [batch][parts], then [batch][kScanThreads]
    T* tab = parts > 1 && events ? tot + batch * parts : nullptr;
    const T* gam = events ? static_cast<const T*>(gamma) : nullptr;
    const T* b = static_cast<const T*>(beta);
    const T* a = static_cast<const T*>(alpha);
    T* o = static_cast<T*>(out);
    const dim3 grid((uint32_t)(batch * parts));
    const dim3 block(kScanThreads);
    prof_begin(RTC_PROFILE_KIND_TAIL, stream);      // (both launches: the totals belong to the scan)
    if (parts > 1) {
      const dim3 grid1((uint32_t)(batch * (parts - 1)));
      if (suffix_min)
        RTC_LAUNCH((segment_extrema_kernel<T, true>), grid1, dim3(256), 0, stream, b, a, tot, (int)n, (int)parts, (int)seg,
                   gam, (int)n_gamma, tab);
      else
        RTC_LAUNCH((segment_extrema_kernel<T, false>), grid1, dim3(256), 0, stream, b, a, tot, (int)n, (int)parts, (int)seg,
                   gam, (int)n_gamma, tab);
    }
    if (events) {
      if (suffix_min)
        RTC_LAUNCH((residual_service_kernel<T, true, true>), grid, block, 0, stream, b, a, o, (int)n, (int)parts, (int)seg,
                   tot, gam, (int)n_gamma, ev_lo, ev_up, tab);
      else
        RTC_LAUNCH((residual_service_kernel<T, false, true>), grid, block, 0, stream, b, a, o, (int)n, (int)parts, (int)seg,
                   tot, gam, (int)n_gamma, ev_lo, ev_up, tab);
    } else if (suffix_min) {
      RTC_LAUNCH((residual_service_kernel<T, true, false>), grid, block, 0, stream, b, a, o, (int)n, (int)parts, (int)seg,
                 tot, gam, 0, nullptr, nullptr, tab);
    } else {
      RTC_LAUNCH((residual_service_kernel<T, false, false>), grid, block, 0, stream, b, a, o, (int)n, (int)parts, (int)seg,
                 tot, gam, 0, nullptr, nullptr, tab);
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
  // about 2048 workgroups in all (8 per CU) where the rows are long enough for that
  const int64_t bpr = (n + kDevPerBlock - 1) / kDevPerBlock;
  int64_t parts = (2048 + batch - 1) / batch;
  if (parts < 32) parts = 32;                    // (up to 32 atomics per row cost nothing measurable)
  if (parts > bpr) parts = bpr;
  const int64_t trips = (bpr + parts - 1) / parts;
  parts = (bpr + trips - 1) / trips;
  if (parts * batch > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_DISPATCH(dt, {
    RTC_LAUNCH(init2_kernel<T>, dim3((uint32_t)((batch + 255) / 256)), dim3(256), 0, stream, out,
                       static_cast<T*>(out_v), (int)batch, std::numeric_limits<T>::has_infinity
                           ? (T)-std::numeric_limits<T>::infinity() : std::numeric_limits<T>::lowest());
    RTC_LAUNCH(hdev_kernel<T>, dim3((uint32_t)(parts * batch)), dim3(256), 0, stream,
                       static_cast<const T*>(alpha), static_cast<const T*>(beta), out, (int)n, (int)parts, (int)trips,
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
  // about 2048 workgroups in all (8 per CU), at least one trip each
  const int64_t trips = (n + kVdevTrip - 1) / kVdevTrip;
  int64_t parts = (2048 + batch - 1) / batch;
  if (parts > trips) parts = trips;
  const int64_t seg = (trips + parts - 1) / parts * kVdevTrip;
  parts = (n + seg - 1) / seg;
  if (parts * batch > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_DISPATCH(dt, {
    RTC_LAUNCH(init_kernel<T>, dim3((uint32_t)((batch + 255) / 256)), dim3(256), 0, stream,
                       static_cast<T*>(out), (int)batch, std::numeric_limits<T>::has_infinity
                           ? (T)-std::numeric_limits<T>::infinity() : std::numeric_limits<T>::lowest());
    RTC_LAUNCH(vdev_kernel<T>, dim3((uint32_t)(parts * batch)), dim3(256), 0, stream,
                       static_cast<const T*>(alpha), static_cast<const T*>(beta), static_cast<T*>(out),
                       (int)n, (int)parts, (int)seg);
    return hip_ok();
  });
}

}  // namespace rtc
