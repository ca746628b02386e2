// Helper kernels of the tropical products: identity fill, range probes (overflow flag, int64
// re-basing and narrowing, packed-path eligibility and slope), preparation of the packed path's
// tables, and the per-row packability decision.  Included by tropical.hip only.
#pragma once

#include "tropical_common.h"

namespace rtc {
namespace {

template <typename T>
__global__ __launch_bounds__(256) void fill_kernel(T* __restrict__ dst, int64_t count, T value) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += step) dst[i] = value;
}

template <typename T>
__global__ __launch_bounds__(256) void copy_rows_kernel(const T* __restrict__ src, T* __restrict__ dst, int64_t count) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += step) dst[i] = src[i];
}

// Shape bits of a row pair: bit 0 f convex (second differences >= 0), bit 1 f concave, bit 2 g
// convex, bit 3 g concave.  second_diff_bits() looks at sample i of one row (1 <= i <= n-2) and
// returns the bits that survive; differences are taken in int64 (int32 rows: always exact; int64
// rows: exact when the row's range is below 2^62, which the caller checks afterwards).
template <typename T>
__device__ __forceinline__ int second_diff_bits(const T* row, int i) {
  const int64_t a = (int64_t)((uint64_t)(int64_t)row[i + 1] - (uint64_t)(int64_t)row[i]);
  const int64_t b = (int64_t)((uint64_t)(int64_t)row[i] - (uint64_t)(int64_t)row[i - 1]);
  return (a >= b ? 1 : 0) | (a <= b ? 2 : 0);
}

// Selector codes shared by the product kernels: 0 = 64-bit kernel, 1 = 32-bit / packed kernels,
// kSelSearch / kSelEnds = the row pair is done by structured_kernel.
constexpr int kSelSearch = 2;
constexpr int kSelEnds = 3;
constexpr int kSelBracket = 4;          // one operand of the right shape: anchors + brackets, see tropical_structured.h
constexpr int kSelBracketSwapped = 5;   // the same with the convolution's operands exchanged
constexpr int kSelPeriodic = 6;         // g is periodic from index 1 on: scan + short window, see tropical_structured.h
constexpr int kSelPeriodicSwapped = 7;  // the same for f of a convolution

// The candidates of one output, c(j) = f[j] + g[t-j] (convolutions) or f[t+j] - g[j]
// (deconvolutions), form a convex sequence in j when (f, g) are (convex, convex) resp.
// (convex, concave), a concave one when (concave, concave) resp. (concave, convex).  A min over a
// concave sequence / max over a convex one sits at an end of the range; a min over a convex / max
// over a concave one is found by bisection on the sign of c(j+1) - c(j).  Returns the selector
// code for the row pair, or `general` when it has no such structure.
__device__ __forceinline__ int structure_code(int op, int bits, int general) {
  const bool fcvx = bits & 1, fccv = bits & 2, gcvx = bits & 4, gccv = bits & 8;
  const bool cvx = op_sub(op) ? (fcvx && gccv) : (fcvx && gcvx);
  const bool ccv = op_sub(op) ? (fccv && gcvx) : (fccv && gccv);
  if (op_max(op) ? cvx : ccv) return kSelEnds;
  if (op_max(op) ? ccv : cvx) return kSelSearch;
  // One operand alone: the candidate matrix M[t][j] = c_t(j) is a Monge matrix when the operand
  // that is indexed by t (g for the convolutions -- or f, they commute -- and f for the
  // deconvolutions) is convex under a min / concave under a max, whatever the other operand is;
  // the optimal j then moves monotonically with t.
  const bool want_cvx = !op_max(op);
  if (op_sub(op)) return (want_cvx ? fcvx : fccv) ? kSelBracket : general;
  if (want_cvx ? gcvx : gccv) return kSelBracket;
  if (want_cvx ? fcvx : fccv) return kSelBracketSwapped;
  return general;
}

// Range probe of one row pair.  Finds min/max of both rows, raises the overflow flag when
// the bounds do not prove that every candidate fits and (optionally) decides eligibility for
// the packed path and the slope to remove, and (optionally, integers) whether the pair's
// convexity lets structured_kernel do it (selector code in sel[row], else 1; always 1 when
// kProbeGeneralOnly is added to op).
constexpr int kProbeGeneralOnly = 0x100;
template <typename T>
__global__ __launch_bounds__(1024) void probe_kernel(const T* __restrict__ f, int64_t stride_f,
                                                     const T* __restrict__ g, int64_t stride_g, int n,
                                                     int op, int32_t* __restrict__ pack_ok,
                                                     int32_t* __restrict__ rho, int32_t* __restrict__ sel,
                                                     int32_t* __restrict__ dev_flags) {
  __shared__ T red[4][16];
  __shared__ int s_bits[16];
  const bool classify = (op & kProbeGeneralOnly) == 0;
  op &= ~kProbeGeneralOnly;
  const bool deconv = op_sub(op);
  const int row = blockIdx.x;
  const T* fr = f + (int64_t)row * stride_f;
  const T* gr = g + (int64_t)row * stride_g;
  T fmin = Lim<T>::hi(), fmax = Lim<T>::lo(), gmin = Lim<T>::hi(), gmax = Lim<T>::lo();
  int bits = classify ? 15 : 0;
  // four strides per trip, their loads in flight together: with few rows one workgroup walks a long
  // row alone and every trip is a round trip to memory
  for (int i0 = threadIdx.x; i0 < n; i0 += 4 * blockDim.x) {
    T fv[4], gv[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = min(i0 + k * (int)blockDim.x, n - 1);   // a repeated sample changes no extremum
      fv[k] = fr[i]; gv[k] = gr[i];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      fmin = sel_min(fmin, fv[k]); fmax = sel_max(fmax, fv[k]);
      gmin = sel_min(gmin, gv[k]); gmax = sel_max(gmax, gv[k]);
    }
    if constexpr (std::numeric_limits<T>::is_integer) {
      if (sel != nullptr && bits != 0) {
        int b[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int i = min(max(i0 + k * (int)blockDim.x, 1), n - 2);   // interior samples only; needs n >= 3
          b[k] = n >= 3 ? second_diff_bits(fr, i) | (second_diff_bits(gr, i) << 2) : 15;
        }
        bits &= b[0] & b[1] & b[2] & b[3];
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    fmin = sel_min(fmin, __shfl_xor(fmin, off)); fmax = sel_max(fmax, __shfl_xor(fmax, off));
    gmin = sel_min(gmin, __shfl_xor(gmin, off)); gmax = sel_max(gmax, __shfl_xor(gmax, off));
    bits &= __shfl_xor(bits, off);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    red[0][wave] = fmin; red[1][wave] = fmax; red[2][wave] = gmin; red[3][wave] = gmax;
    s_bits[wave] = bits;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int nw = (blockDim.x + 63) >> 6;
    for (int w = 1; w < nw; ++w) {
      fmin = sel_min(fmin, red[0][w]); fmax = sel_max(fmax, red[1][w]);
      gmin = sel_min(gmin, red[2][w]); gmax = sel_max(gmax, red[3][w]);
      bits &= s_bits[w];
    }
    if constexpr (!std::numeric_limits<T>::is_integer) {
      (void)dev_flags;
    } else {
      // int64 rows: the second differences were exact only if both ranges are below 2^62
      if (sizeof(T) == 8 && (((uint64_t)fmax - (uint64_t)fmin) >> 62 || ((uint64_t)gmax - (uint64_t)gmin) >> 62)) bits = 0;
      const int code = sel != nullptr ? structure_code(op, bits, 1) : 1;
      if (sel != nullptr) sel[row] = code;
      T dummy;
      const bool bad = deconv ? (__builtin_sub_overflow(fmax, gmin, &dummy) || __builtin_sub_overflow(fmin, gmax, &dummy))
                              : (__builtin_add_overflow(fmax, gmax, &dummy) || __builtin_add_overflow(fmin, gmin, &dummy));
      if (bad && dev_flags) atomicOr(dev_flags, RTC_FLAG_OVERFLOW);
      if (pack_ok) {
        // |values| < 2^29 keeps the detrended rows inside int32 (rho*i <= g[n-1]-g[0] < 2^30)
        const T lim = (T)1 << 29;
        const bool ok = fmin >= -lim && fmax < lim && gmin >= -lim && gmax < lim;
        pack_ok[row] = ok ? 1 : 0;
        // slope of the window operand: g for the convolution, f for the deconvolution
        const T w0 = deconv ? fr[0] : gr[0], w1 = deconv ? fr[n - 1] : gr[n - 1];
        const T u0 = deconv ? gr[0] : fr[0], u1 = deconv ? gr[n - 1] : fr[n - 1];
        int32_t r = 0;
        if (ok && n > 1) {
          r = w1 > w0 ? (int32_t)((w1 - w0) / (T)(n - 1)) : 0;
          // performance heuristic: when the two average slopes differ so much that not even a
          // sub-chunk of the uniform operand stays inside 16 bits after detrending, do not
          // prepare the row
          const int64_t ru = (int64_t)((u1 - u0) / (T)(n - 1));
          const int64_t diff = ru > r ? ru - r : r - ru;
          if (diff * kPkSub > 50000) pack_ok[row] = 0;
        }
        if (code != 1) pack_ok[row] = 0;   // structured_kernel does the row
        rho[row] = r;
      }
    }
  }
}

// Values of the table probe_partial_kernel leaves per (row, segment).
constexpr int kProbePartial = 9;

// Common slope of a row pair, removed from both rows before they are narrowed to 32 bits: with
// f[i] = Bf + fd[i] + rho i and g[i] = Bg + gd[i] + rho i every candidate of the four products is
// the candidate of (fd, gd) plus (Bf +- Bg) + rho t, so cumulative curves that grow far beyond
// 32 bits but stay close to a line (time in nanoseconds, cycles) still take the 32-bit and packed
// kernels.  Half the sum of the two mean slopes; all of this is exact whenever both rows' ranges
// are below 2^62, which the caller checks once it has the extrema.
__device__ __forceinline__ int64_t common_slope(const int64_t* fr, const int64_t* gr, int n) {
  if (n < 2) return 0;
  return wrap_sub(fr[n - 1], fr[0]) / (n - 1) / 2 + wrap_sub(gr[n - 1], gr[0]) / (n - 1) / 2;
}
// The detrended extrema cost as much again as the plain ones, and a pair of monotone rows whose
// end points are less than 2^30 apart is narrow as it is: only pairs with an end-to-end rise of
// 2^30 or more are looked at (a non-monotone pair that is wide between close end points then
// goes without this remedy).
__device__ __forceinline__ bool worth_detrending(const int64_t* fr, const int64_t* gr, int n) {
  const uint64_t lim = 1ull << 30;
  const int64_t df = wrap_sub(fr[n - 1], fr[0]), dg = wrap_sub(gr[n - 1], gr[0]);
  return (uint64_t)(df < 0 ? -(uint64_t)df : (uint64_t)df) >= lim || (uint64_t)(dg < 0 ? -(uint64_t)dg : (uint64_t)dg) >= lim;
}
__device__ __forceinline__ int64_t detrended(int64_t v, int64_t v0, int64_t slope, int i) {
  return wrap_sub(wrap_sub(v, v0), (int64_t)((uint64_t)slope * (uint64_t)i));
}

// Extrema (plain and, with `lines`, with the common slope removed) and shape bits of the samples
// [i_begin, i_end) of one int64 row pair, for the calling thread's share: four strides of the
// workgroup per trip, their loads in flight together (one stride per trip is one round trip to
// memory per trip).  A stride past the end repeats the segment's last sample, which changes
// neither an extremum nor a shape bit.
__device__ __forceinline__ void probe_samples(const int64_t* __restrict__ fr, const int64_t* __restrict__ gr, int i_begin,
                                              int i_end, int n, bool lines, int64_t f0, int64_t g0, int64_t slope,
                                              int64_t& fmin, int64_t& fmax, int64_t& gmin, int64_t& gmax,
                                              int64_t& dfmin, int64_t& dfmax, int64_t& dgmin, int64_t& dgmax, int& bits) {
  constexpr int kTrip = 4;
  for (int i0 = i_begin + (int)threadIdx.x; i0 < i_end; i0 += kTrip * (int)blockDim.x) {
    int64_t fv[kTrip], gv[kTrip];
#pragma unroll
    for (int k = 0; k < kTrip; ++k) {
      const int i = min(i0 + k * (int)blockDim.x, i_end - 1);
      fv[k] = fr[i]; gv[k] = gr[i];
    }
#pragma unroll
    for (int k = 0; k < kTrip; ++k) {
      fmin = sel_min(fmin, fv[k]); fmax = sel_max(fmax, fv[k]);
      gmin = sel_min(gmin, gv[k]); gmax = sel_max(gmax, gv[k]);
    }
    if (lines) {
#pragma unroll
      for (int k = 0; k < kTrip; ++k) {
        const int i = min(i0 + k * (int)blockDim.x, i_end - 1);
        const int64_t fd = detrended(fv[k], f0, slope, i), gd = detrended(gv[k], g0, slope, i);
        dfmin = sel_min(dfmin, fd); dfmax = sel_max(dfmax, fd);
        dgmin = sel_min(dgmin, gd); dgmax = sel_max(dgmax, gd);
      }
    }
    if (bits != 0 && n >= 3) {
      int b[kTrip];
#pragma unroll
      for (int k = 0; k < kTrip; ++k) {
        const int i = min(max(min(i0 + k * (int)blockDim.x, i_end - 1), 1), n - 2);   // interior samples only
        b[k] = second_diff_bits(fr, i) | (second_diff_bits(gr, i) << 2);
      }
#pragma unroll
      for (int k = 0; k < kTrip; ++k) bits &= b[k];
    }
  }
}

// First half of the range probe of long int64 rows: extrema and shape bits of one segment of
// one row pair, [fmin, fmax, gmin, gmax, bits] at partial[(row * segs + seg) * 5].
__global__ __launch_bounds__(1024) void probe_partial_kernel(const int64_t* __restrict__ f, int64_t stride_f,
                                                             const int64_t* __restrict__ g, int64_t stride_g,
                                                             int n, bool structure, int segs,
                                                             int64_t* __restrict__ partial) {
  __shared__ int64_t red[8][16];
  __shared__ int s_bits[16];
  const int row = blockIdx.x / segs, seg = blockIdx.x % segs;
  const int seg_len = (n + segs - 1) / segs;
  const int i_begin = seg * seg_len, i_end = min(n, i_begin + seg_len);
  const int64_t* fr = f + (int64_t)row * stride_f;
  const int64_t* gr = g + (int64_t)row * stride_g;
  int64_t fmin = INT64_MAX, fmax = INT64_MIN, gmin = INT64_MAX, gmax = INT64_MIN;
  int64_t dfmin = INT64_MAX, dfmax = INT64_MIN, dgmin = INT64_MAX, dgmax = INT64_MIN;   // with the common slope removed
  const bool lines = worth_detrending(fr, gr, n);
  const int64_t f0 = fr[0], g0 = gr[0], slope = lines ? common_slope(fr, gr, n) : 0;   // (64-bit divisions: not for nothing)
  int bits = structure ? 15 : 0;
  probe_samples(fr, gr, i_begin, i_end, n, lines, f0, g0, slope, fmin, fmax, gmin, gmax, dfmin, dfmax, dgmin, dgmax, bits);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    fmin = sel_min(fmin, __shfl_xor(fmin, off)); fmax = sel_max(fmax, __shfl_xor(fmax, off));
    gmin = sel_min(gmin, __shfl_xor(gmin, off)); gmax = sel_max(gmax, __shfl_xor(gmax, off));
    bits &= __shfl_xor(bits, off);
  }
  if (lines) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      dfmin = sel_min(dfmin, __shfl_xor(dfmin, off)); dfmax = sel_max(dfmax, __shfl_xor(dfmax, off));
      dgmin = sel_min(dgmin, __shfl_xor(dgmin, off)); dgmax = sel_max(dgmax, __shfl_xor(dgmax, off));
    }
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    red[0][wave] = fmin; red[1][wave] = fmax; red[2][wave] = gmin; red[3][wave] = gmax;
    if (lines) { red[4][wave] = dfmin; red[5][wave] = dfmax; red[6][wave] = dgmin; red[7][wave] = dgmax; }
    s_bits[wave] = bits;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int nw = (blockDim.x + 63) >> 6;
    for (int w = 1; w < nw; ++w) {
      fmin = sel_min(fmin, red[0][w]); fmax = sel_max(fmax, red[1][w]);
      gmin = sel_min(gmin, red[2][w]); gmax = sel_max(gmax, red[3][w]);
      if (lines) {
        dfmin = sel_min(dfmin, red[4][w]); dfmax = sel_max(dfmax, red[5][w]);
        dgmin = sel_min(dgmin, red[6][w]); dgmax = sel_max(dgmax, red[7][w]);
      }
      bits &= s_bits[w];
    }
    int64_t* q = partial + ((int64_t)row * segs + seg) * kProbePartial;
    q[0] = fmin; q[1] = fmax; q[2] = gmin; q[3] = gmax; q[4] = bits;
    q[5] = dfmin; q[6] = dfmax; q[7] = dgmin; q[8] = dgmax;
  }
}

// Range probe of one int64 row pair.  A row whose two value ranges (max - min) are below 2^30
// is re-based to its minima and copied as int32: every candidate of the re-based rows fits
// 32 bits, so the 32-bit kernels compute it exactly and add `out_base[2 row]` (f_min + g_min,
// or f_min - g_min for the deconvolutions) back on store.  With `detrend`, a pair that is too
// wide for that but narrow once the pair's common slope is removed (common_slope) is copied
// without the slope, and `out_base[2 row + 1]`, the slope, times the output index is added
// back as well.  Rows with a wider range keep the
// 64-bit kernel.  Also: overflow flag, packed-path eligibility and slope, and (when `structure`
// is set) the convexity test, as in probe_kernel; narrow_ok[row] receives the selector code.
__global__ __launch_bounds__(1024) void probe_narrow_kernel(const int64_t* __restrict__ f, int64_t stride_f,
                                                            const int64_t* __restrict__ g, int64_t stride_g,
                                                            int n, int op, bool structure,
                                                            int32_t* __restrict__ f32,
                                                            int32_t* __restrict__ g32,
                                                            int32_t* __restrict__ narrow_ok,
                                                            int64_t* __restrict__ out_base,
                                                            int32_t* __restrict__ pack_ok,
                                                            int32_t* __restrict__ rho,
                                                            int32_t* __restrict__ dev_flags, int segs,
                                                            const int64_t* __restrict__ partial, bool detrend) {
  __shared__ int64_t red[8][16];
  __shared__ int64_t s_base[3];
  __shared__ int s_narrow;
  __shared__ int s_bits[16];
  const bool deconv = op_sub(op);
  // long rows are cut into `segs` segments, one workgroup each: the row's extrema and shape bits
  // then come from probe_partial_kernel's table and every workgroup repeats the (cheap)
  // decision; segment 0 publishes it, every segment copies its own part
  const int row = blockIdx.x / segs, seg = blockIdx.x % segs;
  const int seg_len = (n + segs - 1) / segs;
  const int i_begin = seg * seg_len, i_end = min(n, i_begin + seg_len);
  const int64_t* fr = f + (int64_t)row * stride_f;
  const int64_t* gr = g + (int64_t)row * stride_g;
  int64_t fmin = INT64_MAX, fmax = INT64_MIN, gmin = INT64_MAX, gmax = INT64_MIN;
  int64_t dfmin = INT64_MAX, dfmax = INT64_MIN, dgmin = INT64_MAX, dgmax = INT64_MIN;   // with the common slope removed
  const bool lines = worth_detrending(fr, gr, n);
  const int64_t f0 = fr[0], g0 = gr[0], slope = lines ? common_slope(fr, gr, n) : 0;   // (64-bit divisions: not for nothing)
  int bits = structure ? 15 : 0;
  if (partial != nullptr && threadIdx.x == 0) {
    for (int sg = 0; sg < segs; ++sg) {
      const int64_t* q = partial + ((int64_t)row * segs + sg) * kProbePartial;
      fmin = sel_min(fmin, q[0]); fmax = sel_max(fmax, q[1]);
      gmin = sel_min(gmin, q[2]); gmax = sel_max(gmax, q[3]);
      bits &= (int)q[4];
      dfmin = sel_min(dfmin, q[5]); dfmax = sel_max(dfmax, q[6]);
      dgmin = sel_min(dgmin, q[7]); dgmax = sel_max(dgmax, q[8]);
    }
  }
  if (partial == nullptr)
    probe_samples(fr, gr, 0, n, n, lines, f0, g0, slope, fmin, fmax, gmin, gmax, dfmin, dfmax, dgmin, dgmax, bits);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    fmin = sel_min(fmin, __shfl_xor(fmin, off)); fmax = sel_max(fmax, __shfl_xor(fmax, off));
    gmin = sel_min(gmin, __shfl_xor(gmin, off)); gmax = sel_max(gmax, __shfl_xor(gmax, off));
    bits &= __shfl_xor(bits, off);
  }
  if (lines) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      dfmin = sel_min(dfmin, __shfl_xor(dfmin, off)); dfmax = sel_max(dfmax, __shfl_xor(dfmax, off));
      dgmin = sel_min(dgmin, __shfl_xor(dgmin, off)); dgmax = sel_max(dgmax, __shfl_xor(dgmax, off));
    }
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    red[0][wave] = fmin; red[1][wave] = fmax; red[2][wave] = gmin; red[3][wave] = gmax;
    if (lines) { red[4][wave] = dfmin; red[5][wave] = dfmax; red[6][wave] = dgmin; red[7][wave] = dgmax; }
    s_bits[wave] = bits;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int nw = (blockDim.x + 63) >> 6;
    for (int w = 1; w < nw; ++w) {
      fmin = sel_min(fmin, red[0][w]); fmax = sel_max(fmax, red[1][w]);
      gmin = sel_min(gmin, red[2][w]); gmax = sel_max(gmax, red[3][w]);
      if (lines) {
        dfmin = sel_min(dfmin, red[4][w]); dfmax = sel_max(dfmax, red[5][w]);
        dgmin = sel_min(dgmin, red[6][w]); dgmax = sel_max(dgmax, red[7][w]);
      }
      bits &= s_bits[w];
    }
    int64_t dummy;
    const bool bad = deconv ? (__builtin_sub_overflow(fmax, gmin, &dummy) || __builtin_sub_overflow(fmin, gmax, &dummy))
                            : (__builtin_add_overflow(fmax, gmax, &dummy) || __builtin_add_overflow(fmin, gmin, &dummy));
    const bool publish = seg == 0;
    if (bad && dev_flags && publish) atomicOr(dev_flags, RTC_FLAG_OVERFLOW);
    const uint64_t frange = (uint64_t)fmax - (uint64_t)fmin, grange = (uint64_t)gmax - (uint64_t)gmin;
    // the second differences were exact only if both ranges are below 2^62
    if ((frange >> 62) != 0 || (grange >> 62) != 0) bits = 0;
    // narrow as the rows are, or (the rows' ranges permitting exact arithmetic) with the common slope removed
    const bool raw = frange < (1ull << 30) && grange < (1ull << 30);
    const uint64_t dfrange = (uint64_t)dfmax - (uint64_t)dfmin, dgrange = (uint64_t)dgmax - (uint64_t)dgmin;
    const bool lined = !raw && detrend && lines && (frange >> 62) == 0 && (grange >> 62) == 0 && dfrange < (1ull << 30) &&
                       dgrange < (1ull << 30);
    const bool narrow = raw || lined;
    const int64_t rho_row = lined ? slope : 0;
    const int64_t fb = lined ? wrap_add(f0, dfmin) : fmin, gb = lined ? wrap_add(g0, dgmin) : gmin;
    const uint64_t fr32 = lined ? dfrange : frange, gr32 = lined ? dgrange : grange;   // ranges of the int32 copies
    const int code = structure_code(op, bits, narrow ? 1 : 0);
    const bool general = code < kSelSearch;
    s_base[0] = fb; s_base[1] = gb; s_base[2] = rho_row; s_narrow = narrow && general ? 1 : 0;
    // re-based values lie in [0, 2^29): the detrended rows stay inside int32
    const bool ok = general && narrow && fr32 < (1ull << 29) && gr32 < (1ull << 29);
    if (publish) {
      narrow_ok[row] = code;
      out_base[2 * row] = narrow ? (deconv ? wrap_sub(fb, gb) : wrap_add(fb, gb)) : 0;
      out_base[2 * row + 1] = rho_row;
      pack_ok[row] = ok ? 1 : 0;
    }
    int32_t r = 0;
    if (publish && ok && n > 1) {
      // end points of the int32 copies
      const int64_t fa = 0, fz = detrended(fr[n - 1], f0, rho_row, n - 1), ga = 0, gz = detrended(gr[n - 1], g0, rho_row, n - 1);
      const int64_t w0 = deconv ? fa : ga, w1 = deconv ? fz : gz;
      const int64_t u0 = deconv ? ga : fa, u1 = deconv ? gz : fz;
      r = w1 > w0 ? (int32_t)((w1 - w0) / (n - 1)) : 0;
      const int64_t ru = (u1 - u0) / (n - 1);
      const int64_t diff = ru > r ? ru - r : r - ru;
      if (diff * kPkSub > 50000) pack_ok[row] = 0;   // same heuristic as probe_kernel
    }
    if (publish) rho[row] = r;
  }
  __syncthreads();
  if (s_narrow) {
    const int64_t fb = s_base[0], gb = s_base[1];
    const uint64_t rho_row = (uint64_t)s_base[2];
    // (rho_row = 0 when the rows are narrow as they are.)  Four strides per trip, loads first.
    constexpr int kTrip = 4;
    for (int i0 = i_begin + (int)threadIdx.x; i0 < i_end; i0 += kTrip * (int)blockDim.x) {
      int64_t fv[kTrip], gv[kTrip];
#pragma unroll
      for (int k = 0; k < kTrip; ++k) {
        const int i = min(i0 + k * (int)blockDim.x, i_end - 1);
        fv[k] = fr[i]; gv[k] = gr[i];
      }
#pragma unroll
      for (int k = 0; k < kTrip; ++k) {
        const int i = i0 + k * (int)blockDim.x;
        if (i < i_end) {
          f32[(int64_t)row * n + i] = (int32_t)(uint32_t)((uint64_t)fv[k] - (uint64_t)fb - rho_row * (uint64_t)i);
          g32[(int64_t)row * n + i] = (int32_t)(uint32_t)((uint64_t)gv[k] - (uint64_t)gb - rho_row * (uint64_t)i);
        }
      }
    }
  }
}

__device__ __forceinline__ int32_t wave_min(int32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = min(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ int32_t wave_max(int32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off));
  return v;
}

// Prepares the packed path for one (row, chunk of 1024 indices): detrends both operands
// (a = uniform operand, b = window operand, stored in window-index order, i.e. reversed for the
// deconvolution), re-bases the chunk of a to its minimum and packs it into both halves, and
// records the chunk range of a and the minima / maxima of b per block of 256.
constexpr int kPrepThreads = 256;      // per chunk of kPkChunk indices: kPkChunk / kPrepThreads = 4 per thread, 256 apart
__global__ __launch_bounds__(kPrepThreads) void prep_kernel(const int32_t* __restrict__ a, int64_t stride_a,
                                                            const int32_t* __restrict__ b, int64_t stride_b, int n,
                                                            bool deconv, bool neg, int npad, int nchunk, int nblk,
                                                            const int32_t* __restrict__ rho,
                                                            const int32_t* __restrict__ pack_ok,
                                                            uint32_t* __restrict__ apk, uint32_t* __restrict__ apk_s,
                                                            int32_t* __restrict__ ab_s, int32_t* __restrict__ ar_s,
                                                            int nsub, int32_t* __restrict__ bd, int32_t* __restrict__ ab,
                                                            int32_t* __restrict__ ar, int32_t* __restrict__ bmn,
                                                            int32_t* __restrict__ bmx) {
  constexpr int kPer = kPkChunk / kPrepThreads;
  static_assert(kPer * kPrepThreads == kPkChunk && kPrepThreads == kPkBlock && kPkSub == 128,
                "element k * 256 + t of the chunk: block k, sub-chunk 2k + t / 128, group of 64 number 4k + t / 64");
  __shared__ int32_t s_amn[16], s_amx[16], s_bmn[16], s_bmx[16];    // per group of 64 indices of the chunk
  const int row = blockIdx.x / nchunk;
  if (pack_ok[row] == 0) return;   // nothing of this row will be read
  const int c = blockIdx.x % nchunk;
  const int32_t r = rho[row];
  const int wave = threadIdx.x >> 6;
  int32_t adv[kPer], bdv[kPer];
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    // all eight loads are issued before the first is used (a load under its own bounds check is
    // waited for on the spot): positions beyond the row's end read its last sample and drop it
    const int ic = min(c * kPkChunk + k * kPrepThreads + (int)threadIdx.x, n - 1);
    adv[k] = a[(int64_t)row * stride_a + ic];
    bdv[k] = b[(int64_t)row * stride_b + (deconv ? n - 1 - ic : ic)];
  }
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const int i = c * kPkChunk + k * kPrepThreads + threadIdx.x;
    const bool valid = i < n;
    adv[k] = valid ? wrap_sub(adv[k], r * i) : 0;
    if (neg) adv[k] = wrap_sub(0, adv[k]);   // max-plus convolution / min-plus deconvolution: see packed_body
    // positions beyond the row's end are packed as 0: every window position that meets them is
    // poison, which decides the outcome whatever the uniform value
    bdv[k] = !valid ? 0 : deconv ? wrap_add(bdv[k], r * i) : wrap_sub(bdv[k], r * i);
  }
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const bool valid = c * kPkChunk + k * kPrepThreads + (int)threadIdx.x < n;
    const int32_t amn = wave_min(valid ? adv[k] : INT32_MAX), amx = wave_max(valid ? adv[k] : INT32_MIN);
    const int32_t bmn_w = wave_min(valid ? bdv[k] : INT32_MAX), bmx_w = wave_max(valid ? bdv[k] : INT32_MIN);
    if ((threadIdx.x & 63) == 0) {
      s_amn[4 * k + wave] = amn; s_amx[4 * k + wave] = amx; s_bmn[4 * k + wave] = bmn_w; s_bmx[4 * k + wave] = bmx_w;
    }
  }
  __syncthreads();
  int32_t cmn = INT32_MAX, cmx = INT32_MIN;
#pragma unroll
  for (int w = 0; w < 16; ++w) { cmn = min(cmn, s_amn[w]); cmx = max(cmx, s_amx[w]); }
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const int i = c * kPkChunk + k * kPrepThreads + threadIdx.x;
    const bool valid = i < n;
    // both packed arrays run in descending order of the step: word [npad + 15 - i] of a row of
    // npad + 16 words holds step i (the 16 steps of a block are then one aligned run of 16 words;
    // words 0..14 of a row are unused)
    apk[(int64_t)row * (npad + 16) + (npad + 15 - i)] = valid ? min((uint32_t)adv[k] - (uint32_t)cmn, kPkPoison) * 0x10001u : 0u;
    // sub-chunk of 128 indices = 2 groups of 64
    const int sub = 2 * k + (threadIdx.x >> 7);
    const int32_t smn = min(s_amn[2 * sub], s_amn[2 * sub + 1]);
    const int32_t smx = max(s_amx[2 * sub], s_amx[2 * sub + 1]);
    apk_s[(int64_t)row * (npad + 16) + (npad + 15 - i)] = valid ? min((uint32_t)adv[k] - (uint32_t)smn, kPkPoison) * 0x10001u : 0u;
    if ((threadIdx.x & (kPkSub - 1)) == 0) {
      const bool any = smx >= smn;   // false when the sub-chunk lies entirely beyond n
      const int64_t range = (int64_t)smx - (int64_t)smn;
      ab_s[(int64_t)row * nsub + c * kPkSubs + sub] = any ? smn : 0;
      ar_s[(int64_t)row * nsub + c * kPkSubs + sub] = any ? (int32_t)(range < 0x7fffffffLL ? range : 0x7fffffffLL) : 0;
    }
    if (valid) bd[(int64_t)row * ((n + 3) & ~3) + i] = bdv[k];   // rows start 16-byte aligned
    if (threadIdx.x == 0) {        // block k of 256 indices
      const int j = c * (kPkChunk / kPkBlock) + k;
      if (j < nblk) {
        int32_t mn = INT32_MAX, mx = INT32_MIN;
#pragma unroll
        for (int w = 0; w < kPkBlock / 64; ++w) { mn = min(mn, s_bmn[4 * k + w]); mx = max(mx, s_bmx[4 * k + w]); }
        bmn[(int64_t)row * nblk + j] = mn;
        bmx[(int64_t)row * nblk + j] = mx;
      }
    }
  }
  if (threadIdx.x == 0) {
    ab[(int64_t)row * nchunk + c] = cmn;
    const int64_t range = (int64_t)cmx - (int64_t)cmn;
    ar[(int64_t)row * nchunk + c] = (int32_t)(range < 0x7fffffffLL ? range : 0x7fffffffLL);
  }
}

// Performance heuristic only (results are exact either way): samples up to 32 x 32
// (tile, chunk) pairs of a row, weighted by the number of chunks they stand for, and switches the
// packed path off for the row when less than half of its chunk-tiles would qualify -- a mostly
// unpackable row is better left to the 32-bit kernel alone.
constexpr int kDecideSide = 32;   // sampled tiles x sampled chunks per tile

constexpr int kDecideThreads = kDecideSide * kDecideSide;   // one sample per thread: one chain of dependent loads

__global__ __launch_bounds__(kDecideThreads) void decide_kernel(PackAux x, int n, int32_t* __restrict__ pack_ok) {
  __shared__ float s_yes[kDecideThreads / 64], s_all[kDecideThreads / 64];
  const int row = blockIdx.x;
  const int n_t2 = (n + kPkW - 1) / kPkW;
  float yes = 0.f, all = 0.f;
  if (pack_ok[row] != 0) {
    for (int j = threadIdx.x; j < kDecideSide * kDecideSide; j += kDecideThreads) {
      const int it = j / kDecideSide, ic = j % kDecideSide;
      const int nt = min(n_t2, kDecideSide);
      if (it >= nt) continue;
      const int T2 = (int)((int64_t)it * n_t2 / nt);
      const int nc = (min((T2 + 1) * kPkW, n) + kPkChunk - 1) / kPkChunk;   // chunks of this tile
      const int ns = min(nc, kDecideSide);
      if (ic >= ns) continue;
      const int c = (int)((int64_t)ic * nc / ns);
      const float weight = (float)nc / (float)ns * ((float)n_t2 / (float)nt);
      int32_t gb, br;
      all += weight;
      yes += weight * (float)__builtin_popcount(chunk_plan(x, row, T2, c, n, &gb, &br) & 0xFF) * (1.f / kPkSubs);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { yes += __shfl_xor(yes, off); all += __shfl_xor(all, off); }
  if ((threadIdx.x & 63) == 0) { s_yes[threadIdx.x >> 6] = yes; s_all[threadIdx.x >> 6] = all; }
  __syncthreads();
  if (threadIdx.x == 0) {
    yes = all = 0.f;
    for (int w = 0; w < kDecideThreads / 64; ++w) { yes += s_yes[w]; all += s_all[w]; }
    if (2.f * yes < all) pack_ok[row] = 0;
  }
}

}  // namespace
}  // namespace rtc
