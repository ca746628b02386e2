// Shared pieces of the tropical product kernels: semirings, tile geometry, the packed path's
// per-row tables and its ownership predicate, work-item decoding.  Included by tropical.hip only
// (everything lives in an anonymous namespace of that translation unit).
#pragma once

#include <hip/hip_runtime.h>

#include <limits>
#include <type_traits>

#include "rtc_internal.h"

namespace rtc {
namespace {

#ifndef RTC_CHUNK_BLOCKS
#define RTC_CHUNK_BLOCKS 64
#endif
#ifndef RTC_CHUNK_BLOCKS_WIDE
#define RTC_CHUNK_BLOCKS_WIDE 32
#endif
#ifndef RTC_TARGET_ITEMS
#define RTC_TARGET_ITEMS 65536
#endif

template <typename T> struct Lim;
template <> struct Lim<int32_t> {
  static __device__ __forceinline__ int32_t hi() { return INT32_MAX; }
  static __device__ __forceinline__ int32_t lo() { return INT32_MIN; }
};
template <> struct Lim<int64_t> {
  static __device__ __forceinline__ int64_t hi() { return INT64_MAX; }
  static __device__ __forceinline__ int64_t lo() { return INT64_MIN; }
};
template <> struct Lim<double> {
  static __device__ __forceinline__ double hi() { return __builtin_huge_val(); }
  static __device__ __forceinline__ double lo() { return -__builtin_huge_val(); }
};

__device__ __forceinline__ int32_t wrap_add(int32_t a, int32_t b) { return (int32_t)((uint32_t)a + (uint32_t)b); }
__device__ __forceinline__ int32_t wrap_sub(int32_t a, int32_t b) { return (int32_t)((uint32_t)a - (uint32_t)b); }
__device__ __forceinline__ int64_t wrap_add(int64_t a, int64_t b) { return (int64_t)((uint64_t)a + (uint64_t)b); }
__device__ __forceinline__ int64_t wrap_sub(int64_t a, int64_t b) { return (int64_t)((uint64_t)a - (uint64_t)b); }
__device__ __forceinline__ double wrap_add(double a, double b) { return a + b; }
__device__ __forceinline__ double wrap_sub(double a, double b) { return a - b; }

__device__ __forceinline__ int32_t sel_min(int32_t a, int32_t b) { return b < a ? b : a; }
__device__ __forceinline__ int32_t sel_max(int32_t a, int32_t b) { return b > a ? b : a; }
__device__ __forceinline__ int64_t sel_min(int64_t a, int64_t b) { return b < a ? b : a; }
__device__ __forceinline__ int64_t sel_max(int64_t a, int64_t b) { return b > a ? b : a; }
// fp64: the instruction itself.  Written through the compiler's fmin / fmax, every accumulator is
// first re-canonicalised (x = max(x, x)) wherever it enters a basic block, 16 of 528 instructions
// per block of the product kernel, only so that a signalling NaN would be ignored rather than
// quieted; inputs are finite by contract, a quiet NaN is still ignored, and all other values give
// the same bits.
__device__ __forceinline__ double sel_min(double a, double b) {
  double r;
  asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ double sel_max(double a, double b) {
  double r;
  asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// The semiring of one product: identity of REDUCE, COMBINE(window, uniform), REDUCE.
// OP selects the product (the values of rtc_op for the four products):
//   0 min-plus convolution    min_s f[s] + g[t-s]        2 max-plus convolution    max_s f[s] + g[t-s]
//   1 max-plus deconvolution  max_u f[t+u] - g[u]        3 min-plus deconvolution  min_u f[t+u] - g[u]
// op_sub: COMBINE subtracts and the window operand / output index are reversed (the two
// deconvolutions); op_max: REDUCE is max.
constexpr bool op_sub(int op) { return op == 1 || op == 3; }
constexpr bool op_max(int op) { return op == 1 || op == 2; }

template <typename T, int OP> struct Semiring {
  static __device__ __forceinline__ T identity() { return op_max(OP) ? Lim<T>::lo() : Lim<T>::hi(); }
  static __device__ __forceinline__ T combine(T w, T u) { return op_sub(OP) ? wrap_sub(w, u) : wrap_add(w, u); }
  static __device__ __forceinline__ T reduce(T x, T y) { return op_max(OP) ? sel_max(x, y) : sel_min(x, y); }
};

__device__ __forceinline__ void atomic_min(int32_t* p, int32_t v) { atomicMin(p, v); }
__device__ __forceinline__ void atomic_max(int32_t* p, int32_t v) { atomicMax(p, v); }
__device__ __forceinline__ void atomic_min(int64_t* p, int64_t v) { atomicMin((long long*)p, (long long)v); }
__device__ __forceinline__ void atomic_max(int64_t* p, int64_t v) { atomicMax((long long*)p, (long long)v); }
__device__ __forceinline__ void atomic_min(double* p, double v) { atomicMin(p, v); }
__device__ __forceinline__ void atomic_max(double* p, double v) { atomicMax(p, v); }

template <typename T, int R> struct Tile {
  static constexpr int kW = 64 * R;                          // outputs per wave
  static constexpr int kChunk = (sizeof(T) == 8 ? RTC_CHUNK_BLOCKS_WIDE : RTC_CHUNK_BLOCKS) * R;  // steps of s per staged window
  static constexpr int kSlotBytes = R * (int)sizeof(T) + 16; // one group of R values + skew
  static constexpr int kSlots = 64 + kChunk / R;
  static constexpr int kVec = 16 / (int)sizeof(T);           // elements per 16-byte LDS read
};

// Geometry of the packed path: groups of 16 dwords like the int32 tile, two halves of 1024 outputs.
constexpr int kPkR = 16;
constexpr int kPkHalf = 64 * kPkR;
constexpr int kPkW = 2 * kPkHalf;
constexpr int kPkChunk = Tile<int32_t, kPkR>::kChunk;
constexpr int kPkBlock = 256;          // granularity of the window minima / maxima
constexpr int kPkSub = 128;            // finer re-basing granularity of the uniform operand (steps)
constexpr int kPkSubBlocks = kPkSub / kPkR;
constexpr int kPkSubs = kPkChunk / kPkSub;   // sub-chunks per chunk (8: their flags fit a byte)
constexpr uint32_t kPkPoison = 0xFFFFu;
static_assert(kPkSubs == 8, "the packed path keeps one flag bit per sub-chunk in a byte");

// Per-row auxiliary arrays of the packed path (all in the caller's workspace).  The uniform
// operand is re-based at two granularities: per chunk of 1024 steps (one fold per chunk, used
// when the whole chunk's range fits) and per sub-chunk of 128 steps (for operands whose slopes
// differ, where only short runs fit 16 bits).
struct PackAux {
  const uint32_t* apk;     // [B][npad+16] uniform operand, detrended, re-based per chunk, both halves, descending step order
  const uint32_t* apk_s;   // [B][npad+16] the same, re-based per sub-chunk
  const int32_t* bd;       // [B][n up to a multiple of 4]  detrended window operand, in window-index order
  const int32_t* ab;       // [B][nchunk] chunk minimum of the detrended uniform operand
  const int32_t* ar;       // [B][nchunk] chunk range
  const int32_t* ab_s;     // [B][nsub]   sub-chunk minimum
  const int32_t* ar_s;     // [B][nsub]   sub-chunk range
  const int32_t* bmn;      // [B][nblk]   minimum of bd per block of kPkBlock
  const int32_t* bmx;      // [B][nblk]   maximum
  const int32_t* rho;      // [B]         slope removed from both operands
  const int32_t* pack_ok;  // [B]         row is eligible for the packed path
  int32_t npad, nchunk, nsub, nblk;
};

// The tables of the packed path were written by earlier launches and do not change while a product
// kernel runs.  Reading them through the constant address space tells the compiler so: a load at a
// wave-uniform address then becomes a scalar load whatever stores and atomics the kernel contains
// (otherwise it falls back to a vector load with all lanes on one address).
template <typename T>
__device__ __forceinline__ const __attribute__((address_space(4))) T* as_invariant(const T* p) {
  return (const __attribute__((address_space(4))) T*)p;
}

constexpr int kPlanWhole = 0x100;    // chunk_plan: the whole chunk packs with the chunk-level re-basing
constexpr int kPlanNarrow = 0x200;   // chunk_plan: the granted runs also fit the 15-bit flavour

// Two arithmetic flavours of the packed path.
//   wide:   unsigned 16-bit values, saturating add / subtract, packed integer min / max;
//           window range + run range of the uniform operand <= kPkWideBudget.
//   narrow: values stay below 0x7C00, where the bit pattern of a non-negative half float orders
//           like the integer it encodes, so that the three-operand packed half-float minimum /
//           maximum of gfx950 reduces two candidates per instruction exactly.  No saturation is
//           available there: the poison values must survive a plain add / subtract, which costs
//           the run range twice: window range + 2 * run range <= kPkNarrowBudget.
constexpr int32_t kPkWideBudget = 65534;
constexpr int32_t kPkNarrowTop = 0x7BFF;            // largest finite half-float pattern
constexpr int32_t kPkNarrowBudget = kPkNarrowTop - 1;

// Largest run range of the uniform operand that the narrow flavour accepts next to a window of
// range br; the narrow poison values are placed relative to it (see packed_body).
__device__ __forceinline__ int32_t narrow_umax(int32_t br) { return (kPkNarrowBudget - br) / 2; }

// Which part of chunk c of the 2048-wide tile T2 of this row do the packed items own?
// Returns a byte with one bit per sub-chunk of the chunk that packed items process (0: nothing),
// kPlanWhole when the whole chunk runs on the chunk-level base (else every granted sub-chunk on
// its own base), kPlanNarrow when the narrow flavour applies.  Evaluated identically
// (wave-uniform) by packed and 32-bit items.  *gb receives the window base, *br the window range.
// The choice between a larger wide grant and a smaller narrow one weighs the cost of a sub-chunk
// in the narrow, wide and 32-bit kernels (0.5, 1 and 1.5 VALU instructions per candidate plus the
// folds: about 11 : 21 : 30), i.e. what each grant saves against leaving its sub-chunks to the
// 32-bit items.
__device__ __forceinline__ int chunk_plan(const PackAux& x, int row, int T2, int c, int n, int32_t* gb,
                                          int32_t* br) {
  if (as_invariant(x.pack_ok)[row] == 0) return 0;
  const int sc = c * kPkChunk;
  int lo = T2 * kPkW - sc - kPkChunk;
  int hi = T2 * kPkW + kPkW - sc;
  lo = max(lo, 0);
  hi = min(hi, n);
  const int b0 = lo / kPkBlock, b1 = (hi - 1) / kPkBlock;
  const auto* mnp = as_invariant(x.bmn + (int64_t)row * x.nblk);
  const auto* mxp = as_invariant(x.bmx + (int64_t)row * x.nblk);
  int32_t mn = INT32_MAX, mx = INT32_MIN;
  for (int b = b0; b <= b1; ++b) {
    mn = min(mn, mnp[b]);
    mx = max(mx, mxp[b]);
  }
  *gb = mn;
  const int64_t wr = (int64_t)mx - (int64_t)mn;
  if (wr > kPkWideBudget) return 0;
  *br = (int32_t)wr;
  const int64_t cr = as_invariant(x.ar)[(int64_t)row * x.nchunk + c];
  if (wr + 2 * cr <= kPkNarrowBudget) return kPlanNarrow | kPlanWhole | 0xFF;
  const bool wide_whole = wr + cr <= kPkWideBudget;
  const auto* ars = as_invariant(x.ar_s + (int64_t)row * x.nsub + c * kPkSubs);
  int narrow = 0, wide = 0;
#pragma unroll
  for (int j = 0; j < kPkSubs; ++j) {
    const int64_t r = ars[j];
    if (wr + 2 * r <= kPkNarrowBudget) narrow |= 1 << j;
    if (wr + r <= kPkWideBudget) wide |= 1 << j;
  }
  const int n_narrow = __builtin_popcount(narrow), n_wide = wide_whole ? kPkSubs : __builtin_popcount(wide);
  if (n_narrow > 0 && 19 * n_narrow >= 9 * n_wide) return kPlanNarrow | narrow;
  return wide_whole ? (kPlanWhole | 0xFF) : wide;
}

struct TropicalArgs {
  const void* a;        // operand indexed by s (wave-uniform), rows of stride_a elements
  const void* b;        // operand indexed by t-s (window), rows of stride_b elements
  void* out;            // dense [batch][n]
  const void* cap;      // optional dense [batch][n]: out = min(out, cap)
  const int32_t* sel;   // optional per-row selector; a row runs only if sel[row] == sel_want
  int64_t stride_a;
  int64_t stride_b;
  int32_t sel_want;
  int32_t n;
  int32_t batch;
  int32_t n_tiles;
  int32_t fold_width;   // work items launched per folded tile pair (see decode_item)
  int32_t seg;          // steps of s per segment, a multiple of the chunk length
  const int64_t* out_base;  // optional per-row [constant, slope]: constant + slope * (output index) is added to every stored value (narrowed int64 rows)
  int32_t use_aux;      // 1: skip the chunks that the packed items of the same launch own (see aux)
  PackAux aux;
};

// Work item = (tile, segment, row), rows fastest.  Tile k has ceil(s_end(k) / seg) segments,
// which grows linearly with k; tile k is therefore folded with tile n_tiles-1-k so that
// every folded pair owns about the same number of items and few launched workgroups are idle.
// Returns false when this workgroup has nothing to do.
template <int W>
__device__ __forceinline__ bool decode_item(const TropicalArgs& p, uint32_t item, int* row, int* t0, int* sa,
                                            int* sb) {
  const int n = p.n;
  *row = item % (uint32_t)p.batch;
  item /= (uint32_t)p.batch;
  const int j = item % (uint32_t)p.fold_width;
  const int k_lo = item / (uint32_t)p.fold_width;
  const int k_hi = p.n_tiles - 1 - k_lo;
  const int nseg_hi = (min((k_hi + 1) * W, n) + p.seg - 1) / p.seg;
  int tile, seg;
  if (j < nseg_hi) {
    tile = k_hi; seg = j;
  } else {
    if (k_lo == k_hi) return false;
    tile = k_lo; seg = j - nseg_hi;
  }
  *t0 = tile * W;
  const int s_end = min(*t0 + W, n);
  *sa = seg * p.seg;
  if (*sa >= s_end) return false;
  if (p.sel != nullptr && p.sel[*row] != p.sel_want) return false;
  *sb = min(*sa + p.seg, s_end);
  return true;
}

template <typename T, int R>
__device__ __forceinline__ void load_group(T (&dst)[R], const unsigned char* lds, int slot) {
  typedef T Vec __attribute__((ext_vector_type(Tile<T, R>::kVec)));
  const Vec* src = reinterpret_cast<const Vec*>(lds + slot * Tile<T, R>::kSlotBytes);
#pragma unroll
  for (int q = 0; q < R / Tile<T, R>::kVec; ++q) {
    Vec v = src[q];
#pragma unroll
    for (int e = 0; e < Tile<T, R>::kVec; ++e) dst[q * Tile<T, R>::kVec + e] = v[e];
  }
}

// Window buffer of one workgroup; tiles of 4 accumulators also stage a chunk of the uniform operand
// behind it (tropical_body).
template <typename T, int R> constexpr int window_bytes() { return Tile<T, R>::kSlots * Tile<T, R>::kSlotBytes; }
template <typename T, int R> constexpr int lds_bytes() {
  return window_bytes<T, R>() + (R == 4 ? Tile<T, R>::kChunk * (int)sizeof(T) : 0);
}

}  // namespace
}  // namespace rtc
