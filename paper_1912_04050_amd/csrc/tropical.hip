// Tropical (min,+) / (max,-) products on the vector ALUs of gfx950.
//
//   min-plus convolution     out[t] = min_{0<=s<=t}     f[s]   + g[t-s]
//   max-plus deconvolution   out[t] = max_{0<=u<=n-1-t} f[t+u] - g[u]
//
// Both are instances of one triangular product
//   out'[t] = REDUCE_{0<=s<=t} COMBINE(b'[t-s], a[s])
// with (a, b') = (f, g), COMBINE = +, REDUCE = min for the convolution, and
// (a, b') = (g, f reversed), COMBINE = window - uniform, REDUCE = max, output stored
// reversed, for the deconvolution (substitute t -> n-1-t).
//
// Mapping to the machine (one wave64 per workgroup, no barriers between waves):
//   * a wave owns a tile of W = 64*R consecutive outputs; lane l owns the R consecutive
//     outputs t0 + l*R .. t0 + l*R + R-1 and keeps their running reductions in VGPRs;
//   * the operand indexed by s is wave-uniform: it is fetched with scalar loads and used
//     as the SGPR source of the VALU add/sub, so it costs no vector issue slot;
//   * the operand indexed by t-s is a sliding window: per block of R steps a lane needs
//     one new aligned group of R values, read from an LDS copy of the window with
//     16-byte reads.  Groups are stored with a 16-byte skew per group so that the 64 lanes
//     (whose groups are consecutive) hit distinct banks;
//   * per (lane, step, output) the inner loop is exactly one add/sub and one min/max.
// The s range of a tile is cut into segments so that a launch has enough equally sized work
// items; partial results of one tile are merged with atomic min/max (exact and order-free).
// On the diagonal (s-block overlapping the tile) block j only concerns lanes > j, which run
// under an exec mask; each lane's own R x R triangle is finished by a short epilogue.
//
// Packed 16-bit path (int32 arithmetic only).  A common slope rho is removed from both
// operands: with ad[s] = a[s] - rho*s and bd[i] = b'[i] -/+ rho*i (minus for the convolution,
// plus for the deconvolution, whose window operand is the reversed, hence falling, f) every
// candidate equals COMBINE(bd[t-s], ad[s]) +/- rho*t, so the trend is put back once per output.
// Per chunk of 1024 steps the detrended values are re-based to the chunk / window minimum;
// when range(ad chunk) + range(bd window) <= 65534 every candidate of that (tile, chunk) fits
// an unsigned 16-bit lane, and two output halves of a 2048-wide tile are computed at once with
// v_pk_add_u16 + v_pk_min_u16 (v_pk_sub_u16 + v_pk_max_u16 for the deconvolution), both
// saturating: one VALU instruction per pair-op instead of 1.5.
// Positions that do not exist (window index < 0, s >= n) are staged as a poison value that
// saturates and never wins, so the packed kernel needs neither exec masks nor a triangle epilogue.
// The decision is made per (row, tile, chunk) from precomputed block minima / maxima; chunks
// that do not qualify are done by the 32-bit kernel, which evaluates the same predicate and
// skips exactly the chunks the packed kernel owns.  Results are exact in both cases.
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
__device__ __forceinline__ double sel_min(double a, double b) { return __builtin_fmin(a, b); }
__device__ __forceinline__ double sel_max(double a, double b) { return __builtin_fmax(a, b); }

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
  const uint32_t* apk;     // [B][npad]   uniform operand, detrended, re-based per chunk, both halves
  const uint32_t* apk_s;   // [B][npad]   the same, re-based per sub-chunk
  const int32_t* bd;       // [B][n]      detrended window operand, in window-index order
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

constexpr int kPlanWhole = 0x100;   // chunk_plan: the whole chunk packs with the chunk-level re-basing

// Which part of chunk c of the 2048-wide tile T2 of this row do the packed items own?
// Returns kPlanWhole | 0xFF when the whole chunk qualifies with the chunk-level base, else a
// byte with one bit per sub-chunk that qualifies with its own base (0: nothing).  Evaluated
// identically (wave-uniform) by packed and 32-bit items.  *gb receives the window base, *br the
// window range.
__device__ __forceinline__ int chunk_plan(const PackAux& x, int row, int T2, int c, int n, int32_t* gb,
                                          int32_t* br) {
  if (x.pack_ok[row] == 0) return 0;
  const int sc = c * kPkChunk;
  int lo = T2 * kPkW - sc - kPkChunk;
  int hi = T2 * kPkW + kPkW - sc;
  lo = max(lo, 0);
  hi = min(hi, n);
  const int b0 = lo / kPkBlock, b1 = (hi - 1) / kPkBlock;
  const int32_t* mnp = x.bmn + (int64_t)row * x.nblk;
  const int32_t* mxp = x.bmx + (int64_t)row * x.nblk;
  int32_t mn = INT32_MAX, mx = INT32_MIN;
  for (int b = b0; b <= b1; ++b) {
    mn = min(mn, mnp[b]);
    mx = max(mx, mxp[b]);
  }
  *gb = mn;
  const int64_t wr = (int64_t)mx - (int64_t)mn;
  if (wr > 65534) return 0;
  *br = (int32_t)wr;
  if ((int64_t)x.ar[(int64_t)row * x.nchunk + c] + wr <= 65534) return kPlanWhole | 0xFF;
  const int32_t* ars = x.ar_s + (int64_t)row * x.nsub + c * kPkSubs;
  int plan = 0;
#pragma unroll
  for (int j = 0; j < kPkSubs; ++j)
    if ((int64_t)ars[j] + wr <= 65534) plan |= 1 << j;
  return plan;
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
  const int64_t* out_base;  // optional per-row constant added to every stored value (re-based int64 rows)
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

// R steps of s against the R outputs of a lane.  hi = window group [D, D+R), lo = [D-R, D),
// D = (first output of the lane) - (first step of the block); step k, output r reads D+r-k.
template <typename SR, typename T, int R>
__device__ __forceinline__ void block_steps(T (&acc)[R], const T (&u)[R], const T (&lo)[R],
                                            const T (&hi)[R]) {
#pragma unroll
  for (int k = 0; k < R; ++k) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const T w = (r >= k) ? hi[r - k] : lo[R + r - k];
      acc[r] = SR::reduce(acc[r], SR::combine(w, u[k]));
    }
  }
}

template <typename T, int R> constexpr int lds_bytes() { return Tile<T, R>::kSlots * Tile<T, R>::kSlotBytes; }

// Body of one work item of the generic (32-bit / 64-bit / fp64) product.  `lds` is the
// workgroup's window buffer of lds_bytes<T, R>() bytes.
template <typename T, typename OutT, int OP, int R, bool ATOMIC>
__device__ __forceinline__ void tropical_body(const TropicalArgs& p, unsigned char* lds, uint32_t item) {
  using SR = Semiring<T, OP>;
  using TL = Tile<T, R>;

  const int lane = threadIdx.x;
  const int n = p.n;
  int row, t0, sa, sb;
  if (!decode_item<TL::kW>(p, item, &row, &t0, &sa, &sb)) return;
  // with the packed path active (int32 only) the chunks owned by packed items are skipped
  const bool aux = std::is_same<T, int32_t>::value && p.use_aux != 0;
  constexpr bool rev = op_sub(OP);

  const T* __restrict__ arow = static_cast<const T*>(p.a) + (int64_t)row * p.stride_a;
  const T* __restrict__ brow = static_cast<const T*>(p.b) + (int64_t)row * p.stride_b;

  T acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = SR::identity();

  for (int sc = sa; sc < sb; sc += TL::kChunk) {
    const int ce = min(sc + TL::kChunk, sb);
    const int nblk = (ce - sc + R - 1) / R;
    int plan = 0;   // bit j: the blocks of sub-chunk j of this chunk belong to packed items
    if (aux) {
      int32_t gb, br;
      plan = chunk_plan(p.aux, row, t0 / kPkW, sc / kPkChunk, n, &gb, &br) & 0xFF;
      const int need = (1 << ((nblk + kPkSubBlocks - 1) / kPkSubBlocks)) - 1;
      if ((plan & need) == need) continue;
    }
    // LDS slot q holds window elements [gbase + q*R, gbase + q*R + R)
    const int gbase = t0 - (sc + nblk * R);
    const int count = (64 + nblk) * R;
    __syncthreads();
    for (int e = lane; e < count; e += 64) {
      const int idx = gbase + e;
      T v = T(0);
      if (idx >= 0 && idx < n) v = brow[rev ? n - 1 - idx : idx];
      *reinterpret_cast<T*>(lds + (e / R) * TL::kSlotBytes + (e % R) * (int)sizeof(T)) = v;
    }
    __syncthreads();

    T w0[R], w1[R];
    load_group<T, R>(w0, lds, lane + nblk);
    for (int i = 0; i < nblk; i += 2) {
      {
        const int s0 = sc + i * R;
        load_group<T, R>(w1, lds, lane + nblk - i - 1);
        const int j = (s0 >= t0) ? (s0 - t0) / R : -1;
        if ((j < 0 || (s0 + R < n && j < 63)) && !((plan >> (i / kPkSubBlocks)) & 1)) {
          T u[R];
#pragma unroll
          for (int k = 0; k < R; ++k) u[k] = arow[s0 + k];
          if (lane > j) block_steps<SR, T, R>(acc, u, w1, w0);
        }
      }
      if (i + 1 < nblk) {
        const int s0 = sc + (i + 1) * R;
        load_group<T, R>(w0, lds, lane + nblk - i - 2);
        const int j = (s0 >= t0) ? (s0 - t0) / R : -1;
        if ((j < 0 || (s0 + R < n && j < 63)) && !((plan >> ((i + 1) / kPkSubBlocks)) & 1)) {
          T u[R];
#pragma unroll
          for (int k = 0; k < R; ++k) u[k] = arow[s0 + k];
          if (lane > j) block_steps<SR, T, R>(acc, u, w0, w1);
        }
      }
    }
  }

  const int tl = t0 + lane * R;
  // the lane's own triangle: steps s = tl+k against outputs tl+r, r >= k, window index r-k
  bool triangle = sa <= t0 && t0 < sb;
  if (aux && triangle) {
    // the triangle of lane l lies in sub-chunk l*R / kPkSub of the diagonal chunk
    int32_t gb, br;
    const int plan = chunk_plan(p.aux, row, t0 / kPkW, t0 / kPkChunk, n, &gb, &br);
    if ((plan >> (lane * R / kPkSub)) & 1) triangle = false;
  }
  if (triangle) {
    T b0[R];
#pragma unroll
    for (int q = 0; q < R; ++q) {
      const int idx = min(q, n - 1);
      b0[q] = brow[rev ? n - 1 - idx : idx];
    }
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const T ak = arow[min(tl + k, n - 1)];
#pragma unroll
      for (int r = k; r < R; ++r) acc[r] = SR::reduce(acc[r], SR::combine(b0[r - k], ak));
    }
  }

  OutT* __restrict__ orow = static_cast<OutT*>(p.out) + (int64_t)row * n;
  const OutT* __restrict__ crow =
      p.cap ? static_cast<const OutT*>(p.cap) + (int64_t)row * n : nullptr;
  // Transpose the accumulators through LDS (lane-major [lane][R+1] -> output-major) so that
  // the 64 lanes of one store / atomic instruction touch 64 consecutive outputs.
  static_assert(64 * (R + 1) * sizeof(T) <= lds_bytes<T, R>(), "transpose buffer must fit the window buffer");
  T* xp = reinterpret_cast<T*>(lds);
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) xp[lane * (R + 1) + r] = acc[r];
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int x = r * 64 + lane;          // output offset inside the tile
    const int t = t0 + x;
    if (t < n) {
      const int ot = op_sub(OP) ? n - 1 - t : t;
      const T av = xp[x + x / R];
      if (ATOMIC && av == SR::identity()) continue;   // this item saw no candidate of that output
      OutT v = (OutT)av;
      if (p.out_base != nullptr) v += (OutT)p.out_base[row];
      if (crow) v = sel_min(v, crow[ot]);
      if (ATOMIC) {
        if (op_max(OP)) atomic_max(&orow[ot], v); else atomic_min(&orow[ot], v);
      } else {
        orow[ot] = v;
      }
    }
  }
}

// ---- packed 16-bit kernel -----------------------------------------------------------------

typedef unsigned short us2 __attribute__((ext_vector_type(2)));

// 16 steps against the 16 packed accumulators of a lane (window groups as in block_steps).
// The combined values of a whole step are formed before the reductions so that no instruction
// reads the result of its immediate predecessor (the compiler otherwise pads each pair with a
// wait state).
template <bool MAXF>
__device__ __forceinline__ void block_steps_packed(uint32_t (&acc)[kPkR], const uint32_t (&u)[kPkR],
                                                   const uint32_t (&lo)[kPkR], const uint32_t (&hi)[kPkR]) {
#pragma unroll
  for (int k = 0; k < kPkR; ++k) {
    us2 s[kPkR];
#pragma unroll
    for (int r = 0; r < kPkR; ++r) {
      const us2 w = __builtin_bit_cast(us2, (r >= k) ? hi[r - k] : lo[kPkR + r - k]);
      const us2 uu = __builtin_bit_cast(us2, u[k]);
      s[r] = MAXF ? __builtin_elementwise_sub_sat(w, uu) : __builtin_elementwise_add_sat(w, uu);
    }
#pragma unroll
    for (int r = 0; r < kPkR; ++r) {
      const us2 av = __builtin_bit_cast(us2, acc[r]);
      acc[r] = __builtin_bit_cast(uint32_t, MAXF ? __builtin_elementwise_max(av, s[r])
                                                   : __builtin_elementwise_min(av, s[r]));
    }
  }
}

// One wave owns 2048 outputs of the triangular product: the low 16 bits of every packed
// register belong to output t0 + 16*lane + r, the high 16 bits to output t0 + 1024 + 16*lane + r.
// Only the chunks / sub-chunks that chunk_plan() grants are processed; results merge into out with
// atomic min / max.
//   convolution:   lane value = (bd - gb) + (ad - ab); poison 0xFFFF (saturating add, min)
//   deconvolution: lane value = (bd - gb) + ar + 1 - (ad - ab) >= 1; poison 0 for the window,
//                  0xFFFF for the uniform operand (saturating subtract gives 0, max ignores it)
template <typename OutT, int OP>
__device__ __forceinline__ void packed_body(const TropicalArgs& p, unsigned char* lds, uint32_t item) {
  using TL = Tile<int32_t, kPkR>;
  const int lane = threadIdx.x;
  const int n = p.n;
  int row, t0, sa, sb;
  if (!decode_item<kPkW>(p, item, &row, &t0, &sa, &sb)) return;
  const PackAux& x = p.aux;
  if (x.pack_ok[row] == 0) return;
  const uint32_t* __restrict__ apk = x.apk + (int64_t)row * x.npad;
  const uint32_t* __restrict__ apk_s = x.apk_s + (int64_t)row * x.npad;
  const int32_t* __restrict__ bd = x.bd + (int64_t)row * n;
  const int32_t* __restrict__ ab = x.ab + (int64_t)row * x.nchunk;
  const int32_t* __restrict__ ab_s = x.ab_s + (int64_t)row * x.nsub;
  constexpr bool MAXF = op_max(OP);   // arithmetic flavour: saturating subtract + max, or saturating add + min
  constexpr int32_t kIdent = MAXF ? INT32_MIN : INT32_MAX;
  constexpr uint32_t kWinPoison = MAXF ? 0u : kPkPoison;   // staged for window positions that do not exist
  constexpr uint32_t kAccPoison = MAXF ? 0u : kPkPoison;   // a 16-bit lane that saw no existing candidate

  int32_t acc_lo[kPkR], acc_hi[kPkR];
#pragma unroll
  for (int r = 0; r < kPkR; ++r) { acc_lo[r] = kIdent; acc_hi[r] = kIdent; }

  for (int sc = sa; sc < sb; sc += kPkChunk) {
    int32_t gb, br;
    const int c = sc / kPkChunk;
    const int plan = chunk_plan(x, row, t0 / kPkW, c, n, &gb, &br);
    if (plan == 0) continue;
    const int ce = min(sc + kPkChunk, sb);
    const int nblk = (ce - sc + kPkR - 1) / kPkR;
    const int gbase = t0 - (sc + nblk * kPkR);
    const int count = (64 + nblk) * kPkR;
    // max flavour: window values are lifted so that every existing candidate stays >= 1 after
    // the saturating subtraction (the window spans at most br, any packable run of the uniform
    // operand at most 65534 - br)
    const uint32_t lift = MAXF ? 65535u - (uint32_t)br : 0u;
    __syncthreads();
    for (int e = lane; e < count; e += 64) {
      const int il = gbase + e, ih = il + kPkHalf;
      uint32_t vl = kWinPoison, vh = kWinPoison;
      if (il >= 0 && il < n) vl = min((uint32_t)bd[il] - (uint32_t)gb + lift, kPkPoison);
      if (ih >= 0 && ih < n) vh = min((uint32_t)bd[ih] - (uint32_t)gb + lift, kPkPoison);
      *reinterpret_cast<uint32_t*>(lds + (e / kPkR) * TL::kSlotBytes + (e % kPkR) * 4) = vl | (vh << 16);
    }
    __syncthreads();

    // a run = a range of blocks that shares one base of the uniform operand: the whole chunk,
    // or one qualifying sub-chunk
    const bool whole = (plan & kPlanWhole) != 0;
    const uint32_t* __restrict__ usrc = whole ? apk : apk_s;
    const int nrun = whole ? 1 : kPkSubs;
    for (int run = 0; run < nrun; ++run) {
      const int first = whole ? 0 : run * kPkSubBlocks;
      if (first >= nblk) break;
      if (!whole && !((plan >> run) & 1)) continue;
      const int last = whole ? nblk : min(first + kPkSubBlocks, nblk);
      const int32_t ubase = whole ? ab[c] : ab_s[c * kPkSubs + run];

      uint32_t acc[kPkR];
#pragma unroll
      for (int r = 0; r < kPkR; ++r) acc[r] = kAccPoison * 0x10001u;
      uint32_t w0[kPkR], w1[kPkR];
      load_group<uint32_t, kPkR>(w0, lds, lane + nblk - first);
      for (int i = first; i < last; i += 2) {
        {
          const int s0 = sc + i * kPkR;
          load_group<uint32_t, kPkR>(w1, lds, lane + nblk - i - 1);
          uint32_t u[kPkR];
#pragma unroll
          for (int k = 0; k < kPkR; ++k) u[k] = usrc[s0 + k];
          block_steps_packed<MAXF>(acc, u, w1, w0);
        }
        if (i + 1 < last) {
          const int s0 = sc + (i + 1) * kPkR;
          load_group<uint32_t, kPkR>(w0, lds, lane + nblk - i - 2);
          uint32_t u[kPkR];
#pragma unroll
          for (int k = 0; k < kPkR; ++k) u[k] = usrc[s0 + k];
          block_steps_packed<MAXF>(acc, u, w0, w1);
        }
      }
      // fold the run into the 32-bit accumulators (detrended domain, wrap-around arithmetic:
      // every folded value is a true candidate, which fits)
      const uint32_t cb = MAXF ? (uint32_t)gb - (uint32_t)ubase - lift : (uint32_t)ubase + (uint32_t)gb;
#pragma unroll
      for (int r = 0; r < kPkR; ++r) {
        const uint32_t vl = acc[r] & 0xFFFFu, vh = acc[r] >> 16;
        const int32_t cl = vl != kAccPoison ? (int32_t)(cb + vl) : kIdent;
        const int32_t ch = vh != kAccPoison ? (int32_t)(cb + vh) : kIdent;
        acc_lo[r] = MAXF ? max(acc_lo[r], cl) : min(acc_lo[r], cl);
        acc_hi[r] = MAXF ? max(acc_hi[r], ch) : min(acc_hi[r], ch);
      }
    }
  }

  OutT* __restrict__ orow = static_cast<OutT*>(p.out) + (int64_t)row * n;
  const OutT* __restrict__ crow =
      p.cap ? static_cast<const OutT*>(p.cap) + (int64_t)row * n : nullptr;
  const int32_t rho = x.rho[row];
  int32_t* xp = reinterpret_cast<int32_t*>(lds);
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kPkR; ++r) xp[lane * (kPkR + 1) + r] = half == 0 ? acc_lo[r] : acc_hi[r];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kPkR; ++r) {
      const int xo = r * 64 + lane;
      const int t = t0 + half * kPkHalf + xo;
      const int32_t av = xp[xo + xo / kPkR];
      if (t < n && av != kIdent) {
        const int ot = op_sub(OP) ? n - 1 - t : t;
        OutT v = (OutT)(op_sub(OP) ? wrap_sub(av, rho * t) : wrap_add(av, rho * t));
        if (p.out_base != nullptr) v += (OutT)p.out_base[row];
        if (crow) v = sel_min(v, crow[ot]);
        if (op_max(OP)) atomic_max(&orow[ot], v); else atomic_min(&orow[ot], v);
      }
    }
  }
}

template <typename T, typename OutT, int OP, int R, bool ATOMIC>
__global__ __launch_bounds__(64) void tropical_kernel(const TropicalArgs p) {
  __shared__ __align__(16) unsigned char lds[lds_bytes<T, R>()];
  tropical_body<T, OutT, OP, R, ATOMIC>(p, lds, blockIdx.x);
}

// One launch for an int32 product with the packed path: the first n_packed workgroups are
// items of the packed kernel, the rest are items of the 32-bit kernel (which skip the chunks
// the packed items own).  Issuing both kinds together keeps the machine full whatever share of
// the chunks qualifies for 16 bits.
template <typename OutT, int OP>
__global__ __launch_bounds__(64) void fused_kernel(const TropicalArgs pk, const TropicalArgs pg,
                                                   uint32_t n_packed) {
  __shared__ __align__(16) unsigned char lds[lds_bytes<int32_t, kPkR>()];
  if (blockIdx.x < n_packed) packed_body<OutT, OP>(pk, lds, blockIdx.x);
  else tropical_body<int32_t, OutT, OP, kPkR, true>(pg, lds, blockIdx.x - n_packed);
}

template <typename T>
__global__ __launch_bounds__(256) void fill_kernel(T* __restrict__ dst, int64_t count, T value) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += step) dst[i] = value;
}

// Range probe of one row pair.  Finds min/max of both rows, raises the overflow flag when
// the bounds do not prove that every candidate fits and (optionally) decides eligibility for
// the packed path and the slope to remove.
template <typename T>
__global__ __launch_bounds__(1024) void probe_kernel(const T* __restrict__ f, int64_t stride_f,
                                                     const T* __restrict__ g, int64_t stride_g, int n,
                                                     bool deconv, int32_t* __restrict__ pack_ok,
                                                     int32_t* __restrict__ rho,
                                                     int32_t* __restrict__ dev_flags) {
  __shared__ T red[4][16];
  const int row = blockIdx.x;
  const T* fr = f + (int64_t)row * stride_f;
  const T* gr = g + (int64_t)row * stride_g;
  T fmin = Lim<T>::hi(), fmax = Lim<T>::lo(), gmin = Lim<T>::hi(), gmax = Lim<T>::lo();
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const T fv = fr[i], gv = gr[i];
    fmin = sel_min(fmin, fv); fmax = sel_max(fmax, fv);
    gmin = sel_min(gmin, gv); gmax = sel_max(gmax, gv);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    fmin = sel_min(fmin, __shfl_xor(fmin, off)); fmax = sel_max(fmax, __shfl_xor(fmax, off));
    gmin = sel_min(gmin, __shfl_xor(gmin, off)); gmax = sel_max(gmax, __shfl_xor(gmax, off));
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[0][wave] = fmin; red[1][wave] = fmax; red[2][wave] = gmin; red[3][wave] = gmax; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int nw = (blockDim.x + 63) >> 6;
    for (int w = 1; w < nw; ++w) {
      fmin = sel_min(fmin, red[0][w]); fmax = sel_max(fmax, red[1][w]);
      gmin = sel_min(gmin, red[2][w]); gmax = sel_max(gmax, red[3][w]);
    }
    if constexpr (!std::numeric_limits<T>::is_integer) {
      (void)dev_flags;
    } else {
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
        rho[row] = r;
      }
    }
  }
}

// Range probe of one int64 row pair.  A row whose two value ranges (max - min) are below 2^30
// is re-based to its minima and copied as int32: every candidate of the re-based rows fits
// 32 bits, so the 32-bit kernels compute it exactly and add `out_base` (f_min + g_min, or
// f_min - g_min for the deconvolutions) back on store.  Rows with a wider range keep the
// 64-bit kernel.  Also: overflow flag, packed-path eligibility and slope, as in probe_kernel.
__global__ __launch_bounds__(1024) void probe_narrow_kernel(const int64_t* __restrict__ f, int64_t stride_f,
                                                            const int64_t* __restrict__ g, int64_t stride_g,
                                                            int n, bool deconv, int32_t* __restrict__ f32,
                                                            int32_t* __restrict__ g32,
                                                            int32_t* __restrict__ narrow_ok,
                                                            int64_t* __restrict__ out_base,
                                                            int32_t* __restrict__ pack_ok,
                                                            int32_t* __restrict__ rho,
                                                            int32_t* __restrict__ dev_flags) {
  __shared__ int64_t red[4][16];
  __shared__ int64_t s_base[2];
  __shared__ int s_narrow;
  const int row = blockIdx.x;
  const int64_t* fr = f + (int64_t)row * stride_f;
  const int64_t* gr = g + (int64_t)row * stride_g;
  int64_t fmin = INT64_MAX, fmax = INT64_MIN, gmin = INT64_MAX, gmax = INT64_MIN;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const int64_t fv = fr[i], gv = gr[i];
    fmin = sel_min(fmin, fv); fmax = sel_max(fmax, fv);
    gmin = sel_min(gmin, gv); gmax = sel_max(gmax, gv);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    fmin = sel_min(fmin, __shfl_xor(fmin, off)); fmax = sel_max(fmax, __shfl_xor(fmax, off));
    gmin = sel_min(gmin, __shfl_xor(gmin, off)); gmax = sel_max(gmax, __shfl_xor(gmax, off));
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[0][wave] = fmin; red[1][wave] = fmax; red[2][wave] = gmin; red[3][wave] = gmax; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int nw = (blockDim.x + 63) >> 6;
    for (int w = 1; w < nw; ++w) {
      fmin = sel_min(fmin, red[0][w]); fmax = sel_max(fmax, red[1][w]);
      gmin = sel_min(gmin, red[2][w]); gmax = sel_max(gmax, red[3][w]);
    }
    int64_t dummy;
    const bool bad = deconv ? (__builtin_sub_overflow(fmax, gmin, &dummy) || __builtin_sub_overflow(fmin, gmax, &dummy))
                            : (__builtin_add_overflow(fmax, gmax, &dummy) || __builtin_add_overflow(fmin, gmin, &dummy));
    if (bad && dev_flags) atomicOr(dev_flags, RTC_FLAG_OVERFLOW);
    const uint64_t frange = (uint64_t)fmax - (uint64_t)fmin, grange = (uint64_t)gmax - (uint64_t)gmin;
    const bool narrow = frange < (1ull << 30) && grange < (1ull << 30);
    narrow_ok[row] = narrow ? 1 : 0;
    out_base[row] = narrow ? (deconv ? wrap_sub(fmin, gmin) : wrap_add(fmin, gmin)) : 0;
    s_base[0] = fmin; s_base[1] = gmin; s_narrow = narrow ? 1 : 0;
    // re-based values lie in [0, 2^29): the detrended rows stay inside int32
    const bool ok = frange < (1ull << 29) && grange < (1ull << 29);
    pack_ok[row] = ok ? 1 : 0;
    int32_t r = 0;
    if (ok && n > 1) {
      const int64_t w0 = deconv ? fr[0] : gr[0], w1 = deconv ? fr[n - 1] : gr[n - 1];
      const int64_t u0 = deconv ? gr[0] : fr[0], u1 = deconv ? gr[n - 1] : fr[n - 1];
      r = w1 > w0 ? (int32_t)((w1 - w0) / (n - 1)) : 0;
      const int64_t ru = (u1 - u0) / (n - 1);
      const int64_t diff = ru > r ? ru - r : r - ru;
      if (diff * kPkSub > 50000) pack_ok[row] = 0;   // same heuristic as probe_kernel
    }
    rho[row] = r;
  }
  __syncthreads();
  if (s_narrow) {
    const int64_t fb = s_base[0], gb = s_base[1];
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
      f32[(int64_t)row * n + i] = (int32_t)(fr[i] - fb);
      g32[(int64_t)row * n + i] = (int32_t)(gr[i] - gb);
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
__global__ __launch_bounds__(1024) void prep_kernel(const int32_t* __restrict__ a, int64_t stride_a,
                                                    const int32_t* __restrict__ b, int64_t stride_b, int n,
                                                    bool deconv, bool neg, int npad, int nchunk, int nblk,
                                                    const int32_t* __restrict__ rho,
                                                    const int32_t* __restrict__ pack_ok,
                                                    uint32_t* __restrict__ apk, uint32_t* __restrict__ apk_s,
                                                    int32_t* __restrict__ ab_s, int32_t* __restrict__ ar_s,
                                                    int nsub, int32_t* __restrict__ bd, int32_t* __restrict__ ab,
                                                    int32_t* __restrict__ ar, int32_t* __restrict__ bmn,
                                                    int32_t* __restrict__ bmx) {
  __shared__ int32_t s_amn[16], s_amx[16], s_bmn[16], s_bmx[16];
  const int row = blockIdx.x / nchunk;
  if (pack_ok[row] == 0) return;   // nothing of this row will be read
  const int c = blockIdx.x % nchunk;
  const int i = c * kPkChunk + threadIdx.x;
  const int32_t r = rho[row];
  const bool valid = i < n;
  int32_t adv = valid ? wrap_sub(a[(int64_t)row * stride_a + i], r * i) : 0;
  if (neg) adv = wrap_sub(0, adv);   // max-plus convolution / min-plus deconvolution: see packed_body
  int32_t bdv = 0;
  if (valid) bdv = deconv ? wrap_add(b[(int64_t)row * stride_b + (n - 1 - i)], r * i)
                          : wrap_sub(b[(int64_t)row * stride_b + i], r * i);
  const int32_t amn = wave_min(valid ? adv : INT32_MAX), amx = wave_max(valid ? adv : INT32_MIN);
  const int32_t bmn_w = wave_min(valid ? bdv : INT32_MAX), bmx_w = wave_max(valid ? bdv : INT32_MIN);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { s_amn[wave] = amn; s_amx[wave] = amx; s_bmn[wave] = bmn_w; s_bmx[wave] = bmx_w; }
  __syncthreads();
  int32_t cmn = INT32_MAX, cmx = INT32_MIN;
#pragma unroll
  for (int w = 0; w < 16; ++w) { cmn = min(cmn, s_amn[w]); cmx = max(cmx, s_amx[w]); }
  apk[(int64_t)row * npad + i] = valid ? min((uint32_t)adv - (uint32_t)cmn, kPkPoison) * 0x10001u : 0xFFFFFFFFu;
  // sub-chunk of 128 indices = 2 waves
  const int sub = threadIdx.x / kPkSub;
  const int32_t smn = min(s_amn[2 * sub], s_amn[2 * sub + 1]);
  const int32_t smx = max(s_amx[2 * sub], s_amx[2 * sub + 1]);
  apk_s[(int64_t)row * npad + i] = valid ? min((uint32_t)adv - (uint32_t)smn, kPkPoison) * 0x10001u : 0xFFFFFFFFu;
  if ((threadIdx.x & (kPkSub - 1)) == 0) {
    const bool any = smx >= smn;   // false when the sub-chunk lies entirely beyond n
    const int64_t range = (int64_t)smx - (int64_t)smn;
    ab_s[(int64_t)row * nsub + c * kPkSubs + sub] = any ? smn : 0;
    ar_s[(int64_t)row * nsub + c * kPkSubs + sub] = any ? (int32_t)(range < 0x7fffffffLL ? range : 0x7fffffffLL) : 0;
  }
  if (valid) bd[(int64_t)row * n + i] = bdv;
  if (threadIdx.x == 0) {
    ab[(int64_t)row * nchunk + c] = cmn;
    const int64_t range = (int64_t)cmx - (int64_t)cmn;
    ar[(int64_t)row * nchunk + c] = (int32_t)(range < 0x7fffffffLL ? range : 0x7fffffffLL);
  }
  if ((threadIdx.x & (kPkBlock - 1)) == 0) {
    const int j = c * (kPkChunk / kPkBlock) + threadIdx.x / kPkBlock;
    if (j < nblk) {
      int32_t mn = INT32_MAX, mx = INT32_MIN;
#pragma unroll
      for (int w = 0; w < kPkBlock / 64; ++w) { mn = min(mn, s_bmn[wave + w]); mx = max(mx, s_bmx[wave + w]); }
      bmn[(int64_t)row * nblk + j] = mn;
      bmx[(int64_t)row * nblk + j] = mx;
    }
  }
}

// Performance heuristic only (results are exact either way): samples up to 64 x 64
// (tile, chunk) pairs of a row, weighted by the number of chunks they stand for, and switches the
// packed path off for the row when less than half of its chunk-tiles would qualify -- a mostly
// unpackable row is better left to the 32-bit kernel alone.
__global__ __launch_bounds__(256) void decide_kernel(PackAux x, int n, int32_t* __restrict__ pack_ok) {
  __shared__ float s_yes[4], s_all[4];
  const int row = blockIdx.x;
  const int n_t2 = (n + kPkW - 1) / kPkW;
  float yes = 0.f, all = 0.f;
  if (pack_ok[row] != 0) {
    for (int j = threadIdx.x; j < 64 * 64; j += 256) {
      const int it = j / 64, ic = j % 64;
      const int nt = min(n_t2, 64);
      if (it >= nt) continue;
      const int T2 = (int)((int64_t)it * n_t2 / nt);
      const int nc = (min((T2 + 1) * kPkW, n) + kPkChunk - 1) / kPkChunk;   // chunks of this tile
      const int ns = min(nc, 64);
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
    yes = s_yes[0] + s_yes[1] + s_yes[2] + s_yes[3];
    all = s_all[0] + s_all[1] + s_all[2] + s_all[3];
    if (2.f * yes < all) pack_ok[row] = 0;
  }
}

template <typename T> struct RFor { static constexpr int value = 16; };

// Identity of the reduction as a host value (used to pre-fill outputs merged by atomics).
template <typename T, int OP> T host_identity() {
  if (std::numeric_limits<T>::has_infinity)
    return op_max(OP) ? -std::numeric_limits<T>::infinity() : std::numeric_limits<T>::infinity();
  return op_max(OP) ? std::numeric_limits<T>::lowest() : std::numeric_limits<T>::max();
}

struct Plan {
  int n_tiles, fold_width, seg;
  bool atomic;
  int64_t items;
};

// Cut the triangular iteration space (tiles of `width` outputs, chunks of `chunk` steps) into
// about RTC_TARGET_ITEMS work items of equal length.
Plan make_plan(int64_t batch, int64_t n, int width, int chunk) {
  Plan pl;
  pl.n_tiles = (int)((n + width - 1) / width);
  const double total_steps = (double)batch * (double)n * (pl.n_tiles + 1) * 0.5;
  // Measured on MI355X: items shorter than two chunks pay noticeably for their fixed cost
  // (staging, atomics), items much longer than that leave a ragged tail at the end of the launch.
  int64_t seg = (int64_t)(total_steps / (double)RTC_TARGET_ITEMS);
  seg = seg / chunk * chunk;
  if (seg < 2 * chunk) seg = total_steps / (2.0 * chunk) >= 8192.0 ? 2 * chunk : chunk;
  const int64_t span = ((int64_t)pl.n_tiles * width + chunk - 1) / chunk * chunk;  // longest s range, rounded up
  if (seg >= span) seg = span;
  pl.seg = (int)seg;
  auto nseg = [&](int k) { const int64_t e = (int64_t)(k + 1) * width; return (int)(((e < n ? e : n) + seg - 1) / seg); };
  pl.fold_width = 0;
  for (int k_lo = 0; k_lo <= pl.n_tiles - 1 - k_lo; ++k_lo) {
    const int k_hi = pl.n_tiles - 1 - k_lo;
    const int w = nseg(k_hi) + (k_lo != k_hi ? nseg(k_lo) : 0);
    if (w > pl.fold_width) pl.fold_width = w;
  }
  pl.atomic = nseg(pl.n_tiles - 1) > 1;
  pl.items = batch * (int64_t)((pl.n_tiles + 1) / 2) * pl.fold_width;
  return pl;
}

template <typename T> Plan make_plan(int64_t batch, int64_t n) {
  using TL = Tile<T, RFor<T>::value>;
  return make_plan(batch, n, TL::kW, TL::kChunk);
}

template <typename OutT, int OP>
void launch_fill(OutT* out, int64_t count, hipStream_t stream) {
  const int64_t want = (count + 2047) / 2048;
  const int blocks = (int)(want < 65535 ? want : 65535);
  hipLaunchKernelGGL(fill_kernel<OutT>, dim3(blocks), dim3(256), 0, stream, out, count,
                     host_identity<OutT, OP>());
}

// One launch of the generic kernel.  `force_atomic` is set when several kernels contribute to
// one output (the output is then already filled with the identity).
template <typename T, typename OutT, int OP>
int run_product(const T* a, int64_t stride_a, const T* b, int64_t stride_b, OutT* out, const OutT* cap,
                const int32_t* sel, int sel_want, int64_t batch, int64_t n, hipStream_t stream,
                bool prefilled, bool force_atomic, const int64_t* out_base) {
  constexpr int R = RFor<T>::value;
  const Plan pl = make_plan<T>(batch, n);
  if (pl.items > 0x7fffffffLL) return RTC_ERR_SHAPE;
  TropicalArgs args = {};
  args.a = a; args.b = b; args.out = out; args.cap = cap; args.sel = sel;
  args.stride_a = stride_a; args.stride_b = stride_b; args.sel_want = sel_want;
  args.n = (int32_t)n; args.batch = (int32_t)batch;
  args.n_tiles = pl.n_tiles; args.fold_width = pl.fold_width; args.seg = pl.seg;
  args.out_base = out_base;
  constexpr int dtype_code = std::is_same<T, int32_t>::value ? RTC_I32 : std::is_same<T, int64_t>::value ? RTC_I64 : RTC_F64;
  if (pl.atomic || force_atomic) {
    if (!prefilled) launch_fill<OutT, OP>(out, batch * n, stream);
    prof_begin(RTC_PROFILE_KIND(dtype_code, 0, OP), stream);
    hipLaunchKernelGGL((tropical_kernel<T, OutT, OP, R, true>), dim3((uint32_t)pl.items), dim3(64), 0,
                       stream, args);
  } else {
    prof_begin(RTC_PROFILE_KIND(dtype_code, 0, OP), stream);
    hipLaunchKernelGGL((tropical_kernel<T, OutT, OP, R, false>), dim3((uint32_t)pl.items), dim3(64), 0,
                       stream, args);
  }
  prof_end(stream);
  return hip_ok();
}

// Layout of the packed path's arrays inside the workspace.
struct PackLayout {
  int64_t npad, nchunk, nsub, nblk;
  size_t off_apk, off_apk_s, off_bd, off_ab, off_ar, off_ab_s, off_ar_s, off_bmn, off_bmx, off_rho, off_ok, bytes;
};

PackLayout pack_layout(int64_t batch, int64_t n) {
  PackLayout L;
  L.nchunk = (n + kPkChunk - 1) / kPkChunk;
  L.npad = L.nchunk * kPkChunk;
  L.nsub = L.nchunk * kPkSubs;
  L.nblk = (n + kPkBlock - 1) / kPkBlock;
  size_t o = 0;
  auto take = [&](size_t elems) { const size_t at = o; o += (elems * 4 + 255) / 256 * 256; return at; };
  L.off_apk = take((size_t)batch * L.npad);
  L.off_apk_s = take((size_t)batch * L.npad);
  L.off_bd = take((size_t)batch * n);
  L.off_ab = take((size_t)batch * L.nchunk);
  L.off_ar = take((size_t)batch * L.nchunk);
  L.off_ab_s = take((size_t)batch * L.nsub);
  L.off_ar_s = take((size_t)batch * L.nsub);
  L.off_bmn = take((size_t)batch * L.nblk);
  L.off_bmx = take((size_t)batch * L.nblk);
  L.off_rho = take((size_t)batch);
  L.off_ok = take((size_t)batch);
  L.bytes = o;
  return L;
}

// int32 product with the packed fast path.  f32 / g32 are int32 rows (the caller's own,
// or the narrowed copies of int64 rows); pack_ok / rho were written by the probe and the output
// is already filled with the identity.  `sel` (optional) restricts both kernels to rows with
// sel[row] == 1.
template <typename OutT, int OP>
int run_packed(const int32_t* f32, int64_t stride_f, const int32_t* g32, int64_t stride_g, OutT* out,
               const OutT* cap, const int32_t* sel, const int64_t* out_base, int64_t batch, int64_t n, char* wsp,
               const PackLayout& L, hipStream_t stream) {
  PackAux aux;
  aux.apk = reinterpret_cast<uint32_t*>(wsp + L.off_apk);
  aux.apk_s = reinterpret_cast<uint32_t*>(wsp + L.off_apk_s);
  aux.ab_s = reinterpret_cast<int32_t*>(wsp + L.off_ab_s);
  aux.ar_s = reinterpret_cast<int32_t*>(wsp + L.off_ar_s);
  aux.bd = reinterpret_cast<int32_t*>(wsp + L.off_bd);
  aux.ab = reinterpret_cast<int32_t*>(wsp + L.off_ab);
  aux.ar = reinterpret_cast<int32_t*>(wsp + L.off_ar);
  aux.bmn = reinterpret_cast<int32_t*>(wsp + L.off_bmn);
  aux.bmx = reinterpret_cast<int32_t*>(wsp + L.off_bmx);
  aux.rho = reinterpret_cast<int32_t*>(wsp + L.off_rho);
  aux.pack_ok = reinterpret_cast<int32_t*>(wsp + L.off_ok);
  aux.npad = (int32_t)L.npad; aux.nchunk = (int32_t)L.nchunk; aux.nsub = (int32_t)L.nsub;
  aux.nblk = (int32_t)L.nblk;
  if (batch * L.nchunk > 0x7fffffffLL) return RTC_ERR_SHAPE;
  // uniform operand: f for the convolution, g for the deconvolution; window operand: the other
  hipLaunchKernelGGL(prep_kernel, dim3((uint32_t)(batch * L.nchunk)), dim3(1024), 0, stream,
                     op_sub(OP) ? g32 : f32, op_sub(OP) ? stride_g : stride_f, op_sub(OP) ? f32 : g32,
                     op_sub(OP) ? stride_f : stride_g, (int)n, op_sub(OP), op_sub(OP) != op_max(OP), (int)L.npad, (int)L.nchunk, (int)L.nblk,
                     aux.rho, aux.pack_ok, const_cast<uint32_t*>(aux.apk), const_cast<uint32_t*>(aux.apk_s),
                     const_cast<int32_t*>(aux.ab_s), const_cast<int32_t*>(aux.ar_s), (int)L.nsub,
                     const_cast<int32_t*>(aux.bd), const_cast<int32_t*>(aux.ab), const_cast<int32_t*>(aux.ar),
                     const_cast<int32_t*>(aux.bmn), const_cast<int32_t*>(aux.bmx));
  hipLaunchKernelGGL(decide_kernel, dim3((uint32_t)batch), dim3(256), 0, stream, aux, (int)n,
                     const_cast<int32_t*>(aux.pack_ok));
  const Plan pk = make_plan(batch, n, kPkW, kPkChunk);
  const Plan pg = make_plan<int32_t>(batch, n);
  if (pk.items + pg.items > 0x7fffffffLL) return RTC_ERR_SHAPE;
  TropicalArgs ak = {};
  ak.out = out; ak.cap = cap; ak.sel = sel; ak.sel_want = 1; ak.out_base = out_base;
  ak.n = (int32_t)n; ak.batch = (int32_t)batch;
  ak.n_tiles = pk.n_tiles; ak.fold_width = pk.fold_width; ak.seg = pk.seg;
  ak.use_aux = 1; ak.aux = aux;
  // the 32-bit items work on the caller's rows and skip the chunks owned by the packed items
  TropicalArgs ag = ak;
  ag.a = op_sub(OP) ? g32 : f32; ag.stride_a = op_sub(OP) ? stride_g : stride_f;
  ag.b = op_sub(OP) ? f32 : g32; ag.stride_b = op_sub(OP) ? stride_f : stride_g;
  ag.n_tiles = pg.n_tiles; ag.fold_width = pg.fold_width; ag.seg = pg.seg;
  prof_begin(RTC_PROFILE_KIND(RTC_I32, 1, OP), stream);
  hipLaunchKernelGGL((fused_kernel<OutT, OP>), dim3((uint32_t)(pk.items + pg.items)), dim3(64), 0, stream,
                     ak, ag, (uint32_t)pk.items);
  prof_end(stream);
  return hip_ok();
}

}  // namespace

double g_packed_min_work = 1073741824.0;   // batch * n^2 from which the packed path is used

namespace {

bool packed_worthwhile(int64_t batch, int64_t n) {
  return (double)batch * (double)n * (double)n >= g_packed_min_work;
}

template <typename T, int OP>
int run_typed(const void* f, const void* g, void* out, int64_t batch, int64_t n, int64_t stride_f,
              int64_t stride_g, const void* cap, void* ws, size_t ws_bytes, int32_t* dev_flags,
              hipStream_t stream) {
  // convolution: uniform operand f, window g.  deconvolution: uniform g, window f (reversed).
  const T* a = static_cast<const T*>(op_sub(OP) ? g : f);
  const T* b = static_cast<const T*>(op_sub(OP) ? f : g);
  const int64_t sa = op_sub(OP) ? stride_g : stride_f;
  const int64_t sb = op_sub(OP) ? stride_f : stride_g;
  if constexpr (std::is_same<T, int32_t>::value) {
    const PackLayout L = pack_layout(batch, n);
    // tiny problems are launch-bound: the extra kernels of the packed path would only cost
    if (ws != nullptr && ws_bytes >= L.bytes && packed_worthwhile(batch, n)) {
      char* wsp = static_cast<char*>(ws);
      hipLaunchKernelGGL(probe_kernel<int32_t>, dim3((uint32_t)batch), dim3(1024), 0, stream,
                         static_cast<const int32_t*>(f), stride_f, static_cast<const int32_t*>(g), stride_g,
                         (int)n, op_sub(OP), reinterpret_cast<int32_t*>(wsp + L.off_ok),
                         reinterpret_cast<int32_t*>(wsp + L.off_rho), dev_flags);
      launch_fill<int32_t, OP>(static_cast<int32_t*>(out), batch * n, stream);
      return run_packed<int32_t, OP>(static_cast<const int32_t*>(f), stride_f,
                                         static_cast<const int32_t*>(g), stride_g, static_cast<int32_t*>(out),
                                         static_cast<const int32_t*>(cap), nullptr, nullptr, batch, n, wsp, L,
                                         stream);
    }
  }
  if (dev_flags != nullptr && std::numeric_limits<T>::is_integer) {
    hipLaunchKernelGGL(probe_kernel<T>, dim3((uint32_t)batch), dim3(1024), 0, stream,
                       static_cast<const T*>(f), stride_f, static_cast<const T*>(g), stride_g, (int)n,
                       op_sub(OP), (int32_t*)nullptr, (int32_t*)nullptr, dev_flags);
  }
  return run_product<T, T, OP>(a, sa, b, sb, static_cast<T*>(out), static_cast<const T*>(cap),
                                   nullptr, 0, batch, n, stream, false, false, nullptr);
}

// Bytes of the narrowed copies + selector that precede the packed-path arrays for int64 rows.
size_t narrow_base_offset(int64_t batch, int64_t n) {
  return ((size_t)(2 * batch * n + batch) * sizeof(int32_t) + 255) / 256 * 256;
}
size_t narrow_bytes(int64_t batch, int64_t n) {
  return narrow_base_offset(batch, n) + ((size_t)batch * sizeof(int64_t) + 255) / 256 * 256;
}

template <int OP>
int run_i64(const void* f, const void* g, void* out, int64_t batch, int64_t n, int64_t stride_f,
            int64_t stride_g, const void* cap, void* ws, int32_t* dev_flags, hipStream_t stream) {
  // workspace: [f32: batch*n][g32: batch*n][narrow_ok: batch][out_base: batch int64][packed-path arrays]
  int32_t* f32 = static_cast<int32_t*>(ws);
  int32_t* g32 = f32 + batch * n;
  int32_t* ok = g32 + batch * n;
  int64_t* base = reinterpret_cast<int64_t*>(static_cast<char*>(ws) + narrow_base_offset(batch, n));
  char* wsp = static_cast<char*>(ws) + narrow_bytes(batch, n);
  const PackLayout L = pack_layout(batch, n);
  hipLaunchKernelGGL(probe_narrow_kernel, dim3((uint32_t)batch), dim3(1024), 0, stream,
                     static_cast<const int64_t*>(f), stride_f, static_cast<const int64_t*>(g), stride_g,
                     (int)n, op_sub(OP), f32, g32, ok, base, reinterpret_cast<int32_t*>(wsp + L.off_ok),
                     reinterpret_cast<int32_t*>(wsp + L.off_rho), dev_flags);
  // Several kernels see every row; the selector makes each row run in exactly one family.
  // The output is filled once with the identity, before all of them.
  launch_fill<int64_t, OP>(static_cast<int64_t*>(out), batch * n, stream);
  int rc;
  if (packed_worthwhile(batch, n)) {
    rc = run_packed<int64_t, OP>(f32, n, g32, n, static_cast<int64_t*>(out), static_cast<const int64_t*>(cap),
                                 ok, base, batch, n, wsp, L, stream);
  } else {
    rc = run_product<int32_t, int64_t, OP>(op_sub(OP) ? g32 : f32, n, op_sub(OP) ? f32 : g32, n,
                                           static_cast<int64_t*>(out), static_cast<const int64_t*>(cap), ok, 1,
                                           batch, n, stream, true, true, base);
  }
  if (rc != RTC_OK) return rc;
  const int64_t* a = static_cast<const int64_t*>(op_sub(OP) ? g : f);
  const int64_t* b = static_cast<const int64_t*>(op_sub(OP) ? f : g);
  return run_product<int64_t, int64_t, OP>(a, op_sub(OP) ? stride_g : stride_f, b,
                                               op_sub(OP) ? stride_f : stride_g, static_cast<int64_t*>(out),
                                               static_cast<const int64_t*>(cap), ok, 0, batch, n, stream,
                                               true, true, nullptr);
}

}  // namespace

size_t tropical_workspace_bytes(int64_t batch, int64_t n, int dt) {
  if (dt == RTC_I64) return narrow_bytes(batch, n) + pack_layout(batch, n).bytes;
  if (dt == RTC_I32) return pack_layout(batch, n).bytes;
  return 0;
}

int launch_tropical(int op, const void* f, const void* g, void* out, int64_t batch, int64_t n,
                    int64_t stride_f, int64_t stride_g, int dt, const void* cap, void* ws,
                    size_t ws_bytes, int32_t* dev_flags, hipStream_t stream) {
  if (dt == RTC_I64 && (ws == nullptr || ws_bytes < tropical_workspace_bytes(batch, n, dt)))
    return RTC_ERR_WORKSPACE;
#define RTC_BY_OP(CALL)                                  \
  switch (op) {                                          \
    case RTC_OP_CONV: { constexpr int OP = 0; return CALL; }     \
    case RTC_OP_DECONV: { constexpr int OP = 1; return CALL; }   \
    case RTC_OP_MAXCONV: { constexpr int OP = 2; return CALL; }  \
    case RTC_OP_MINDECONV: { constexpr int OP = 3; return CALL; }\
    default: return RTC_ERR_MODE;                        \
  }
  switch (dt) {
    case RTC_I32:
      RTC_BY_OP((run_typed<int32_t, OP>(f, g, out, batch, n, stride_f, stride_g, cap, ws, ws_bytes, dev_flags, stream)))
    case RTC_F64:
      RTC_BY_OP((run_typed<double, OP>(f, g, out, batch, n, stride_f, stride_g, cap, ws, ws_bytes, dev_flags, stream)))
    case RTC_I64:
      RTC_BY_OP((run_i64<OP>(f, g, out, batch, n, stride_f, stride_g, cap, ws, dev_flags, stream)))
    default:
      return RTC_ERR_DTYPE;
  }
#undef RTC_BY_OP
}

}  // namespace rtc
