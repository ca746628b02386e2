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
#include <hip/hip_runtime.h>

#include <limits>

#include "rtc_internal.h"

namespace rtc {
namespace {

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
template <typename T, bool DECONV> struct Semiring {
  static __device__ __forceinline__ T identity() { return DECONV ? Lim<T>::lo() : Lim<T>::hi(); }
  static __device__ __forceinline__ T combine(T w, T u) { return DECONV ? wrap_sub(w, u) : wrap_add(w, u); }
  static __device__ __forceinline__ T reduce(T x, T y) { return DECONV ? sel_max(x, y) : sel_min(x, y); }
};

__device__ __forceinline__ void atomic_min(int32_t* p, int32_t v) { atomicMin(p, v); }
__device__ __forceinline__ void atomic_max(int32_t* p, int32_t v) { atomicMax(p, v); }
__device__ __forceinline__ void atomic_min(int64_t* p, int64_t v) { atomicMin((long long*)p, (long long)v); }
__device__ __forceinline__ void atomic_max(int64_t* p, int64_t v) { atomicMax((long long*)p, (long long)v); }
__device__ __forceinline__ void atomic_min(double* p, double v) { atomicMin(p, v); }
__device__ __forceinline__ void atomic_max(double* p, double v) { atomicMax(p, v); }

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
  int32_t fold_width;   // work items launched per folded tile pair (see item decode)
  int32_t seg;          // steps of s per segment, a multiple of the chunk length
};

#ifndef RTC_CHUNK_BLOCKS
#define RTC_CHUNK_BLOCKS 64
#endif
#ifndef RTC_TARGET_ITEMS
#define RTC_TARGET_ITEMS 65536
#endif

template <typename T, int R> struct Tile {
  static constexpr int kW = 64 * R;                          // outputs per wave
  static constexpr int kChunk = RTC_CHUNK_BLOCKS * R;        // steps of s per staged window
  static constexpr int kSlotBytes = R * (int)sizeof(T) + 16; // one group of R values + skew
  static constexpr int kSlots = 64 + kChunk / R;
  static constexpr int kVec = 16 / (int)sizeof(T);           // elements per 16-byte LDS read
};

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

template <typename T, typename OutT, bool DECONV, int R, bool ATOMIC>
__global__ __launch_bounds__(64) void tropical_kernel(const TropicalArgs p) {
  using SR = Semiring<T, DECONV>;
  using TL = Tile<T, R>;
  __shared__ __align__(16) unsigned char lds[TL::kSlots * TL::kSlotBytes];

  const int lane = threadIdx.x;
  const int n = p.n;
  // Work item = (tile, segment, row), rows fastest.  Tile k has ceil(s_end(k) / seg) segments,
  // which grows linearly with k; tile k is therefore folded with tile n_tiles-1-k so that
  // every folded pair owns about the same number of items and few launched workgroups are idle.
  uint32_t item = blockIdx.x;
  const int row = item % (uint32_t)p.batch;
  item /= (uint32_t)p.batch;
  const int j = item % (uint32_t)p.fold_width;
  const int k_lo = item / (uint32_t)p.fold_width;
  const int k_hi = p.n_tiles - 1 - k_lo;
  const int nseg_hi = (min((k_hi + 1) * TL::kW, n) + p.seg - 1) / p.seg;
  int tile, seg;
  if (j < nseg_hi) {
    tile = k_hi; seg = j;
  } else {
    if (k_lo == k_hi) return;
    tile = k_lo; seg = j - nseg_hi;
  }
  const int t0 = tile * TL::kW;
  const int s_end = min(t0 + TL::kW, n);
  const int sa = seg * p.seg;
  if (sa >= s_end) return;
  if (p.sel != nullptr && p.sel[row] != p.sel_want) return;
  const int sb = min(sa + p.seg, s_end);

  const T* __restrict__ arow = static_cast<const T*>(p.a) + (int64_t)row * p.stride_a;
  const T* __restrict__ brow = static_cast<const T*>(p.b) + (int64_t)row * p.stride_b;

  T acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = SR::identity();

  for (int sc = sa; sc < sb; sc += TL::kChunk) {
    const int ce = min(sc + TL::kChunk, sb);
    const int nblk = (ce - sc + R - 1) / R;
    // LDS slot q holds window elements [gbase + q*R, gbase + q*R + R)
    const int gbase = t0 - (sc + nblk * R);
    const int count = (64 + nblk) * R;
    __syncthreads();
    for (int e = lane; e < count; e += 64) {
      const int idx = gbase + e;
      T v = T(0);
      if (idx >= 0 && idx < n) v = brow[DECONV ? n - 1 - idx : idx];
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
        if (j < 0 || (s0 + R < n && j < 63)) {
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
        if (j < 0 || (s0 + R < n && j < 63)) {
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
  if (sa <= t0 && t0 < sb) {
    T b0[R];
#pragma unroll
    for (int q = 0; q < R; ++q) {
      const int idx = min(q, n - 1);
      b0[q] = brow[DECONV ? n - 1 - idx : idx];
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
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int t = tl + r;
    if (t < n) {
      const int ot = DECONV ? n - 1 - t : t;
      OutT v = (OutT)acc[r];
      if (crow) v = sel_min(v, crow[ot]);
      if (ATOMIC) {
        if (DECONV) atomic_max(&orow[ot], v); else atomic_min(&orow[ot], v);
      } else {
        orow[ot] = v;
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void fill_kernel(T* __restrict__ dst, int64_t count, T value) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += step) dst[i] = value;
}

// Range probe of one row pair.  Finds min/max of both rows, raises the overflow flag when
// the bounds do not prove that every candidate fits, and (int64 only) writes 32-bit copies
// of both rows plus a selector saying whether the 32-bit kernel may be used for this row.
template <typename T>
__global__ __launch_bounds__(1024) void probe_kernel(const T* __restrict__ f, int64_t stride_f,
                                                     const T* __restrict__ g, int64_t stride_g, int n,
                                                     bool deconv, int32_t* __restrict__ f32,
                                                     int32_t* __restrict__ g32,
                                                     int32_t* __restrict__ narrow_ok,
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
    if (f32) {
      f32[(int64_t)row * n + i] = (int32_t)fv;
      g32[(int64_t)row * n + i] = (int32_t)gv;
    }
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
      if (narrow_ok) {
        const T lim = (T)1 << 30;
        narrow_ok[row] = (fmin >= -lim && fmax < lim && gmin >= -lim && gmax < lim) ? 1 : 0;
      }
    }
  }
}

template <typename T> struct RFor { static constexpr int value = 16; };

// Identity of the reduction as a host value (used to pre-fill outputs merged by atomics).
template <typename T, bool DECONV> T host_identity() {
  if (std::numeric_limits<T>::has_infinity)
    return DECONV ? -std::numeric_limits<T>::infinity() : std::numeric_limits<T>::infinity();
  return DECONV ? std::numeric_limits<T>::lowest() : std::numeric_limits<T>::max();
}

struct Plan {
  int n_tiles, fold_width, seg;
  bool atomic;
  int64_t items;
};

// Cut the triangular iteration space into about RTC_TARGET_ITEMS work items of equal length.
template <typename T>
Plan make_plan(int64_t batch, int64_t n) {
  constexpr int R = RFor<T>::value;
  using TL = Tile<T, R>;
  Plan pl;
  pl.n_tiles = (int)((n + TL::kW - 1) / TL::kW);
  const double total_steps = (double)batch * (double)n * (pl.n_tiles + 1) * 0.5;
  // Measured on MI355X: items shorter than two chunks pay noticeably for their fixed cost
  // (staging, atomics), items much longer than that leave a ragged tail at the end of the launch.
  int64_t seg = (int64_t)(total_steps / (double)RTC_TARGET_ITEMS);
  seg = seg / TL::kChunk * TL::kChunk;
  if (seg < 2 * TL::kChunk) seg = total_steps / (2.0 * TL::kChunk) >= 8192.0 ? 2 * TL::kChunk : TL::kChunk;
  const int64_t span = (int64_t)pl.n_tiles * TL::kW;  // longest s range, rounded up
  if (seg >= span) seg = span;
  pl.seg = (int)seg;
  auto nseg = [&](int k) { const int64_t e = (int64_t)(k + 1) * TL::kW; return (int)(((e < n ? e : n) + seg - 1) / seg); };
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

template <typename T, typename OutT, bool DECONV>
int run_product(const T* a, int64_t stride_a, const T* b, int64_t stride_b, OutT* out, const OutT* cap,
                const int32_t* sel, int sel_want, int64_t batch, int64_t n, hipStream_t stream,
                bool prefilled) {
  constexpr int R = RFor<T>::value;
  const Plan pl = make_plan<T>(batch, n);
  if (pl.items > 0x7fffffffLL) return RTC_ERR_SHAPE;
  TropicalArgs args;
  args.a = a; args.b = b; args.out = out; args.cap = cap; args.sel = sel;
  args.stride_a = stride_a; args.stride_b = stride_b; args.sel_want = sel_want;
  args.n = (int32_t)n; args.batch = (int32_t)batch;
  args.n_tiles = pl.n_tiles; args.fold_width = pl.fold_width; args.seg = pl.seg;
  if (pl.atomic) {
    if (!prefilled) {
      const int64_t count = batch * n;
      const int64_t want = (count + 2047) / 2048;
      const int blocks = (int)(want < 65535 ? want : 65535);
      hipLaunchKernelGGL(fill_kernel<OutT>, dim3(blocks), dim3(256), 0, stream, out, count,
                         host_identity<OutT, DECONV>());
    }
    hipLaunchKernelGGL((tropical_kernel<T, OutT, DECONV, R, true>), dim3((uint32_t)pl.items), dim3(64), 0,
                       stream, args);
  } else {
    hipLaunchKernelGGL((tropical_kernel<T, OutT, DECONV, R, false>), dim3((uint32_t)pl.items), dim3(64), 0,
                       stream, args);
  }
  return hip_ok();
}

template <typename T, bool DECONV>
int run_typed(const void* f, const void* g, void* out, int64_t batch, int64_t n, int64_t stride_f,
              int64_t stride_g, const void* cap, void* ws, int32_t* dev_flags, hipStream_t stream) {
  // convolution: uniform operand f, window g.  deconvolution: uniform g, window f (reversed).
  const T* a = static_cast<const T*>(DECONV ? g : f);
  const T* b = static_cast<const T*>(DECONV ? f : g);
  const int64_t sa = DECONV ? stride_g : stride_f;
  const int64_t sb = DECONV ? stride_f : stride_g;
  if (dev_flags != nullptr && std::numeric_limits<T>::is_integer) {
    hipLaunchKernelGGL(probe_kernel<T>, dim3((uint32_t)batch), dim3(1024), 0, stream,
                       static_cast<const T*>(f), stride_f, static_cast<const T*>(g), stride_g, (int)n,
                       DECONV, (int32_t*)nullptr, (int32_t*)nullptr, (int32_t*)nullptr, dev_flags);
  }
  (void)ws;
  return run_product<T, T, DECONV>(a, sa, b, sb, static_cast<T*>(out), static_cast<const T*>(cap),
                                   nullptr, 0, batch, n, stream, false);
}

template <bool DECONV>
int run_i64(const void* f, const void* g, void* out, int64_t batch, int64_t n, int64_t stride_f,
            int64_t stride_g, const void* cap, void* ws, int32_t* dev_flags, hipStream_t stream) {
  // workspace: [f32: batch*n][g32: batch*n][narrow_ok: batch]
  int32_t* f32 = static_cast<int32_t*>(ws);
  int32_t* g32 = f32 + batch * n;
  int32_t* ok = g32 + batch * n;
  hipLaunchKernelGGL(probe_kernel<int64_t>, dim3((uint32_t)batch), dim3(1024), 0, stream,
                     static_cast<const int64_t*>(f), stride_f, static_cast<const int64_t*>(g), stride_g,
                     (int)n, DECONV, f32, g32, ok, dev_flags);
  // Both kernels see every row; the selector makes each row run in exactly one of them.
  // When segments are merged with atomics the output is filled once, before both.
  const Plan p32 = make_plan<int32_t>(batch, n);
  const Plan p64 = make_plan<int64_t>(batch, n);
  bool prefilled = false;
  if (p32.atomic || p64.atomic) {
    const int64_t count = batch * n;
    const int64_t want = (count + 2047) / 2048;
    const int blocks = (int)(want < 65535 ? want : 65535);
    hipLaunchKernelGGL(fill_kernel<int64_t>, dim3(blocks), dim3(256), 0, stream,
                       static_cast<int64_t*>(out), count, host_identity<int64_t, DECONV>());
    prefilled = true;
  }
  int rc = run_product<int32_t, int64_t, DECONV>(DECONV ? g32 : f32, n, DECONV ? f32 : g32, n,
                                                 static_cast<int64_t*>(out),
                                                 static_cast<const int64_t*>(cap), ok, 1, batch, n,
                                                 stream, prefilled);
  if (rc != RTC_OK) return rc;
  const int64_t* a = static_cast<const int64_t*>(DECONV ? g : f);
  const int64_t* b = static_cast<const int64_t*>(DECONV ? f : g);
  return run_product<int64_t, int64_t, DECONV>(a, DECONV ? stride_g : stride_f, b,
                                               DECONV ? stride_f : stride_g, static_cast<int64_t*>(out),
                                               static_cast<const int64_t*>(cap), ok, 0, batch, n, stream,
                                               prefilled);
}

}  // namespace

size_t tropical_workspace_bytes(int64_t batch, int64_t n, int dt) {
  if (dt == RTC_I64) return (size_t)(2 * batch * n + batch) * sizeof(int32_t) + 256;
  return 0;
}

int launch_tropical(bool deconv, const void* f, const void* g, void* out, int64_t batch, int64_t n,
                    int64_t stride_f, int64_t stride_g, int dt, const void* cap, void* ws,
                    size_t ws_bytes, int32_t* dev_flags, hipStream_t stream) {
  if (ws_bytes < tropical_workspace_bytes(batch, n, dt) || (dt == RTC_I64 && ws == nullptr))
    return RTC_ERR_WORKSPACE;
  switch (dt) {
    case RTC_I32:
      return deconv ? run_typed<int32_t, true>(f, g, out, batch, n, stride_f, stride_g, cap, ws, dev_flags, stream)
                    : run_typed<int32_t, false>(f, g, out, batch, n, stride_f, stride_g, cap, ws, dev_flags, stream);
    case RTC_F64:
      return deconv ? run_typed<double, true>(f, g, out, batch, n, stride_f, stride_g, cap, ws, dev_flags, stream)
                    : run_typed<double, false>(f, g, out, batch, n, stride_f, stride_g, cap, ws, dev_flags, stream);
    case RTC_I64:
      return deconv ? run_i64<true>(f, g, out, batch, n, stride_f, stride_g, cap, ws, dev_flags, stream)
                    : run_i64<false>(f, g, out, batch, n, stride_f, stride_g, cap, ws, dev_flags, stream);
    default:
      return RTC_ERR_DTYPE;
  }
}

}  // namespace rtc
