// int64 rows whose values span more than 32 bits but vary slowly: the generic product in 32-bit
// arithmetic on values re-based per chunk.  Included by tropical.hip only.
//
// A work item of the generic kernel meets, per chunk of 1024 steps, 1024 consecutive values of
// the uniform operand and a window of at most 2048 consecutive values of the window operand
// (both aligned to 1024).  When for every chunk and window of a row pair
//     range(chunk of a) + range(window of b) <= 2^31 - 2
// (decided per row from tables of block minima / maxima; with `detrend`, of the rows minus the
// pair's common slope times the index, see common_slope, so that steep lines of different slopes
// qualify as long as the slopes differ by less than about 10^6 per step), each chunk's candidates,
// taken relative to (min of the chunk) +- (min of the window), fit 32 bits: the chunk is reduced by the
// 32-bit inner loop (1.5 VALU instructions per candidate instead of the 4 to 5 of the 64-bit one)
// and its partial results are folded into 64-bit accumulators with the bases added back, once
// per chunk.  Every candidate is the exact integer of the definition, so the result has the same
// bits.  Rows that do not qualify stay with the 64-bit kernel.
#pragma once

#include "tropical_common.h"
#include "tropical_generic.h"
#include "tropical_prepare.h"

namespace rtc {
namespace {

constexpr int kSelRebased = -1;        // selector of the row pairs this path takes (narrow_ok array)
// Row pairs that do not qualify but whose values all lie within +-2^51: every sum and difference
// of two of them is an integer below 2^53 in magnitude, which fp64 adds, subtracts and compares
// exactly -- they run through the fp64 kernel (one add and one min per candidate instead of the
// 64-bit integer kernel's four to five instructions) on copies converted to double, and the
// results convert back exactly.
constexpr int kSelDouble = -2;
constexpr int64_t kDoubleExact = (int64_t)1 << 51;
constexpr int kWideR = 16;
constexpr int kWideBlock = Tile<int32_t, kWideR>::kChunk;   // 1024: chunk of steps = tile of outputs
static_assert(kWideBlock == Tile<int32_t, kWideR>::kW, "windows are pairs of aligned blocks");
constexpr uint64_t kWideBudget = 0x7ffffffeull;

__host__ __device__ inline int wide_blocks(int64_t n) { return (int)((n + kWideBlock - 1) / kWideBlock); }
inline size_t wide_table_elems(int64_t batch, int64_t n) { return (size_t)batch * wide_blocks(n) * 4 + (size_t)batch; }   // tables, then the slope per row

// One workgroup of 16 wavefronts per row pair with sel[row] == 0.
// tab[(row * nb + m) * 4 + {0, 1, 2, 3}] = min a, max a, min b, max b over block m, where a is
// the uniform operand at steps [1024 m, 1024 m + 1024) and b the window operand at the same
// window indices (reversed row for the deconvolutions); each wavefront takes a contiguous range
// of blocks (plus the one before it, for the window that straddles the boundary).  Then:
// largest range of a chunk of a plus largest range of a window of b (a pair of neighbouring
// blocks) within the budget -> sel[row] = kSelRebased.
constexpr int kWideThreads = 1024;
template <int OP>
__global__ __launch_bounds__(kWideThreads) void wide_tables_kernel(const int64_t* __restrict__ f, int64_t stride_f,
                                                                   const int64_t* __restrict__ g, int64_t stride_g,
                                                                   int32_t* __restrict__ sel, int64_t* __restrict__ tab,
                                                                   int64_t* __restrict__ slopes,
                                                                   double* __restrict__ a_dbl, double* __restrict__ b_dbl,
                                                                   int n, int nb, bool detrend) {
  constexpr int kWaves = kWideThreads / 64;
  __shared__ uint64_t red[2][kWaves];
  __shared__ int64_t s_raw[4][kWaves];
  __shared__ int64_t s_rho;
  const int row = blockIdx.x;
  if (sel[row] != 0) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t* a = op_sub(OP) ? g + (int64_t)row * stride_g : f + (int64_t)row * stride_f;
  const int64_t* b = op_sub(OP) ? f + (int64_t)row * stride_f : g + (int64_t)row * stride_g;
  if (threadIdx.x == 0) s_rho = detrend ? common_slope(a, b, n) : 0;     // (64-bit divisions: one thread)
  __syncthreads();
  const uint64_t rho = (uint64_t)s_rho;
  int64_t ra_lo = Lim<int64_t>::hi(), ra_hi = Lim<int64_t>::lo(), rb_lo = ra_lo, rb_hi = ra_hi;   // extrema of the rows as they are
  const int per = (nb + kWaves - 1) / kWaves;
  const int first = wave * per, last = min(first + per, nb);       // this wavefront's blocks [first, last)
  uint64_t ra = 0, rb = 0;
  int64_t prev_lo = 0, prev_hi = 0;
  bool have_prev = false;
  for (int m = max(first - 1, 0); m < last; ++m) {
    int64_t amin = Lim<int64_t>::hi(), amax = Lim<int64_t>::lo(), bmin = amin, bmax = amax;
#pragma unroll 8
    for (int i = lane; i < kWideBlock; i += 64) {
      const int idx = min(m * kWideBlock + i, n - 1);          // past the end: the last value again
      const int bi = op_sub(OP) ? n - 1 - idx : idx;
      const int64_t ar = a[idx], br = b[bi];
      ra_lo = sel_min(ra_lo, ar); ra_hi = sel_max(ra_hi, ar);
      rb_lo = sel_min(rb_lo, br); rb_hi = sel_max(rb_hi, br);
      if (m >= first) {     // copies for the fp64 kernel (exact if the pair ends up there), rows as they are
        a_dbl[(int64_t)row * n + idx] = (double)ar;
        b_dbl[(int64_t)row * n + bi] = (double)br;
      }
      const int64_t av = (int64_t)((uint64_t)ar - rho * (uint64_t)idx), bv = (int64_t)((uint64_t)br - rho * (uint64_t)bi);
      amin = sel_min(amin, av); amax = sel_max(amax, av);
      bmin = sel_min(bmin, bv); bmax = sel_max(bmax, bv);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      amin = sel_min(amin, __shfl_xor(amin, off)); amax = sel_max(amax, __shfl_xor(amax, off));
      bmin = sel_min(bmin, __shfl_xor(bmin, off)); bmax = sel_max(bmax, __shfl_xor(bmax, off));
    }
    if (m >= first) {
      if (lane == 0) {
        int64_t* t = tab + ((int64_t)row * nb + m) * 4;
        t[0] = amin; t[1] = amax; t[2] = bmin; t[3] = bmax;
      }
      const uint64_t r = (uint64_t)amax - (uint64_t)amin;
      ra = r > ra ? r : ra;
    }
    // window = this block together with the one before it (alone if there is none)
    const int64_t lo = have_prev ? sel_min(prev_lo, bmin) : bmin, hi = have_prev ? sel_max(prev_hi, bmax) : bmax;
    const uint64_t w = (uint64_t)hi - (uint64_t)lo;
    if (m >= first) rb = w > rb ? w : rb;
    prev_lo = bmin; prev_hi = bmax; have_prev = true;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    ra_lo = sel_min(ra_lo, __shfl_xor(ra_lo, off)); ra_hi = sel_max(ra_hi, __shfl_xor(ra_hi, off));
    rb_lo = sel_min(rb_lo, __shfl_xor(rb_lo, off)); rb_hi = sel_max(rb_hi, __shfl_xor(rb_hi, off));
  }
  if (lane == 0) {
    red[0][wave] = ra; red[1][wave] = rb;
    s_raw[0][wave] = ra_lo; s_raw[1][wave] = ra_hi; s_raw[2][wave] = rb_lo; s_raw[3][wave] = rb_hi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < kWaves; ++w) {
      ra = red[0][w] > ra ? red[0][w] : ra; rb = red[1][w] > rb ? red[1][w] : rb;
      ra_lo = sel_min(ra_lo, s_raw[0][w]); ra_hi = sel_max(ra_hi, s_raw[1][w]);
      rb_lo = sel_min(rb_lo, s_raw[2][w]); rb_hi = sel_max(rb_hi, s_raw[3][w]);
    }
    // with a slope removed the arithmetic is exact only for rows whose own ranges stay below 2^62
    const bool exact = rho == 0 || ((((uint64_t)ra_hi - (uint64_t)ra_lo) >> 62) == 0 && (((uint64_t)rb_hi - (uint64_t)rb_lo) >> 62) == 0);
    slopes[row] = (int64_t)rho;
    const bool small = ra_lo >= -kDoubleExact && ra_hi <= kDoubleExact && rb_lo >= -kDoubleExact && rb_hi <= kDoubleExact;
    if (exact && ra <= kWideBudget && rb <= kWideBudget && ra + rb <= kWideBudget) sel[row] = kSelRebased;
    else if (small) sel[row] = kSelDouble;
  }
}

// Work item of the re-based product: tropical_body's walk over the chunks of a segment with a
// 32-bit inner loop per chunk and 64-bit accumulators across chunks.
template <int OP>
__device__ __forceinline__ void rebased_body(const TropicalArgs& p, const int64_t* __restrict__ tab,
                                             const int64_t* __restrict__ slopes, int nb, unsigned char* lds,
                                             uint32_t item) {
  constexpr int R = kWideR;
  using SR = Semiring<int32_t, OP>;
  using SR64 = Semiring<int64_t, OP>;
  using TL = Tile<int32_t, R>;
  const int lane = threadIdx.x;
  const int n = p.n;
  int row, t0, sa, sb;
  if (!decode_item<TL::kW>(p, item, &row, &t0, &sa, &sb)) return;
  constexpr bool rev = op_sub(OP);
  const int64_t* __restrict__ arow = static_cast<const int64_t*>(p.a) + (int64_t)row * p.stride_a;
  const int64_t* __restrict__ brow = static_cast<const int64_t*>(p.b) + (int64_t)row * p.stride_b;
  const int64_t* __restrict__ trow = tab + (int64_t)row * nb * 4;
  const uint64_t rho = (uint64_t)slopes[row];     // common slope removed from both rows (0: none)
  // value of the window operand at window index idx / of the uniform operand at step s, slope removed
  auto b_at = [&](int idx) { const int ri = rev ? n - 1 - idx : idx; return (uint64_t)brow[ri] - rho * (uint64_t)ri; };
  auto a_at = [&](int s) { return (uint64_t)arow[s] - rho * (uint64_t)s; };

  int64_t acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = SR64::identity();
  // fold a chunk's 32-bit results, taken relative to `base`, into the 64-bit accumulators
  auto fold = [&](const int32_t (&part)[R], int64_t base) {
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (part[r] != SR::identity()) acc[r] = SR64::reduce(acc[r], wrap_add((int64_t)part[r], base));
  };

  for (int sc = sa; sc < sb; sc += TL::kChunk) {
    const int ce = min(sc + TL::kChunk, sb);
    const int nblk = (ce - sc + R - 1) / R;
    // bases: the chunk's block of a, the window's pair of blocks of b (the lower one may not exist)
    const int64_t abase = trow[(sc / kWideBlock) * 4 + 0];
    const int mw = (t0 - sc) / kWideBlock;
    int64_t wbase = trow[mw * 4 + 2];
    if (mw > 0) wbase = sel_min(wbase, trow[(mw - 1) * 4 + 2]);
    // LDS slot q holds window elements [gbase + q*R, gbase + q*R + R), re-based
    const int gbase = t0 - (sc + nblk * R);
    const int count = (64 + nblk) * R;
    __syncthreads();
    for (int e = lane; e < count; e += 64) {
      const int idx = gbase + e;
      int32_t v = 0;
      if (idx >= 0 && idx < n) v = (int32_t)(uint32_t)(b_at(idx) - (uint64_t)wbase);
      *reinterpret_cast<int32_t*>(lds + (e / R) * TL::kSlotBytes + (e % R) * 4) = v;
    }
    __syncthreads();

    int32_t part[R];
#pragma unroll
    for (int r = 0; r < R; ++r) part[r] = SR::identity();
    int32_t w0[R], w1[R];
    load_group<int32_t, R>(w0, lds, lane + nblk);
    for (int i = 0; i < nblk; i += 2) {
      {
        const int s0 = sc + i * R;
        load_group<int32_t, R>(w1, lds, lane + nblk - i - 1);
        const int j = (s0 >= t0) ? (s0 - t0) / R : -1;
        if (j < 0 || (s0 + R < n && j < 63)) {
          int32_t u[R];
#pragma unroll
          for (int k = 0; k < R; ++k) u[k] = (int32_t)(uint32_t)(a_at(s0 + k) - (uint64_t)abase);
          if (lane > j) block_steps<SR, int32_t, R>(part, u, w1, w0);
        }
      }
      if (i + 1 < nblk) {
        const int s0 = sc + (i + 1) * R;
        load_group<int32_t, R>(w0, lds, lane + nblk - i - 2);
        const int j = (s0 >= t0) ? (s0 - t0) / R : -1;
        if (j < 0 || (s0 + R < n && j < 63)) {
          int32_t u[R];
#pragma unroll
          for (int k = 0; k < R; ++k) u[k] = (int32_t)(uint32_t)(a_at(s0 + k) - (uint64_t)abase);
          if (lane > j) block_steps<SR, int32_t, R>(part, u, w0, w1);
        }
      }
    }
    fold(part, op_sub(OP) ? wrap_sub(wbase, abase) : wrap_add(wbase, abase));
  }

  const int tl = t0 + lane * R;
  // the lane's own triangle: steps s = tl+k against outputs tl+r, r >= k, window index r-k
  if (sa <= t0 && t0 < sb) {
    const int64_t abase = trow[(t0 / kWideBlock) * 4 + 0], wbase = trow[2];
    int32_t b0[R], part[R];
#pragma unroll
    for (int q = 0; q < R; ++q) {
      const int idx = min(q, n - 1);
      b0[q] = (int32_t)(uint32_t)(b_at(idx) - (uint64_t)wbase);
      part[q] = SR::identity();
    }
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const int32_t ak = (int32_t)(uint32_t)(a_at(min(tl + k, n - 1)) - (uint64_t)abase);
#pragma unroll
      for (int r = k; r < R; ++r) part[r] = SR::reduce(part[r], SR::combine(b0[r - k], ak));
    }
    fold(part, op_sub(OP) ? wrap_sub(wbase, abase) : wrap_add(wbase, abase));
  }

  int64_t* __restrict__ orow = static_cast<int64_t*>(p.out) + (int64_t)row * n;
  const int64_t* __restrict__ crow = p.cap ? static_cast<const int64_t*>(p.cap) + (int64_t)row * n : nullptr;
  // transpose through LDS as the generic kernel does, then merge with atomics
  static_assert(64 * (R + 1) * sizeof(int64_t) <= lds_bytes<int32_t, R>(), "transpose buffer must fit the window buffer");
  int64_t* xp = reinterpret_cast<int64_t*>(lds);
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) xp[lane * (R + 1) + r] = acc[r];
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int x = r * 64 + lane;
    const int t = t0 + x;
    if (t < n) {
      const int ot = op_sub(OP) ? n - 1 - t : t;
      int64_t v = xp[x + x / R];
      if (v == SR64::identity()) continue;        // this item saw no candidate of that output
      v = (int64_t)((uint64_t)v + rho * (uint64_t)ot);   // the slope's share of every candidate of output ot
      if (crow) v = sel_min(v, crow[ot]);
      if (op_max(OP)) atomic_max(&orow[ot], v); else atomic_min(&orow[ot], v);
    }
  }
}

// `parts` workgroups per row, each looks at its row's selector once and either leaves or walks
// every parts-th item of the row (items are numbered rows fastest).
template <int OP>
__global__ __launch_bounds__(64) void rebased_rows_kernel(const TropicalArgs p, const int64_t* __restrict__ tab,
                                                          const int64_t* __restrict__ slopes, int nb,
                                                          uint32_t items_per_row, uint32_t parts) {
  __shared__ __align__(16) unsigned char lds[lds_bytes<int32_t, kWideR>()];
  const uint32_t row = blockIdx.x % (uint32_t)p.batch, part = blockIdx.x / (uint32_t)p.batch;
  if (p.sel[row] != p.sel_want) return;
  for (uint32_t j = part; j < items_per_row; j += parts) rebased_body<OP>(p, tab, slopes, nb, lds, j * (uint32_t)p.batch + row);
}

}  // namespace
}  // namespace rtc
