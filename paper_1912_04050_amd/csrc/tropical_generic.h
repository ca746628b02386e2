// Work-item body of the generic tropical product (int32 / int64 / fp64 arithmetic).
// Included by tropical.hip only.
#pragma once

#include "tropical_common.h"

namespace rtc {
namespace {

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
    // eight strides of loads in flight per trip (clamped addresses, no branches) instead of one
    // round trip to memory per stride
    constexpr int kStageBatch = 8;
    for (int e0 = lane; e0 < count; e0 += 64 * kStageBatch) {
      T raw[kStageBatch];
#pragma unroll
      for (int q = 0; q < kStageBatch; ++q) {
        const int idx = min(max(gbase + e0 + 64 * q, 0), n - 1);
        raw[q] = brow[rev ? n - 1 - idx : idx];
      }
#pragma unroll
      for (int q = 0; q < kStageBatch; ++q) {
        const int e = e0 + 64 * q, idx = gbase + e;
        const T v = (idx >= 0 && idx < n) ? raw[q] : T(0);
        if (e < count) *reinterpret_cast<T*>(lds + (e / R) * TL::kSlotBytes + (e % R) * (int)sizeof(T)) = v;
      }
    }
    if constexpr (R == 4) {
      // small tiles also stage the chunk of the uniform operand (see the grouped blocks below)
      T* ust = reinterpret_cast<T*>(lds + window_bytes<T, R>());
      if (!aux)
        for (int e = lane; e < nblk * R; e += 64) ust[e] = arow[min(sc + e, n - 1)];
    }
    __syncthreads();

    T w0[R], w1[R];
    load_group<T, R>(w0, lds, lane + nblk);
    int i = 0;
    if constexpr (R == 4) {
      // Small tiles: a block is only 16 candidates per lane, and a problem that takes them has about
      // one wavefront per CU, so nothing hides the loads that every block waits for: a scalar load
      // of the uniform operand that misses the scalar cache once per 64 bytes, and an LDS read.
      // Here the chunk of the uniform operand was staged in LDS with the window (all its cache
      // misses in flight at once), and four blocks are taken at a time: their 16 operand values and
      // four window groups are read together, with one wait for all.  Each block keeps its own
      // conditions (inside the row; from the tile's first output on, only the lanes behind it).
      if (!aux) {
        typedef T Vec __attribute__((ext_vector_type(TL::kVec)));
        const T* ust = reinterpret_cast<const T*>(lds + window_bytes<T, R>());
        for (; i + 4 <= nblk; i += 4) {
          T ug[4 * R], wa[R], wb[R], wc[R], wd[R];
          const Vec* up = reinterpret_cast<const Vec*>(ust + i * R);
#pragma unroll
          for (int q = 0; q < 4 * R / TL::kVec; ++q) {
            const Vec v = up[q];
#pragma unroll
            for (int e = 0; e < TL::kVec; ++e) ug[q * TL::kVec + e] = v[e];
          }
          load_group<T, R>(wa, lds, lane + nblk - i - 1);
          load_group<T, R>(wb, lds, lane + nblk - i - 2);
          load_group<T, R>(wc, lds, lane + nblk - i - 3);
          load_group<T, R>(wd, lds, lane + nblk - i - 4);
          T u0[R], u1[R], u2[R], u3[R];
#pragma unroll
          for (int k = 0; k < R; ++k) { u0[k] = ug[k]; u1[k] = ug[R + k]; u2[k] = ug[2 * R + k]; u3[k] = ug[3 * R + k]; }
          auto one = [&](int b, const T (&u)[R], const T (&lo)[R], const T (&hi)[R]) {
            const int s0 = sc + (i + b) * R;
            const int j = (s0 >= t0) ? (s0 - t0) / R : -1;
            if (j < 0 || (s0 + R < n && j < 63)) {
              if (lane > j) block_steps<SR, T, R>(acc, u, lo, hi);
            }
          };
          one(0, u0, wa, w0);
          one(1, u1, wb, wa);
          one(2, u2, wc, wb);
          one(3, u3, wd, wc);
#pragma unroll
          for (int k = 0; k < R; ++k) w0[k] = wd[k];
        }
      }
    }
    for (; i < nblk; i += 2) {
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
  static_assert(64 * (R + 1) * sizeof(T) <= window_bytes<T, R>(), "transpose buffer must fit the window buffer");
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
      if (p.out_base != nullptr) v += (OutT)(p.out_base[2 * row] + p.out_base[2 * row + 1] * ot);   // base + slope * output index
      if (crow) v = sel_min(v, crow[ot]);
      if (ATOMIC) {
        if (op_max(OP)) atomic_max(&orow[ot], v); else atomic_min(&orow[ot], v);
      } else {
        orow[ot] = v;
      }
    }
  }
}

}  // namespace
}  // namespace rtc
