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
