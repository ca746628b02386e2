// Work-item body of the packed 16-bit tropical product (int32-exact arithmetic).
// Included by tropical.hip only.
#pragma once

#include "tropical_common.h"

namespace rtc {
namespace {

// ---- packed 16-bit kernel -----------------------------------------------------------------

typedef unsigned short us2 __attribute__((ext_vector_type(2)));
typedef _Float16 hf2 __attribute__((ext_vector_type(2)));

// R steps against the R packed accumulators of a lane (window groups as in block_steps).
// The combined values of a whole step (wide flavour) or of two steps (narrow flavour) are formed
// before the reductions so that no instruction reads the result of its immediate predecessor
// (the compiler otherwise pads each pair with a wait state).
//   wide:   saturating add / subtract, then one packed integer min / max per step
//   narrow: plain add / subtract, then one three-operand packed half-float minimum / maximum per
//           two steps; every value involved is a pattern below 0x7C00, where the half-float
//           order is the integer order (nested elementwise minimum / maximum compile to the
//           three-operand instruction)
template <bool MAXF, bool NARROW, int R>
__device__ __forceinline__ void block_steps_packed(uint32_t (&acc)[R], const uint32_t (&u)[R],
                                                   const uint32_t (&lo)[R], const uint32_t (&hi)[R]) {
  if constexpr (NARROW) {
#pragma unroll
    for (int k = 0; k < R; k += 2) {
      const us2 ua = __builtin_bit_cast(us2, u[k]), ub = __builtin_bit_cast(us2, u[k + 1]);
#pragma unroll
      for (int h = 0; h < R; h += R / 2) {   // half of the accumulators at a time: fewer live registers
        us2 s1[R / 2], s2[R / 2];
#pragma unroll
        for (int q = 0; q < R / 2; ++q) {
          const int r = h + q;
          const us2 wa = __builtin_bit_cast(us2, (r >= k) ? hi[r - k] : lo[R + r - k]);
          const us2 wb = __builtin_bit_cast(us2, (r >= k + 1) ? hi[r - k - 1] : lo[R + r - k - 1]);
          s1[q] = MAXF ? wa - ua : wa + ua;
          s2[q] = MAXF ? wb - ub : wb + ub;
        }
#pragma unroll
        for (int q = 0; q < R / 2; ++q) {
          const hf2 av = __builtin_bit_cast(hf2, acc[h + q]);
          const hf2 x1 = __builtin_bit_cast(hf2, s1[q]), x2 = __builtin_bit_cast(hf2, s2[q]);
          acc[h + q] = __builtin_bit_cast(
              uint32_t, MAXF ? __builtin_elementwise_maximum(__builtin_elementwise_maximum(av, x1), x2)
                             : __builtin_elementwise_minimum(__builtin_elementwise_minimum(av, x1), x2));
        }
      }
    }
  } else {
#pragma unroll
    for (int k = 0; k < R; ++k) {
      us2 s[R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const us2 w = __builtin_bit_cast(us2, (r >= k) ? hi[r - k] : lo[R + r - k]);
        const us2 uu = __builtin_bit_cast(us2, u[k]);
        s[r] = MAXF ? __builtin_elementwise_sub_sat(w, uu) : __builtin_elementwise_add_sat(w, uu);
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const us2 av = __builtin_bit_cast(us2, acc[r]);
        acc[r] = __builtin_bit_cast(uint32_t, MAXF ? __builtin_elementwise_max(av, s[r])
                                                     : __builtin_elementwise_min(av, s[r]));
      }
    }
  }
}

// Blocks [first, last) of the staged chunk (block i = steps sc + R i ...) against the packed
// accumulators; usrc is the packed uniform operand on the base of this run.
template <bool MAXF, bool NARROW, int R>
__device__ __forceinline__ void run_blocks(uint32_t (&acc)[R], const uint32_t* __restrict__ usrc,
                                           const unsigned char* lds, int lane, int sc, int nblk, int first,
                                           int last) {
  uint32_t w0[R], w1[R];
  load_group<uint32_t, R>(w0, lds, lane + nblk - first);
  for (int i = first; i < last; i += 2) {
    {
      const int s0 = sc + i * R;
      load_group<uint32_t, R>(w1, lds, lane + nblk - i - 1);
      uint32_t u[R];
#pragma unroll
      for (int k = 0; k < R; ++k) u[k] = usrc[s0 + k];
      block_steps_packed<MAXF, NARROW, R>(acc, u, w1, w0);
    }
    if (i + 1 < last) {
      const int s0 = sc + (i + 1) * R;
      load_group<uint32_t, R>(w0, lds, lane + nblk - i - 2);
      uint32_t u[R];
#pragma unroll
      for (int k = 0; k < R; ++k) u[k] = usrc[s0 + k];
      block_steps_packed<MAXF, NARROW, R>(acc, u, w0, w1);
    }
  }
}

// One wave owns 128 R outputs of the triangular product (R = 16, or 8 for short rows where the
// half-empty diagonal of a wide tile weighs more): the low 16 bits of every packed register belong
// to output t0 + R*lane + r, the high 16 bits to output t0 + 64 R + R*lane + r.
// Only the chunks / sub-chunks that chunk_plan() grants are processed; results merge into out with
// atomic min / max.  With w = bd - gb in [0, br] (window), u = ad - base in [0, ur] (uniform
// operand, 0 beyond the row's end, where every window position is poison) a 16-bit lane holds
//   min flavour:  w + lift + u, window poison P: every poisoned sum stays >= P > any candidate
//   max flavour:  w + lift - u, window poison Q: every poisoned difference stays <= Q < any candidate
//   wide:    min: lift 0, P = 0xFFFF (the add saturates);  max: lift 65535 - br, Q = 0 (the
//            subtraction saturates)
//   narrow:  with m = narrow_umax(br) >= ur:  min: lift 0, P = 0x7BFF - m;  max: lift 2m + 1,
//            Q = m;  nothing leaves [0, 0x7BFF]
template <typename OutT, int OP, int R>
__device__ __forceinline__ void packed_body(const TropicalArgs& p, unsigned char* lds, uint32_t item) {
  using TL = Tile<int32_t, R>;
  const int lane = threadIdx.x;
  const int n = p.n;
  int row, t0, sa, sb;
  constexpr int kHalf = 64 * R;          // outputs per 16-bit half of the tile
  if (!decode_item<2 * kHalf>(p, item, &row, &t0, &sa, &sb)) return;
  const PackAux& x = p.aux;
  if (x.pack_ok[row] == 0) return;
  const uint32_t* __restrict__ apk = x.apk + (int64_t)row * x.npad;
  const uint32_t* __restrict__ apk_s = x.apk_s + (int64_t)row * x.npad;
  const int32_t* __restrict__ bd = x.bd + (int64_t)row * n;
  const int32_t* __restrict__ ab = x.ab + (int64_t)row * x.nchunk;
  const int32_t* __restrict__ ab_s = x.ab_s + (int64_t)row * x.nsub;
  constexpr bool MAXF = op_max(OP);   // arithmetic flavour: subtract + max, or add + min
  constexpr int32_t kIdent = MAXF ? INT32_MIN : INT32_MAX;

  int32_t acc_lo[R], acc_hi[R];
#pragma unroll
  for (int r = 0; r < R; ++r) { acc_lo[r] = kIdent; acc_hi[r] = kIdent; }

  for (int sc = sa; sc < sb; sc += kPkChunk) {
    int32_t gb, br;
    const int c = sc / kPkChunk;
    const int plan = chunk_plan(x, row, t0 / kPkW, c, n, &gb, &br);
    if ((plan & 0xFF) == 0) continue;
    const int ce = min(sc + kPkChunk, sb);
    const int nblk = (ce - sc + R - 1) / R;
    const int gbase = t0 - (sc + nblk * R);
    const int count = (64 + nblk) * R;
    const bool narrow = (plan & kPlanNarrow) != 0;
    const uint32_t m = (uint32_t)narrow_umax(br);
    const uint32_t top = narrow ? (uint32_t)kPkNarrowTop : kPkPoison;        // largest value a lane may hold
    const uint32_t lift = MAXF ? (narrow ? 2u * m + 1u : 65535u - (uint32_t)br) : 0u;
    const uint32_t poison = MAXF ? (narrow ? m : 0u) : (narrow ? top - m : top);
    __syncthreads();
    for (int e = lane; e < count; e += 64) {
      const int il = gbase + e, ih = il + kHalf;
      uint32_t vl = poison, vh = poison;
      if (il >= 0 && il < n) vl = min((uint32_t)bd[il] - (uint32_t)gb + lift, top);
      if (ih >= 0 && ih < n) vh = min((uint32_t)bd[ih] - (uint32_t)gb + lift, top);
      *reinterpret_cast<uint32_t*>(lds + (e / R) * TL::kSlotBytes + (e % R) * 4) = vl | (vh << 16);
    }
    __syncthreads();

    // a run = a range of blocks that shares one base of the uniform operand: the whole chunk,
    // or one granted sub-chunk
    const bool whole = (plan & kPlanWhole) != 0;
    const uint32_t* __restrict__ usrc = whole ? apk : apk_s;
    const int nrun = whole ? 1 : kPkSubs;
    for (int run = 0; run < nrun; ++run) {
      const int first = whole ? 0 : run * (kPkSub / R);
      if (first >= nblk) break;
      if (!whole && !((plan >> run) & 1)) continue;
      const int last = whole ? nblk : min(first + kPkSub / R, nblk);
      const int32_t ubase = whole ? ab[c] : ab_s[c * kPkSubs + run];

      uint32_t acc[R];
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] = (MAXF ? 0u : top) * 0x10001u;
      if (narrow) run_blocks<MAXF, true, R>(acc, usrc, lds, lane, sc, nblk, first, last);
      else run_blocks<MAXF, false, R>(acc, usrc, lds, lane, sc, nblk, first, last);
      // fold the run into the 32-bit accumulators (detrended domain, wrap-around arithmetic:
      // every folded value is a true candidate, which fits); a lane on the poison side of the
      // threshold saw no existing candidate
      const uint32_t cb = MAXF ? (uint32_t)gb - (uint32_t)ubase - lift : (uint32_t)ubase + (uint32_t)gb;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const uint32_t vl = acc[r] & 0xFFFFu, vh = acc[r] >> 16;
        const bool okl = MAXF ? vl > poison : vl < poison, okh = MAXF ? vh > poison : vh < poison;
        const int32_t cl = okl ? (int32_t)(cb + vl) : kIdent;
        const int32_t ch = okh ? (int32_t)(cb + vh) : kIdent;
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
    for (int r = 0; r < R; ++r) xp[lane * (R + 1) + r] = half == 0 ? acc_lo[r] : acc_hi[r];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int xo = r * 64 + lane;
      const int t = t0 + half * kHalf + xo;
      const int32_t av = xp[xo + xo / R];
      if (t < n && av != kIdent) {
        const int ot = op_sub(OP) ? n - 1 - t : t;
        OutT v = (OutT)(op_sub(OP) ? wrap_sub(av, rho * t) : wrap_add(av, rho * t));
        if (p.out_base != nullptr) v += (OutT)(p.out_base[2 * row] + p.out_base[2 * row + 1] * ot);   // base + slope * output index
        if (crow) v = sel_min(v, crow[ot]);
        if (op_max(OP)) atomic_max(&orow[ot], v); else atomic_min(&orow[ot], v);
      }
    }
  }
}

}  // namespace
}  // namespace rtc
