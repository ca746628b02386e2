// Work-item body of the packed 16-bit tropical product (int32-exact arithmetic).
// Included by tropical.hip only.
#pragma once

#include "tropical_common.h"

namespace rtc {
namespace {

// ---- packed 16-bit kernel -----------------------------------------------------------------

typedef unsigned short us2 __attribute__((ext_vector_type(2)));
typedef _Float16 hf2 __attribute__((ext_vector_type(2)));

// The packed uniform operand of a row is stored in descending order of the step: a row has
// npad + 16 words and word [npad + 15 - g] holds step g (the value in both 16-bit halves), so that
// with ur = row + npad + 15, ur[-g] is step g.  The 16 steps of a block are one aligned run of 16
// consecutive words, and a pair of consecutive words is (step k+1, step k), the order in which the
// 64-bit additions of the narrow flavour need them.

// Wide flavour, R steps against the R packed accumulators of a lane (window groups as in
// block_steps): saturating add / subtract, then one packed integer min / max per step.  The
// combined values of a whole step are formed before the reductions so that no instruction reads
// the result of its immediate predecessor.  u[k] is step k of the block.
template <bool MAXF, int R>
__device__ __forceinline__ void block_steps_wide(uint32_t (&acc)[R], const uint32_t (&u)[R],
                                                 const uint32_t (&lo)[R], const uint32_t (&hi)[R]) {
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

// acc = min(acc, x1, x2) per 16-bit half, on patterns below 0x7C00, where the half-float order is
// the integer order (nested elementwise minimum compiles to the three-operand instruction).
__device__ __forceinline__ uint32_t pk_min3(uint32_t acc, uint32_t x1, uint32_t x2) {
  const hf2 a = __builtin_bit_cast(hf2, acc), b = __builtin_bit_cast(hf2, x1), c = __builtin_bit_cast(hf2, x2);
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_minimum(__builtin_elementwise_minimum(a, b), c));
}

// Narrow flavour (always add + min; the max flavours arrive here with the window mirrored, see
// packed_body).  Every 16-bit field stays below 0x7C00, so no addition carries into the next
// field and ONE 64-bit addition forms the candidates of two consecutive steps for both halves of
// an accumulator: (window[p], window[p+1]) as a register pair plus (step k+1, step k) as a
// scalar register pair; one three-operand packed minimum then folds both into the accumulator --
// two instructions for four candidates.  A register pair must start at an even register, i.e. at
// an even window position p = R + r - k - 1, so accumulators of odd r pair the steps (k, k+1) with
// k even and those of even r with k odd.  The even ones therefore take step 0 of a run's first
// block alone, pair step R-1 of every block with step 0 of the next, and take step R-1 of the
// run's last block alone.
//   ue[j] = (step k+1, step k) for k = R-2-2j, low word first, as loaded; the pairs for odd k,
//   uo[j] = (step k+1, step k) for k = R-1-2j, are put together from their words (scalar moves),
//   the low word of uo[0] being step 0 of the next block (`next0`; unused in a run's last block).
template <int R>
__device__ __forceinline__ void block_steps_narrow(uint32_t (&acc)[R], const uint64_t (&ue)[R / 2],
                                                   uint32_t next0, const uint32_t (&lo)[R],
                                                   const uint32_t (&hi)[R], bool first, bool last) {
  auto W = [&](int j) -> uint32_t { return j < R ? lo[j] : hi[j - R]; };
  uint64_t uo[R / 2];
  uo[0] = ((uint64_t)(uint32_t)ue[0] << 32) | next0;
#pragma unroll
  for (int j = 1; j < R / 2; ++j) uo[j] = ((uint64_t)(uint32_t)ue[j] << 32) | (uint32_t)(ue[j - 1] >> 32);
  if (first) {
    const uint32_t u0 = (uint32_t)(ue[R / 2 - 1] >> 32);
#pragma unroll
    for (int r = 0; r < R; r += 2) {
      const uint32_t c = W(R + r) + u0;
      acc[r] = pk_min3(acc[r], c, c);
    }
  }
  // descending j = ascending steps: the first half of the pairs reads window positions >= R only,
  // i.e. the group that is already in registers, while the new group and the next block's scalar
  // operand are still on their way
#pragma unroll
  for (int j = R / 2 - 1; j >= 0; --j) {
    uint64_t c[R / 2];
#pragma unroll
    for (int q = 0; q < R / 2; ++q) {          // odd accumulators, steps k = R-2-2j and k+1
      const int r = 2 * q + 1, pos = R + r - (R - 2 - 2 * j) - 1;
      c[q] = (((uint64_t)W(pos + 1) << 32) | W(pos)) + ue[j];
    }
#pragma unroll
    for (int q = 0; q < R / 2; ++q) acc[2 * q + 1] = pk_min3(acc[2 * q + 1], (uint32_t)c[q], (uint32_t)(c[q] >> 32));
    if (j == 0 && last) {                      // even accumulators, step R-1 alone
      const uint32_t ul = (uint32_t)(uo[0] >> 32);
#pragma unroll
      for (int q = 0; q < R / 2; ++q) {
        const uint32_t x = W(2 * q + 1) + ul;
        acc[2 * q] = pk_min3(acc[2 * q], x, x);
      }
    } else {                                   // even accumulators, steps k = R-1-2j and k+1
#pragma unroll
      for (int q = 0; q < R / 2; ++q) {
        const int r = 2 * q, pos = R + r - (R - 1 - 2 * j) - 1;
        c[q] = (((uint64_t)W(pos + 1) << 32) | W(pos)) + uo[j];
      }
#pragma unroll
      for (int q = 0; q < R / 2; ++q) acc[2 * q] = pk_min3(acc[2 * q], (uint32_t)c[q], (uint32_t)(c[q] >> 32));
    }
  }
}

// Scalar operand of the block of steps s0 .. s0+R-1 for the narrow flavour (see block_steps_narrow),
// and step s0+R, the word below them.  The loads are volatile so that they stay where they are
// written, one block ahead of their use: the compiler would otherwise move a load of invariant
// memory down to its first use, and the wave would wait for it there.
template <int R>
__device__ __forceinline__ void load_pairs(uint64_t (&ue)[R / 2], uint32_t* next0, const uint32_t* __restrict__ ur,
                                           int s0) {
  typedef uint32_t WordsR __attribute__((ext_vector_type(R)));
  // (the single word first: volatile accesses keep their order, and the block load is the one
  // that must not sink)
  *next0 = *reinterpret_cast<const volatile __attribute__((address_space(4))) uint32_t*>(as_invariant(ur - s0 - R));
  const WordsR v = *reinterpret_cast<const volatile __attribute__((address_space(4))) WordsR*>(as_invariant(ur - s0 - (R - 1)));
#pragma unroll
  for (int j = 0; j < R / 2; ++j) ue[j] = ((uint64_t)v[2 * j + 1] << 32) | v[2 * j];
}

// Blocks [first, last) of the staged chunk (block i = steps sc + R i ...) against the packed
// accumulators; ur is the packed uniform operand on the base of this run (ur[-g] = step g).
template <bool MAXF, bool NARROW, int R>
__device__ __forceinline__ void run_blocks(uint32_t (&acc)[R], const uint32_t* __restrict__ ur,
                                           const unsigned char* lds, int lane, int sc, int nblk, int first,
                                           int last) {
  uint32_t w0[R], w1[R];
  load_group<uint32_t, R>(w0, lds, lane + nblk - first);
  if constexpr (NARROW) {
    // the scalar operand is fetched one block ahead, so that a block starts on registers it
    // already has (its pairs are ordered accordingly) while its new window group arrives
    uint64_t ue[R / 2], ne[R / 2];
    uint32_t u16, n16;     // step 0 of the block after the one ue / ne belong to
    load_pairs<R>(ue, &u16, ur, sc + first * R);
    // The first block needs all of this at once.  Said here, once, it keeps the compiler from
    // placing the same wait at the top of the loop body, where it would also wait for the loads
    // that every iteration has just issued.
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
    for (int i = first; i < last; i += 2) {
      load_group<uint32_t, R>(w1, lds, lane + nblk - i - 1);
      load_pairs<R>(ne, &n16, ur, sc + min(i + 1, last - 1) * R);
      block_steps_narrow<R>(acc, ue, u16, w1, w0, i == first, i + 1 == last);
      if (i + 1 < last) {
        load_group<uint32_t, R>(w0, lds, lane + nblk - i - 2);
        load_pairs<R>(ue, &u16, ur, sc + min(i + 2, last - 1) * R);
        block_steps_narrow<R>(acc, ne, n16, w0, w1, false, i + 2 == last);
      }
    }
  } else {
    for (int i = first; i < last; i += 2) {
      {
        const int s0 = sc + i * R;
        load_group<uint32_t, R>(w1, lds, lane + nblk - i - 1);
        uint32_t u[R];
        const auto* up = as_invariant(ur - s0 - (R - 1));
#pragma unroll
        for (int k = 0; k < R; ++k) u[k] = up[R - 1 - k];
        block_steps_wide<MAXF, R>(acc, u, w1, w0);
      }
      if (i + 1 < last) {
        const int s0 = sc + (i + 1) * R;
        load_group<uint32_t, R>(w0, lds, lane + nblk - i - 2);
        uint32_t u[R];
        const auto* up = as_invariant(ur - s0 - (R - 1));
#pragma unroll
        for (int k = 0; k < R; ++k) u[k] = up[R - 1 - k];
        block_steps_wide<MAXF, R>(acc, u, w0, w1);
      }
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
//   narrow:  with m = narrow_umax(br) >= ur, always the min arithmetic w' + u with window poison
//            P = 0x7BFF - m: for the min flavours w' = w, for the max flavours the window is
//            mirrored, w' = br - w, and max(w - u) = br - min(w' + u); nothing leaves [0, 0x7BFF]
//            and no 16-bit field ever carries into its neighbour
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
  // descending order of the step: word [npad + 15 - g] of a row of npad + 16 words holds step g
  const uint32_t* __restrict__ apk = x.apk + (int64_t)row * (x.npad + 16) + x.npad + 15;
  const uint32_t* __restrict__ apk_s = x.apk_s + (int64_t)row * (x.npad + 16) + x.npad + 15;
  const int32_t* __restrict__ bd = x.bd + (int64_t)row * ((n + 3) & ~3);   // rows start 16-byte aligned
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
    const bool mirror = MAXF && narrow;      // max flavour in min arithmetic
    const uint32_t lift = MAXF && !narrow ? 65535u - (uint32_t)br : 0u;
    const uint32_t poison = narrow ? top - m : (MAXF ? 0u : top);
    __syncthreads();
    if (gbase >= 0 && gbase + count + kHalf <= n) {
      // every staged position exists (all chunks but those next to the diagonal and the row's
      // ends): four consecutive positions per lane, one 16-byte load per half, one 16-byte LDS
      // write, and no conditions.  A valid position needs no clamp either: the window base and
      // range that chunk_plan returns cover exactly the staged positions.
      typedef uint32_t Quad __attribute__((ext_vector_type(4)));
      const uint32_t shift = mirror ? (uint32_t)gb + (uint32_t)br : (uint32_t)gb - lift;
      for (int e0 = 4 * lane; e0 < count; e0 += 256 * 4) {
        Quad ql[4], qh[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int e = min(e0 + 256 * q, count - 4);
          ql[q] = *reinterpret_cast<const Quad*>(bd + gbase + e);
          qh[q] = *reinterpret_cast<const Quad*>(bd + gbase + e + kHalf);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int e = e0 + 256 * q;
          Quad o;
#pragma unroll
          for (int z = 0; z < 4; ++z) {
            const uint32_t vl = mirror ? shift - ql[q][z] : ql[q][z] - shift;
            const uint32_t vh = mirror ? shift - qh[q][z] : qh[q][z] - shift;
            o[z] = vl | (vh << 16);
          }
          if (e < count) *reinterpret_cast<Quad*>(lds + (e / R) * TL::kSlotBytes + (e % R) * 4) = o;
        }
      }
    } else {
      // eight strides of loads in flight per trip (clamped addresses, no branches): the staging
      // of a chunk is then four round trips to memory instead of thirty-two
      constexpr int kStageBatch = 8;
      for (int e0 = lane; e0 < count; e0 += 64 * kStageBatch) {
        int32_t rl[kStageBatch], rh[kStageBatch];
#pragma unroll
        for (int q = 0; q < kStageBatch; ++q) {
          const int il = gbase + e0 + 64 * q, ih = il + kHalf;
          rl[q] = bd[min(max(il, 0), n - 1)];
          rh[q] = bd[min(max(ih, 0), n - 1)];
        }
#pragma unroll
        for (int q = 0; q < kStageBatch; ++q) {
          const int e = e0 + 64 * q;
          const int il = gbase + e, ih = il + kHalf;
          const uint32_t wl = (uint32_t)rl[q] - (uint32_t)gb, wh = (uint32_t)rh[q] - (uint32_t)gb;
          const uint32_t vl = (il >= 0 && il < n) ? min(mirror ? (uint32_t)br - wl : wl + lift, top) : poison;
          const uint32_t vh = (ih >= 0 && ih < n) ? min(mirror ? (uint32_t)br - wh : wh + lift, top) : poison;
          if (e < count) *reinterpret_cast<uint32_t*>(lds + (e / R) * TL::kSlotBytes + (e % R) * 4) = vl | (vh << 16);
        }
      }
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
      for (int r = 0; r < R; ++r) acc[r] = (MAXF && !narrow ? 0u : top) * 0x10001u;
      if (narrow) run_blocks<MAXF, true, R>(acc, usrc, lds, lane, sc, nblk, first, last);
      else run_blocks<MAXF, false, R>(acc, usrc, lds, lane, sc, nblk, first, last);
      // fold the run into the 32-bit accumulators (detrended domain, wrap-around arithmetic:
      // every folded value is a true candidate, which fits); a lane on the poison side of the
      // threshold saw no existing candidate
      const uint32_t cb = MAXF ? (uint32_t)gb - (uint32_t)ubase - lift + (mirror ? (uint32_t)br : 0u)
                               : (uint32_t)ubase + (uint32_t)gb;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const uint32_t vl = acc[r] & 0xFFFFu, vh = acc[r] >> 16;
        const bool up = MAXF && !narrow;       // the lane holds a maximum (else a minimum)
        const bool okl = up ? vl > poison : vl < poison, okh = up ? vh > poison : vh < poison;
        const int32_t cl = okl ? (int32_t)(mirror ? cb - vl : cb + vl) : kIdent;
        const int32_t ch = okh ? (int32_t)(mirror ? cb - vh : cb + vh) : kIdent;
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
