// Work-item body of the packed 16-bit tropical product (int32-exact arithmetic).
// Included by tropical.hip only.
#pragma once

#include "tropical_common.h"

namespace rtc {
namespace {

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

}  // namespace
}  // namespace rtc
