// Tropical products of row pairs whose shape makes most candidates superfluous (integers only;
// every candidate that is formed is the definition's exact integer, so the results have the same
// bits as the general kernels'):
//   both rows convex / concave    the ends of the candidate range, or a bisection   (structured_kernel)
//   one row convex / concave      monotone optima: anchors, then brackets          (bracket_anchor_body)
//   one row periodic              a scan along residue classes, then a window of one period
//                                 (period_kernel, periodic_scan_body, periodic_product_body)
// Three launches serve all of them: structured_first_kernel, bracket_fine_kernel,
// structured_kernel.  Included by tropical.hip only.
#pragma once

#include "tropical_common.h"
#include "tropical_prepare.h"

namespace rtc {
namespace {

constexpr int kBracketCoarse = 4096;   // spacing of the anchors that scan all their candidates
constexpr int kBracketFine = 64;       // spacing of the anchors that scan between two coarse optima

__host__ __device__ inline int bracket_anchors(int64_t n, int step) { return (int)((n + step - 1) / step) + 1; }

// Bracket path, the anchors.  When the operand indexed by t is convex (min) / concave (max), the
// leftmost optimal j of output t is monotone in t: nondecreasing for the convolutions,
// nonincreasing for the deconvolutions (Monge property of c_t(j); candidates that do not exist
// count as +-infinity and keep it), so the leftmost optimum of an output lies between the
// leftmost optima of any two outputs around it.  Anchor a of a level with spacing STEP is output
// t_a = min(STEP a, n-1); one workgroup finds its leftmost optimal j and stores it in
// jstar[row][a].  The coarse level (coarse == nullptr; the workgroup's four wavefronts share one
// anchor) scans all candidates of its anchors, the fine level (one anchor per wavefront) only
// those between the optima of the two coarse anchors around it, and
// structured_kernel those between two fine anchors: about n^2 / 8192 + 128 n candidates per row
// pair instead of n^2 / 2.
template <typename T, int OP, int STEP, bool SHARED>
__device__ __forceinline__ void bracket_anchor_body(const T* __restrict__ f, int64_t stride_f,
                                                    const T* __restrict__ g, int64_t stride_g,
                                                    const int32_t* __restrict__ sel,
                                                    const int32_t* __restrict__ coarse, int coarse_anchors,
                                                    int32_t* __restrict__ jstar, int n, int anchors, int block) {
  constexpr int kWaves = 4;
  constexpr int kThreads = SHARED ? 256 : 64;    // lanes that share one anchor
  constexpr int kNone = 0x7fffffff;
  __shared__ T s_val[kWaves];
  __shared__ int s_idx[kWaves];
  const int groups = SHARED ? anchors : (anchors + kWaves - 1) / kWaves;   // workgroups per row
  const int row = block / groups;
  const int code = sel[row];
  if (code != kSelBracket && code != kSelBracketSwapped) return;
  const int lane = SHARED ? threadIdx.x : threadIdx.x & 63;
  const int a = SHARED ? block % groups : (block % groups) * kWaves + (threadIdx.x >> 6);
  if (a >= anchors) return;                       // SHARED: never; else whole wavefronts, and no barrier follows
  const int t = min(a * STEP, n - 1);
  const bool swapped = code == kSelBracketSwapped;       // convolutions only: they commute
  const T* fr = (swapped ? g + (int64_t)row * stride_g : f + (int64_t)row * stride_f);
  const T* gr = (swapped ? f + (int64_t)row * stride_f : g + (int64_t)row * stride_g);
  const int m = op_sub(OP) ? n - 1 - t : t;
  int lo = 0, hi = m;
  if (coarse != nullptr) {
    const int32_t* cs = coarse + (int64_t)row * coarse_anchors + min(t / kBracketCoarse, coarse_anchors - 2);
    const int ja = cs[0], jb = cs[1];            // optima of the coarse anchors below and above t
    // (clamped: with exact sums 0 <= lo <= hi <= m holds by monotonicity; rows that break the
    // API's no-overflow precondition must still index inside the row)
    lo = min(max(op_sub(OP) ? jb : ja, 0), m);
    hi = max(min(op_sub(OP) ? ja : jb, m), lo);
  }
  T best = Semiring<T, OP>::identity();
  int best_j = kNone;
#pragma unroll 4
  for (int j = lo + lane; j <= hi; j += kThreads) {
    const T c = op_sub(OP) ? wrap_sub(fr[t + j], gr[j]) : wrap_add(fr[j], gr[t - j]);
    if (best_j == kNone || (op_max(OP) ? c > best : c < best)) { best = c; best_j = j; }   // ascending j: the first optimum stays
  }
  // leftmost optimum over the workgroup: better value, or equal value and smaller j
  auto merge = [&](T v, int j) {
    if (j == kNone) return;
    if (best_j == kNone || (op_max(OP) ? v > best : v < best) || (v == best && j < best_j)) { best = v; best_j = j; }
  };
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) merge(__shfl_xor(best, off), __shfl_xor(best_j, off));
  if constexpr (SHARED) {
    if ((threadIdx.x & 63) == 0) { s_val[threadIdx.x >> 6] = best; s_idx[threadIdx.x >> 6] = best_j; }
    __syncthreads();
    if (threadIdx.x == 0)
      for (int w = 1; w < kWaves; ++w) merge(s_val[w], s_idx[w]);
  }
  if (lane == 0) jstar[(int64_t)row * anchors + a] = best_j;
}

// ---- periodic operands -------------------------------------------------------------------------
// A row w is periodic from index 1 on with period p and increment c when w[i+p] = w[i] + c for
// all 1 <= i, i+p <= n-1 (periodic event streams with jitter, TDMA service; index 0 is left out
// because such curves are 0 there whatever follows).  With the candidates of the convolution
// (f (x) w)[t] = min_j f[t-j] + w[j] grouped by j = 1 + r + q p, 0 <= r < p:
//   F[u]   = min_{q >= 0, u - q p >= 0} f[u - q p] + q c        (one scan along each residue class)
//   out[t] = min( f[t] + w[0],  min_{0 <= r < p, r <= t-1} F[t-1-r] + w[1+r] )
// and for the deconvolution (f (/) w)[t] = max_j f[t+j] - w[j]:
//   F[u]   = max_{q >= 0, u + q p <= n-1} f[u + q p] - q c
//   out[t] = max( f[t] - w[0],  max_{0 <= r < p, t+1+r <= n-1} F[t+1+r] - w[1+r] )
// (max-plus convolution and min-plus deconvolution alike).  n p candidates per row pair instead of
// n^2 / 2, in exact integer arithmetic: F holds f[s] + (w[j] - w[1+r]), which the row ranges
// must keep inside the type (checked by period_kernel), and F + w[1+r] is the definition's
// candidate itself.  Any multiple of a period is a period: short periods are multiplied up
// (period_target).
constexpr int kPeriodMax = 1024;     // longest period looked for
constexpr int kPeriodTries = 4;      // full verifications per operand
constexpr int kPeriodRun = 128;      // consecutive positions of the first test
// Periods shorter than this are multiplied up.  The scan walks n / p steps per residue class one
// after the other (about 0.1 us each, whatever the batch), the window product reduces
// batch n p candidates at about 12 T/s: the sum is smallest near p = sqrt(1.2e6 / batch).
inline int period_target(int64_t batch) {
  int t = 32;
  while (t < 256 && (int64_t)(t + 1) * (t + 1) * batch <= 1200000) ++t;
  return t;
}
__host__ __device__ inline int period_limit(int64_t n) { return n / 16 < kPeriodMax ? (int)(n / 16) : kPeriodMax; }

// One workgroup per row pair that no other structured path took (sel < kSelSearch): looks for
// the smallest period <= period_limit(n) of g, and for the convolutions (unless g's is short
// enough already) of f: every period is screened at a few positions, what passes is tested at
// kPeriodRun consecutive positions, three spread ones and across the whole row along two residue
// classes, and the survivors (in ascending order, at most kPeriodTries per operand) at all
// positions.  On success sel[row] becomes kSelPeriodic /
// kSelPeriodicSwapped and period[row] (if given) the period to use.
constexpr int kPeriodThreads = 1024;

template <typename T>
__global__ __launch_bounds__(kPeriodThreads) void period_kernel(const T* __restrict__ f, int64_t stride_f,
                                                                const T* __restrict__ g, int64_t stride_g,
                                                                int32_t* __restrict__ sel,
                                                                int32_t* __restrict__ period,
                                                                int32_t* __restrict__ pack_ok, int n, int op, int target) {
  constexpr int kWaves = kPeriodThreads / 64;
  __shared__ uint32_t s_cand[2][kPeriodMax / 32];
  __shared__ T s_red[4][kWaves];
  __shared__ T s_w[2][kPeriodRun + 2 * kPeriodMax];   // w[1 ...], the head of each row
  __shared__ uint32_t s_seen[2][kPeriodMax / 32];     // periods that passed the screening
  const int row = blockIdx.x;
  if (sel[row] >= kSelSearch) return;
  const int pmax = period_limit(n);
  if (pmax < 1) return;
  const int run = min(kPeriodRun, n - 2 - pmax);      // positions 1 .. run of the first test; >= 1 as n >= 16 pmax
  const int nrows = op_sub(op) ? 1 : 2;               // g, and f of a convolution
  const T* rows[2] = {g + (int64_t)row * stride_g, f + (int64_t)row * stride_f};
  for (int k = threadIdx.x; k < 2 * (kPeriodMax / 32); k += kPeriodThreads) {
    (&s_cand[0][0])[k] = 0;
    (&s_seen[0][0])[k] = 0;
  }
  const int staged = min(run + 2 * pmax, n - 1);      // w[1 .. staged]
  {
    // both rows, every load of a thread issued before the first is stored (a loop of "load, store
    // to LDS" waits for each load on the spot); an index past the end repeats the last one
    constexpr int kLoads = (2 * (kPeriodRun + 2 * kPeriodMax) + kPeriodThreads - 1) / kPeriodThreads;
    const T* const w0 = g + (int64_t)row * stride_g;
    const T* const w1 = f + (int64_t)row * stride_f;
    const int count = nrows * staged;
    T head[kLoads];
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const int at = min(k * kPeriodThreads + (int)threadIdx.x, count - 1);
      head[k] = at >= staged ? w1[1 + at - staged] : w0[1 + at];
    }
    asm volatile("" ::: "memory");
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const int at = k * kPeriodThreads + (int)threadIdx.x;
      if (at < count) (&s_w[0][0])[at >= staged ? (kPeriodRun + 2 * kPeriodMax) + at - staged : at] = head[k];
    }
  }
  __syncthreads();
  // Screening, one thread per (row, period), from the staged head of the row alone: eight
  // consecutive positions and the far ends, inside the staged window, of the residue classes
  // of positions 1 and 1 + p/2, w[i + k p] = w[i] + k c (a plateau agrees with every short
  // period locally, not across a window longer than the true period).
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pmax64 = (pmax + 63) & ~63;                // a wavefront's 64 periods share a row and two words
  for (int item = threadIdx.x; item < nrows * pmax64; item += kPeriodThreads) {
    const int which = item / pmax64, p = min(item % pmax64 + 1, pmax);
    const T* sw = s_w[which];
    const T c = wrap_sub(sw[p], sw[0]);
    const int i2 = p / 2;
    const int k1 = (staged - 1) / p, k2 = (staged - 1 - i2) / p;
    int same = (wrap_sub(sw[k1 * p], sw[0]) == (T)((T)k1 * c)) & (wrap_sub(sw[i2 + k2 * p], sw[i2]) == (T)((T)k2 * c));
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int at = min(k, run - 1);
      same &= wrap_sub(sw[at + p], sw[at]) == c;
    }
    const uint64_t pass = __ballot(same != 0 && item % pmax64 < pmax);
    if ((lane & 31) == 0) s_seen[which][(item % pmax64) >> 5] = (lane & 32) ? (uint32_t)(pass >> 32) : (uint32_t)pass;
  }
  __syncthreads();
  // (The common case, rows without a period: nothing passed -- both rows' sets are 64 words, one
  // per lane -- and every wavefront leaves here instead of walking empty sets word by word.)
  static_assert(2 * (kPeriodMax / 32) == 64, "one word of the two rows' sets per lane");
  if (__ballot((&s_seen[0][0])[lane] != 0u) == 0) return;
  // First test of what passed, in ascending order, one wavefront per period and kWaves at a
  // time: a run of consecutive positions (staircases agree with many wrong periods at scattered
  // ones), three positions spread over the row and the far ends of two residue classes over
  // the whole row.  What passes becomes a candidate (every multiple of a period passes too: the
  // search of a row ends with its kPeriodTries smallest candidates).
  {
    // the wavefronts are shared out between the rows, so that one round serves both
    const int per = kWaves / nrows;                    // wavefronts per row
    const int which = wave / per, slot = wave % per;
    const T* w = rows[which];
    const T* sw = s_w[which];
    // position of a period in a row's set: prefix popcounts over its 32 words
    uint32_t word[2];
    int incl[2], total[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      word[r] = (r < nrows && lane < kPeriodMax / 32) ? s_seen[r][lane] : 0u;
      incl[r] = __popc(word[r]);
#pragma unroll
      for (int off = 1; off < 32; off <<= 1) {
        const int up = __shfl_up(incl[r], off);
        if (lane >= off) incl[r] += up;
      }
      total[r] = __shfl(incl[r], 31);
    }
    const uint32_t my_word = which ? word[1] : word[0];
    const int my_incl = which ? incl[1] : incl[0], my_total = which ? total[1] : total[0];
    // this wavefront tests the slot-th, (slot + per)-th, ... period of its row's set (no barrier:
    // the wavefronts run on their own)
    for (int k = slot; k < my_total; k += per) {
      {
        const uint64_t holds = __ballot(lane < 32 && my_incl > k);       // first word whose prefix count exceeds k
        const int wi = __builtin_ctzll(holds);
        uint32_t bits = __shfl(my_word, wi);
        int skip = k - (__shfl(my_incl, wi) - __popc(bits));
        while (skip-- > 0) bits &= bits - 1;
        const int p = wi * 32 + __builtin_ctz(bits) + 1;
        // stop once kPeriodTries smaller periods have passed: the full test below looks at no more
        // than that many, in ascending order, so the kPeriodTries smallest that pass are always
        // found, whatever the order in which the wavefronts get here
        {
          const int below = p - 1 - lane * 32;       // bits of word `lane` that stand for periods < p
          const uint32_t seen = lane < kPeriodMax / 32 ? ((volatile uint32_t*)s_cand[which])[lane] : 0u;
          int passed = __popc(below >= 32 ? seen : below <= 0 ? 0u : seen & ((1u << below) - 1u));
#pragma unroll
          for (int off = 32; off > 0; off >>= 1) passed += __shfl_xor(passed, off);
          if (passed >= kPeriodTries) break;
        }
        const T c = wrap_sub(sw[p], sw[0]);
        bool ok = true;
        for (int i = lane; i < run; i += 64) ok = ok && wrap_sub(sw[i + p], sw[i]) == c;
        ok = __all(ok);                               // (the row itself is only read for periods that got this far)
        if (ok && lane < 5) {
          const int span = n - 2 - p;                  // positions 1 .. 1 + span have a partner
          const int i2 = 1 + p / 2;
          const int first = lane == 0 ? 1 + span : lane == 1 ? 1 + span / 2 : lane == 2 ? 1 + span / 3 : lane == 3 ? 1 : i2;
          const int steps = lane == 3 ? (n - 2) / p : lane == 4 ? (n - 1 - i2) / p : 1;
          ok = wrap_sub(w[first + steps * p], w[first]) == (T)((T)steps * c);
        }
        if (__all(ok) && lane == 0) atomicOr(&s_cand[which][(p - 1) >> 5], 1u << ((p - 1) & 31));
      }
    }
  }
  __syncthreads();
  if (__ballot((&s_cand[0][0])[lane] != 0u) == 0) return;   // (no survivor: as above)
  // full test of the survivors in ascending order; the first full pass also takes the extrema of
  // both rows over the indices >= 1
  // (target = period_target(batch): periods below it are multiplied up anyway)
  int best_p = 0, best_which = 0;
  bool have_mm = false;
  int mm_which = 0;                                                     // the row that wmn / wmx describe
  T wmn = 0, wmx = 0, omn = 0, omx = 0;
  for (int which = 0; which < nrows; ++which) {
    if (best_p != 0 && best_p <= target) break;
    const T* w = rows[which];
    const T* o = rows[which ^ 1];
    int tries = 0;
    bool done = false;
    for (int word = 0; word < kPeriodMax / 32 && !done; ++word) {
      uint32_t bits = s_cand[which][word];
      while (bits != 0 && !done) {
        const int p = word * 32 + __builtin_ctz(bits) + 1;
        bits &= bits - 1;
        if ((best_p != 0 && p >= best_p) || tries++ == kPeriodTries) { done = true; break; }
        const T c = wrap_sub(s_w[which][p], s_w[which][0]);
        int bad = 0;
        if (!have_mm) {
          wmn = wmx = w[1]; omn = omx = o[1];
#pragma unroll 4
          for (int i = 1 + threadIdx.x; i <= n - 1; i += kPeriodThreads) {
            const T wv = w[i], ov = o[i], wp = w[min(i + p, n - 1)];
            bad |= (i + p <= n - 1) && wrap_sub(wp, wv) != c;
            wmn = sel_min(wmn, wv); wmx = sel_max(wmx, wv);
            omn = sel_min(omn, ov); omx = sel_max(omx, ov);
          }
          have_mm = true;
          mm_which = which;
        } else {
#pragma unroll 8
          for (int i = 1 + threadIdx.x; i + p <= n - 1; i += kPeriodThreads) bad |= wrap_sub(w[i + p], w[i]) != c;
        }
        if (__syncthreads_or(bad) == 0) { best_p = p; best_which = which; done = true; }
      }
    }
  }
  if (best_p == 0) return;
  // ranges: every f[s] +- (w[j] - w[j']) must fit the type
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    wmn = sel_min(wmn, __shfl_xor(wmn, off)); wmx = sel_max(wmx, __shfl_xor(wmx, off));
    omn = sel_min(omn, __shfl_xor(omn, off)); omx = sel_max(omx, __shfl_xor(omx, off));
  }
  if ((threadIdx.x & 63) == 0) {
    const int wave = threadIdx.x >> 6;
    s_red[0][wave] = wmn; s_red[1][wave] = wmx; s_red[2][wave] = omn; s_red[3][wave] = omx;
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  for (int k = 1; k < kWaves; ++k) {
    wmn = sel_min(wmn, s_red[0][k]); wmx = sel_max(wmx, s_red[1][k]);
    omn = sel_min(omn, s_red[2][k]); omx = sel_max(omx, s_red[3][k]);
  }
  const bool same = best_which == mm_which;
  const T wmin = same ? wmn : omn, wmax = same ? wmx : omx;
  const T u0 = rows[best_which ^ 1][0];
  const T umin = sel_min(same ? omn : wmn, u0), umax = sel_max(same ? omx : wmx, u0);
  T span, dummy;
  if (__builtin_sub_overflow(wmax, wmin, &span) || __builtin_add_overflow(umax, span, &dummy) ||
      __builtin_sub_overflow(umin, span, &dummy))
    return;
  // multiply short periods up: enough residue classes for the scan, still a short window
  int p = best_p;
  if (p < target) {
    p = best_p * ((target + best_p - 1) / best_p);
    if (p > pmax) p = best_p * (pmax / best_p);
  }
  sel[row] = best_which ? kSelPeriodicSwapped : kSelPeriodic;
  if (period != nullptr) period[row] = p;
  if (pack_ok != nullptr) pack_ok[row] = 0;          // no packed-path preparation for this row
}

// F of the rows that period_kernel selected: one thread per residue class.
template <typename T, int OP>
__device__ __forceinline__ void periodic_scan_body(const T* __restrict__ f, int64_t stride_f,
                                                   const T* __restrict__ g, int64_t stride_g,
                                                   const int32_t* __restrict__ sel,
                                                   const int32_t* __restrict__ period, T* __restrict__ F, int n,
                                                   int blocks_per_row, int block) {
  const int row = block / blocks_per_row;
  const int code = sel[row];
  if (code != kSelPeriodic && code != kSelPeriodicSwapped) return;
  const int p = period[row];
  const int rho = (block % blocks_per_row) * 256 + threadIdx.x;
  if (rho >= p) return;
  const bool swapped = code == kSelPeriodicSwapped;
  const T* u = swapped ? g + (int64_t)row * stride_g : f + (int64_t)row * stride_f;
  const T* w = swapped ? f + (int64_t)row * stride_f : g + (int64_t)row * stride_g;
  T* Fr = F + (int64_t)row * n;
  const T c = wrap_sub(w[1 + p], w[1]);
  const int steps = (n - 1 - rho) / p;               // the class is rho, rho + p, ..., rho + steps p
  if (!op_sub(OP)) {
    T acc = u[rho];
    Fr[rho] = acc;
#pragma unroll 8
    for (int k = 1; k <= steps; ++k) {
      const int i = rho + k * p;
      acc = Semiring<T, OP>::reduce(u[i], wrap_add(acc, c));
      Fr[i] = acc;
    }
  } else {
    T acc = u[rho + steps * p];
    Fr[rho + steps * p] = acc;
#pragma unroll 8
    for (int k = steps - 1; k >= 0; --k) {
      const int i = rho + k * p;
      acc = Semiring<T, OP>::reduce(u[i], wrap_sub(acc, c));
      Fr[i] = acc;
    }
  }
}

// The short window over F for the kPeriodicOutputs = 1024 outputs from t0 on of a selected row
// (the whole workgroup comes here; each thread takes four outputs 256 apart, which spreads the
// fixed cost of a workgroup -- a chain of dependent loads before the first candidate -- over
// four times the work): the F values they need (1024 + p - 1 of them) staged in LDS (s_F,
// kPeriodicOutputs + kPeriodMax values), the periodic operand's first period read through
// uniform loads.  Candidates outside the triangle exist only in a row's first (convolutions) or
// last (deconvolutions) workgroup, which takes the checked loop.
constexpr int kPeriodicPer = 4;                         // outputs per thread
constexpr int kPeriodicOutputs = 256 * kPeriodicPer;
template <typename T, int OP>
__device__ __forceinline__ void periodic_product_body(const T* __restrict__ f, int64_t stride_f,
                                                      const T* __restrict__ g, int64_t stride_g,
                                                      T* __restrict__ out, const T* __restrict__ cap,
                                                      const int32_t* __restrict__ period,
                                                      const T* __restrict__ F, T* s_F, int n, int row, int code,
                                                      int t0) {
  constexpr int E = kPeriodicPer;
  const int p = period[row];
  const int tid = threadIdx.x;
  const bool swapped = code == kSelPeriodicSwapped;
  const T* u = swapped ? g + (int64_t)row * stride_g : f + (int64_t)row * stride_f;
  const T* w = swapped ? f + (int64_t)row * stride_f : g + (int64_t)row * stride_g;
  const T* Fr = F + (int64_t)row * n;
  // convolutions read F[t - r1], deconvolutions F[t + r1], r1 = 1 .. p:  s_F[k] = F[base + k]
  // (index clamped where F does not exist: never used there; unrolled so that the loads of
  // several rounds are in flight together)
  const int base = op_sub(OP) ? t0 + 1 : t0 - p;
  const T w_0 = w[0];
  T v[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const T u_t = u[min(t0 + e * 256 + tid, n - 1)];
    v[e] = op_sub(OP) ? wrap_sub(u_t, w_0) : wrap_add(u_t, w_0);
  }
#pragma unroll 4
  for (int k = tid; k < kPeriodicOutputs - 1 + p; k += 256) s_F[k] = Fr[min(max(base + k, 0), n - 1)];
  __syncthreads();
  const int at = op_sub(OP) ? tid - 1 : tid + p;        // output e, step r1: s_F[at + 256 e +- r1]
  const bool whole = op_sub(OP) ? t0 + kPeriodicOutputs - 1 + p <= n - 1 : t0 >= p;   // every candidate of every output exists
  if (whole) {
#pragma unroll 4
    for (int r1 = 1; r1 <= p; ++r1) {
      const T wv = w[r1];
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const T fv = s_F[at + e * 256 + (op_sub(OP) ? r1 : -r1)];
        v[e] = Semiring<T, OP>::reduce(v[e], op_sub(OP) ? wrap_sub(fv, wv) : wrap_add(fv, wv));
      }
    }
  } else {
#pragma unroll 2
    for (int r1 = 1; r1 <= p; ++r1) {
      const T wv = w[r1];
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int t = t0 + e * 256 + tid;
        const bool exists = op_sub(OP) ? r1 <= n - 1 - t : r1 <= t;
        const T fv = s_F[at + e * 256 + (op_sub(OP) ? r1 : -r1)];
        const T r = Semiring<T, OP>::reduce(v[e], op_sub(OP) ? wrap_sub(fv, wv) : wrap_add(fv, wv));
        v[e] = exists ? r : v[e];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int t = t0 + e * 256 + tid;
    if (t < n) {
      T r = v[e];
      if (cap != nullptr) r = sel_min(r, cap[(int64_t)row * n + t]);
      out[(int64_t)row * n + t] = r;
    }
  }
}

// Rows with sel[row] == kSelEnds or kSelSearch (decided by the probe kernels, see
// structure_code) are computed here, every other row is left alone.  The candidates of output t
// are c(j), 0 <= j <= m:
//   convolutions    c(j) = f[j] + g[t-j],   m = t
//   deconvolutions  c(j) = f[t+j] - g[j],   m = n-1-t
// kSelEnds:   the reduction of c(0) and c(m) (min over a concave / max over a convex sequence).
// kSelSearch: bisection for the first j with c(j+1) >= c(j) (min over a convex sequence) resp.
//             c(j+1) <= c(j) (max over a concave one); c there is the result.
// kSelBracket(Swapped): the reduction over the candidates between the optima of the two anchors
//             around t (bracket_fine_kernel; one wavefront = the 64 outputs
//             between two anchors).
// kSelPeriodic(Swapped): the short window over F, periodic_product_body.
// Each candidate is formed exactly as the general kernels form it (one wrap-around add or
// subtract; the periodic path's in two exact steps), so the result is the same value bit for bit.
template <typename T, int OP>
__global__ __launch_bounds__(256) void structured_kernel(const T* __restrict__ f, int64_t stride_f,
                                                         const T* __restrict__ g, int64_t stride_g,
                                                         T* __restrict__ out, const T* __restrict__ cap,
                                                         const int32_t* __restrict__ sel,
                                                         const int32_t* __restrict__ jstar,
                                                         const int32_t* __restrict__ period,
                                                         const T* __restrict__ F, int n, int blocks_per_row,
                                                         int batch) {
  static_assert(256 % kBracketFine == 0 && kBracketFine == 64, "one wavefront = the outputs between two fine anchors");
  __shared__ T s_F[kPeriodicOutputs + kPeriodMax];
  // rows fastest: the workgroups that have work (every kPeriodicPer-th block of a periodic row)
  // then come in runs of `batch` consecutive ones, which the dispatcher spreads over all XCDs and
  // CUs; with blocks fastest they would all land on a quarter of them
  const int row = blockIdx.x % batch;
  const int code = sel[row];
  if (code < kSelSearch) return;
  const int block = blockIdx.x / batch;
  if (code >= kSelPeriodic) {      // every kPeriodicPer-th workgroup of the row, for that many blocks of 256 outputs
    if (block % kPeriodicPer == 0)
      periodic_product_body<T, OP>(f, stride_f, g, stride_g, out, cap, period, F, s_F, n, row, code, block * 256);
    return;
  }
  const int t = block * 256 + threadIdx.x;
  if (t >= n) return;
  const bool swapped = code == kSelBracketSwapped;
  const T* fr = swapped ? g + (int64_t)row * stride_g : f + (int64_t)row * stride_f;
  const T* gr = swapped ? f + (int64_t)row * stride_f : g + (int64_t)row * stride_g;
  auto c = [&](int j) -> T { return op_sub(OP) ? wrap_sub(fr[t + j], gr[j]) : wrap_add(fr[j], gr[t - j]); };
  const int m = op_sub(OP) ? n - 1 - t : t;
  T v;
  if (code == kSelEnds) {
    v = Semiring<T, OP>::reduce(c(0), c(m));
  } else if (code >= kSelBracket) {
    const int32_t* js = jstar + (int64_t)row * bracket_anchors(n, kBracketFine) + t / kBracketFine;
    const int ja = js[0], jb = js[1];            // optima of the fine anchors below and above t
    const int lo = min(max(op_sub(OP) ? jb : ja, 0), m);     // clamped as in bracket_anchor_body
    const int hi = min(op_sub(OP) ? ja : jb, m);
    v = c(lo);
#pragma unroll 4
    for (int j = lo + 1; j <= hi; ++j) v = Semiring<T, OP>::reduce(v, c(j));
  } else {
    int lo = 0, hi = m;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      const T a = c(mid), b = c(mid + 1);
      if (op_max(OP) ? b <= a : b >= a) hi = mid; else lo = mid + 1;
    }
    v = c(lo);
  }
  if (cap != nullptr) v = sel_min(v, cap[(int64_t)row * n + t]);
  out[(int64_t)row * n + t] = v;
}

// First launch of the structured rows: the coarse anchors of the bracket path and the scan of
// the periodic path (different rows; both feed the launches that follow).
template <typename T, int OP>
__global__ __launch_bounds__(256) void structured_first_kernel(const T* __restrict__ f, int64_t stride_f,
                                                               const T* __restrict__ g, int64_t stride_g,
                                                               const int32_t* __restrict__ sel,
                                                               int32_t* __restrict__ jcoarse, int coarse_anchors,
                                                               int anchor_blocks, const int32_t* __restrict__ period,
                                                               T* __restrict__ F, int n, int scan_blocks_per_row) {
  if ((int)blockIdx.x < anchor_blocks)
    bracket_anchor_body<T, OP, kBracketCoarse, true>(f, stride_f, g, stride_g, sel, nullptr, 0, jcoarse, n,
                                                     coarse_anchors, blockIdx.x);
  else
    periodic_scan_body<T, OP>(f, stride_f, g, stride_g, sel, period, F, n, scan_blocks_per_row,
                              blockIdx.x - anchor_blocks);
}

template <typename T, int OP>
__global__ __launch_bounds__(256) void bracket_fine_kernel(const T* __restrict__ f, int64_t stride_f,
                                                           const T* __restrict__ g, int64_t stride_g,
                                                           const int32_t* __restrict__ sel,
                                                           const int32_t* __restrict__ jcoarse, int coarse_anchors,
                                                           int32_t* __restrict__ jstar, int n, int anchors) {
  bracket_anchor_body<T, OP, kBracketFine, false>(f, stride_f, g, stride_g, sel, jcoarse, coarse_anchors, jstar, n,
                                                  anchors, blockIdx.x);
}

// Runs after the probe kernels (which write sel) and before any kernel that reads sel.
template <typename T>
void launch_period(const T* f, int64_t stride_f, const T* g, int64_t stride_g, int32_t* sel, int32_t* period,
                   int32_t* pack_ok, int64_t batch, int64_t n, int op, hipStream_t stream) {
  if (period_limit(n) < 1) return;
  RTC_LAUNCH(period_kernel<T>, dim3((uint32_t)batch), dim3(kPeriodThreads), 0, stream, f, stride_f, g, stride_g, sel,
                     period, pack_ok, (int)n, op, period_target(batch));
}

inline size_t bracket_jstar_elems(int64_t batch, int64_t n) {
  return (size_t)batch * ((size_t)bracket_anchors(n, kBracketFine) + (size_t)bracket_anchors(n, kBracketCoarse));
}

template <typename T, int OP>
int launch_structured(const T* f, int64_t stride_f, const T* g, int64_t stride_g, T* out, const T* cap,
                      const int32_t* sel, int32_t* jstar, const int32_t* period, T* F, int64_t batch, int64_t n,
                      hipStream_t stream) {
  const int64_t bpr = (n + 255) / 256;
  const int fine = bracket_anchors(n, kBracketFine), coarse = bracket_anchors(n, kBracketCoarse);
  if (batch * fine > 0x7fffffffLL) return RTC_ERR_SHAPE;
  // jstar: [batch][fine] optima of the fine anchors, then [batch][coarse] of the coarse ones
  // (bracket_jstar_elems() int32 in all)
  int32_t* jcoarse = jstar + batch * fine;
  const int pblocks = (period_limit(n) + 255) / 256;
  if (batch * (coarse + pblocks) > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_LAUNCH((structured_first_kernel<T, OP>), dim3((uint32_t)(batch * (coarse + pblocks))), dim3(256), 0,
                     stream, f, stride_f, g, stride_g, sel, jcoarse, coarse, (int)(batch * coarse), period, F, (int)n,
                     pblocks);
  RTC_LAUNCH((bracket_fine_kernel<T, OP>), dim3((uint32_t)(batch * ((fine + 3) / 4))), dim3(256), 0, stream,
                     f, stride_f, g, stride_g, sel, jcoarse, coarse, jstar, (int)n, fine);
  RTC_LAUNCH((structured_kernel<T, OP>), dim3((uint32_t)(batch * bpr)), dim3(256), 0, stream, f, stride_f, g,
                     stride_g, out, cap, sel, jstar, period, F, (int)n, (int)bpr, (int)batch);
  return hip_ok();
}

}  // namespace
}  // namespace rtc
