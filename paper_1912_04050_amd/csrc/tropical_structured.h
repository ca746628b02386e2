// Tropical products of row pairs whose convexity makes the reduction trivial: one thread per
// output, O(1) or O(log n) candidates instead of all of them.  Included by tropical.hip only.
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
__global__ __launch_bounds__(256) void bracket_anchor_kernel(const T* __restrict__ f, int64_t stride_f,
                                                                 const T* __restrict__ g, int64_t stride_g,
                                                                 const int32_t* __restrict__ sel,
                                                                 const int32_t* __restrict__ coarse, int coarse_anchors,
                                                                 int32_t* __restrict__ jstar, int n, int anchors) {
  constexpr int kWaves = 4;
  constexpr int kThreads = SHARED ? 256 : 64;    // lanes that share one anchor
  constexpr int kNone = 0x7fffffff;
  __shared__ T s_val[kWaves];
  __shared__ int s_idx[kWaves];
  const int groups = SHARED ? anchors : (anchors + kWaves - 1) / kWaves;   // workgroups per row
  const int row = blockIdx.x / groups;
  const int code = sel[row];
  if (code != kSelBracket && code != kSelBracketSwapped) return;
  const int lane = SHARED ? threadIdx.x : threadIdx.x & 63;
  const int a = SHARED ? blockIdx.x % groups : (blockIdx.x % groups) * kWaves + (threadIdx.x >> 6);
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
    lo = op_sub(OP) ? jb : ja;
    hi = min(op_sub(OP) ? ja : jb, m);
  }
  T best = Semiring<T, OP>::identity();
  int best_j = kNone;
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

// Rows with sel[row] == kSelEnds or kSelSearch (decided by the probe kernels, see
// structure_code) are computed here, every other row is left alone.  The candidates of output t
// are c(j), 0 <= j <= m:
//   convolutions    c(j) = f[j] + g[t-j],   m = t
//   deconvolutions  c(j) = f[t+j] - g[j],   m = n-1-t
// kSelEnds:   the reduction of c(0) and c(m) (min over a concave / max over a convex sequence).
// kSelSearch: bisection for the first j with c(j+1) >= c(j) (min over a convex sequence) resp.
//             c(j+1) <= c(j) (max over a concave one); c there is the result.
// kSelBracket(Swapped): the reduction over the candidates between the optima of the two anchors
//             around t (bracket_anchor_kernel's fine level; one wavefront = the 64 outputs
//             between two anchors).
// Each candidate is formed exactly as the general kernels form it (one wrap-around add or
// subtract), so the result is the same value bit for bit.
template <typename T, int OP>
__global__ __launch_bounds__(256) void structured_kernel(const T* __restrict__ f, int64_t stride_f,
                                                         const T* __restrict__ g, int64_t stride_g,
                                                         T* __restrict__ out, const T* __restrict__ cap,
                                                         const int32_t* __restrict__ sel,
                                                         const int32_t* __restrict__ jstar, int n,
                                                         int blocks_per_row) {
  static_assert(256 % kBracketFine == 0 && kBracketFine == 64, "one wavefront = the outputs between two fine anchors");
  const int row = blockIdx.x / blocks_per_row;
  const int code = sel[row];
  if (code < kSelSearch) return;
  const int block = blockIdx.x % blocks_per_row;
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
    const int lo = op_sub(OP) ? jb : ja;
    const int hi = min(op_sub(OP) ? ja : jb, m);
    v = c(lo);
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

inline size_t bracket_jstar_elems(int64_t batch, int64_t n) {
  return (size_t)batch * ((size_t)bracket_anchors(n, kBracketFine) + (size_t)bracket_anchors(n, kBracketCoarse));
}

template <typename T, int OP>
int launch_structured(const T* f, int64_t stride_f, const T* g, int64_t stride_g, T* out, const T* cap,
                      const int32_t* sel, int32_t* jstar, int64_t batch, int64_t n, hipStream_t stream) {
  const int64_t bpr = (n + 255) / 256;
  const int fine = bracket_anchors(n, kBracketFine), coarse = bracket_anchors(n, kBracketCoarse);
  if (batch * fine > 0x7fffffffLL) return RTC_ERR_SHAPE;
  // jstar: [batch][fine] optima of the fine anchors, then [batch][coarse] of the coarse ones
  // (bracket_jstar_elems() int32 in all)
  int32_t* jcoarse = jstar + batch * fine;
  hipLaunchKernelGGL((bracket_anchor_kernel<T, OP, kBracketCoarse, true>), dim3((uint32_t)(batch * coarse)), dim3(256), 0,
                     stream, f, stride_f, g, stride_g, sel, nullptr, 0, jcoarse, (int)n, coarse);
  hipLaunchKernelGGL((bracket_anchor_kernel<T, OP, kBracketFine, false>), dim3((uint32_t)(batch * ((fine + 3) / 4))),
                     dim3(256), 0, stream, f, stride_f, g, stride_g, sel, jcoarse, coarse, jstar, (int)n, fine);
  hipLaunchKernelGGL((structured_kernel<T, OP>), dim3((uint32_t)(batch * bpr)), dim3(256), 0, stream, f, stride_f, g,
                     stride_g, out, cap, sel, jstar, (int)n, (int)bpr);
  return hip_ok();
}

}  // namespace
}  // namespace rtc
