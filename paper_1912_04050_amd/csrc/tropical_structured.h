// Tropical products of row pairs whose convexity makes the reduction trivial: one thread per
// output, O(1) or O(log n) candidates instead of all of them.  Included by tropical.hip only.
#pragma once

#include "tropical_common.h"
#include "tropical_prepare.h"

namespace rtc {
namespace {

// Rows with sel[row] == kSelEnds or kSelSearch (decided by the probe kernels, see
// structure_code) are computed here, every other row is left alone.  The candidates of output t
// are c(j), 0 <= j <= m:
//   convolutions    c(j) = f[j] + g[t-j],   m = t
//   deconvolutions  c(j) = f[t+j] - g[j],   m = n-1-t
// kSelEnds:   the reduction of c(0) and c(m) (min over a concave / max over a convex sequence).
// kSelSearch: bisection for the first j with c(j+1) >= c(j) (min over a convex sequence) resp.
//             c(j+1) <= c(j) (max over a concave one); c there is the result.
// Each candidate is formed exactly as the general kernels form it (one wrap-around add or
// subtract), so the result is the same value bit for bit.
template <typename T, int OP>
__global__ __launch_bounds__(256) void structured_kernel(const T* __restrict__ f, int64_t stride_f,
                                                         const T* __restrict__ g, int64_t stride_g,
                                                         T* __restrict__ out, const T* __restrict__ cap,
                                                         const int32_t* __restrict__ sel, int n,
                                                         int blocks_per_row) {
  const int row = blockIdx.x / blocks_per_row;
  const int code = sel[row];
  if (code < kSelSearch) return;
  const int t = (blockIdx.x % blocks_per_row) * 256 + threadIdx.x;
  if (t >= n) return;
  const T* fr = f + (int64_t)row * stride_f;
  const T* gr = g + (int64_t)row * stride_g;
  auto c = [&](int j) -> T { return op_sub(OP) ? wrap_sub(fr[t + j], gr[j]) : wrap_add(fr[j], gr[t - j]); };
  const int m = op_sub(OP) ? n - 1 - t : t;
  T v;
  if (code == kSelEnds) {
    v = Semiring<T, OP>::reduce(c(0), c(m));
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

template <typename T, int OP>
int launch_structured(const T* f, int64_t stride_f, const T* g, int64_t stride_g, T* out, const T* cap,
                      const int32_t* sel, int64_t batch, int64_t n, hipStream_t stream) {
  const int64_t bpr = (n + 255) / 256;
  if (batch * bpr > 0x7fffffffLL) return RTC_ERR_SHAPE;
  hipLaunchKernelGGL((structured_kernel<T, OP>), dim3((uint32_t)(batch * bpr)), dim3(256), 0, stream, f, stride_f, g,
                     stride_g, out, cap, sel, (int)n, (int)bpr);
  return hip_ok();
}

}  // namespace
}  // namespace rtc
