// CPU oracle for the (min,+) curve algebra of real-time calculus.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, literal reference that the
// tests, the smoke check and the benchmark's cpu_baseline leg compare the GPU
// library against.  It shares no code with the HIP path and must never be called
// from the product path.
//
// Curves are sampled functions over Delta = 0..n-1 (arrival curves alpha^u/alpha^l,
// service curves beta^u/beta^l, workload curves gamma^u/gamma^l and their
// pseudo-inverses, in the notation of the paper's curve macros).  The paper gives
// the symbols only; every operator below is the textbook definition written out
// as loops, in the same order as the definition, with no blocking or pruning:
//
//   min-plus convolution     (f (x) g)[t] = min_{0<=s<=t} f[s] + g[t-s]
//   max-plus deconvolution   (f (/) g)[t] = max_{0<=u<=n-1-t} f[t+u] - g[u]
//                            (finite horizon: only pairs whose samples both exist)
//   max-plus convolution     max_{0<=s<=t} f[s] + g[t-s]          (the two dual products)
//   min-plus deconvolution   min_{0<=u<=n-1-t} f[t+u] - g[u]
//   lower pseudo-inverse     min{k : f[k] >= x}, n if there is none
//   upper pseudo-inverse     max{k : f[k] <= x}, -1 if there is none
//   composition              out[D] = outer[clamp(inner[D], 0, n_outer-1)]
//   greedy processing component (upper arrival / lower service outputs)
//                            alpha'^u = min((alpha^u (x) beta^u) (/) beta^l, beta^u)
//                            beta'^l[D] = max(0, max_{l<=D} beta^l[l] - alpha^u[l])
//                            alpha'^l = min((alpha^l (/) beta^u) (x) beta^l, beta^l)
//                            beta'^u[D] = max(0, min_{l>=D} beta^u[l] - alpha^l[l])
//   sub-additive closure     min(delta_0, f, f (x) f, f (x) f (x) f, ...), f[0] read as 0
//   super-additive closure   the same with max and the max-plus convolution
//   chain                    curves[0] (x) curves[1] (x) ... (x) curves[count-1]
//   horizontal deviation     max_D max(0, lower-inverse_beta(alpha[D]) - D)
//   vertical deviation       max_D alpha[D] - beta[D]
//
// Pins (tests/test_oracle_*.py, all CPU): closed forms for token bucket against
// rate latency, brute force in Python on curves of at most 64 points, algebraic
// invariants, numpy.searchsorted for the pseudo-inverses.  Whole-configuration
// outputs have no published value to compare with: parity unpinned by the paper.
//
// OpenMP only distributes independent outputs over threads; each output is
// computed by one thread in the order of the definition.
#include <cstdint>
#include <cstddef>
#include <omp.h>
#include <type_traits>

namespace {

// Every sum and difference of two samples goes through oadd / osub: plain + and - in the normal
// build.  Built with -DORACLE_CHECK_OVERFLOW (the debug build that tests/test_oracle_hygiene.py
// uses) the integer ones are checked with __builtin_add_overflow / __builtin_sub_overflow and
// counted, which asserts the precondition of the whole algebra -- no candidate leaves the
// element type -- on the inputs the benchmark configurations generate.
#ifdef ORACLE_CHECK_OVERFLOW
long long g_overflows = 0;
template <typename T> inline T oadd(T a, T b) {
  if constexpr (std::is_integral<T>::value) {
    T r;
    if (__builtin_add_overflow(a, b, &r)) {
#pragma omp atomic
      ++g_overflows;
    }
    return r;
  } else {
    return a + b;
  }
}
template <typename T> inline T osub(T a, T b) {
  if constexpr (std::is_integral<T>::value) {
    T r;
    if (__builtin_sub_overflow(a, b, &r)) {
#pragma omp atomic
      ++g_overflows;
    }
    return r;
  } else {
    return a - b;
  }
}
#else
template <typename T> inline T oadd(T a, T b) { return a + b; }
template <typename T> inline T osub(T a, T b) { return a - b; }
#endif

template <typename T>
void conv_one(const T* f, const T* g, T* out, int64_t n) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t t = 0; t < n; ++t) {
    T m = oadd(f[0], g[t]);
    for (int64_t s = 1; s <= t; ++s) {
      T v = oadd(f[s], g[t - s]);
      if (v < m) m = v;
    }
    out[t] = m;
  }
}

template <typename T>
void deconv_one(const T* f, const T* g, T* out, int64_t n) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t t = 0; t < n; ++t) {
    T m = osub(f[t], g[0]);
    for (int64_t u = 1; u <= n - 1 - t; ++u) {
      T v = osub(f[t + u], g[u]);
      if (v > m) m = v;
    }
    out[t] = m;
  }
}

template <typename T>
void maxconv_one(const T* f, const T* g, T* out, int64_t n) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t t = 0; t < n; ++t) {
    T m = oadd(f[0], g[t]);
    for (int64_t s = 1; s <= t; ++s) {
      T v = oadd(f[s], g[t - s]);
      if (v > m) m = v;
    }
    out[t] = m;
  }
}

template <typename T>
void mindeconv_one(const T* f, const T* g, T* out, int64_t n) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t t = 0; t < n; ++t) {
    T m = osub(f[t], g[0]);
    for (int64_t u = 1; u <= n - 1 - t; ++u) {
      T v = osub(f[t + u], g[u]);
      if (v < m) m = v;
    }
    out[t] = m;
  }
}

// Single outputs of the two products, for spot checks of large problems: the same loop
// as one iteration of conv_one / deconv_one.
template <typename T>
void product_at(const T* f, const T* g, int64_t n, const int64_t* t_idx, int64_t m, T* out, bool deconv) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t j = 0; j < m; ++j) {
    const int64_t t = t_idx[j];
    T r;
    if (!deconv) {
      r = oadd(f[0], g[t]);
      for (int64_t s = 1; s <= t; ++s) {
        T v = oadd(f[s], g[t - s]);
        if (v < r) r = v;
      }
    } else {
      r = osub(f[t], g[0]);
      for (int64_t u = 1; u <= n - 1 - t; ++u) {
        T v = osub(f[t + u], g[u]);
        if (v > r) r = v;
      }
    }
    out[j] = r;
  }
}

template <typename T>
int32_t pinv_lower_one(const T* f, int64_t n, T x) {
  for (int64_t k = 0; k < n; ++k)
    if (f[k] >= x) return (int32_t)k;
  return (int32_t)n;
}

template <typename T>
int32_t pinv_upper_one(const T* f, int64_t n, T x) {
  int32_t best = -1;
  for (int64_t k = 0; k < n; ++k)
    if (f[k] <= x) best = (int32_t)k;
  return best;
}

template <typename T>
void pinv_rows(const T* f, int64_t n, const T* x, int64_t m, int32_t* out, int64_t batch, int mode) {
  for (int64_t b = 0; b < batch; ++b) {
    const T* fr = f + b * n;
    const T* xr = x + b * m;
    int32_t* o = out + b * m;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t j = 0; j < m; ++j)
      o[j] = mode == 0 ? pinv_lower_one(fr, n, xr[j]) : pinv_upper_one(fr, n, xr[j]);
  }
}

template <typename T>
void compose_rows(const T* outer, int64_t n_outer, const int32_t* inner, int64_t n, T* out,
                  int64_t batch, int32_t* flags) {
  int32_t fl = 0;
  for (int64_t b = 0; b < batch; ++b)
    for (int64_t d = 0; d < n; ++d) {
      int64_t k = inner[b * n + d];
      if (k < 0) { k = 0; fl |= 2; }
      if (k > n_outer - 1) { k = n_outer - 1; fl |= 2; }
      out[b * n + d] = outer[b * n_outer + k];
    }
  if (flags) *flags |= fl;
}

template <typename T>
void gpc_rows(const T* au, const T* bu, const T* bl, T* au_out, T* bl_out, T* tmp, int64_t batch,
              int64_t n) {
  for (int64_t b = 0; b < batch; ++b) {
    const T* a = au + b * n;
    const T* u = bu + b * n;
    const T* l = bl + b * n;
    T* c = tmp + b * n;
    T* d = au_out + b * n;
    conv_one(a, u, c, n);
    deconv_one(c, l, d, n);
    for (int64_t k = 0; k < n; ++k)
      if (u[k] < d[k]) d[k] = u[k];
    T run = osub(l[0], a[0]);
    for (int64_t k = 0; k < n; ++k) {
      T v = osub(l[k], a[k]);
      if (v > run) run = v;
      bl_out[b * n + k] = run > (T)0 ? run : (T)0;
    }
  }
}

// lower arrival / upper service side of the component
template <typename T>
void gpc_lower_rows(const T* al, const T* bu, const T* bl, T* al_out, T* bu_out, T* tmp, int64_t batch,
                    int64_t n) {
  for (int64_t b = 0; b < batch; ++b) {
    const T* a = al + b * n;
    const T* u = bu + b * n;
    const T* l = bl + b * n;
    T* d = tmp + b * n;
    T* c = al_out + b * n;
    deconv_one(a, u, d, n);
    conv_one(d, l, c, n);
    for (int64_t k = 0; k < n; ++k)
      if (l[k] < c[k]) c[k] = l[k];
    T run = osub(u[n - 1], a[n - 1]);
    for (int64_t k = n - 1; k >= 0; --k) {
      T v = osub(u[k], a[k]);
      if (v < run) run = v;
      bu_out[b * n + k] = run > (T)0 ? run : (T)0;
    }
  }
}

// Closure by its definition: every k-fold convolution power of f (with f[0] read as 0, the value
// delta_0 contributes), k = 1 .. max(1, n-1); longer products only add zero-length parts.
template <typename T>
void closure_rows(const T* f, T* out, T* h, T* h2, T* f0, int64_t batch, int64_t n, bool super, int32_t* flags) {
  int32_t fl = 0;
  for (int64_t b = 0; b < batch; ++b) {
    const T* fr = f + b * n;
    T* o = out + b * n;
    if (super ? fr[0] > (T)0 : fr[0] < (T)0) fl |= 2;
    for (int64_t t = 0; t < n; ++t) f0[t] = fr[t];
    f0[0] = (T)0;
    for (int64_t t = 0; t < n; ++t) { h[t] = f0[t]; o[t] = f0[t]; }
    for (int64_t k = 2; k <= n - 1; ++k) {
      if (super) maxconv_one(h, f0, h2, n); else conv_one(h, f0, h2, n);
      for (int64_t t = 0; t < n; ++t) {
        h[t] = h2[t];
        if (super ? h[t] > o[t] : h[t] < o[t]) o[t] = h[t];
      }
    }
  }
  if (flags) *flags |= fl;
}

template <typename T>
void chain_rows(const T* curves, int64_t count, T* out, T* tmp, int64_t batch, int64_t n) {
  for (int64_t b = 0; b < batch; ++b) {
    T* o = out + b * n;
    for (int64_t t = 0; t < n; ++t) o[t] = curves[b * n + t];
    for (int64_t k = 1; k < count; ++k) {
      conv_one(o, curves + (k * batch + b) * n, tmp, n);
      for (int64_t t = 0; t < n; ++t) o[t] = tmp[t];
    }
  }
}

template <typename T>
void hdev_rows(const T* alpha, const T* beta, int32_t* out, int64_t batch, int64_t n, int32_t* flags) {
  int32_t fl = 0;
  for (int64_t b = 0; b < batch; ++b) {
    const T* a = alpha + b * n;
    const T* be = beta + b * n;
    int32_t h = 0;
    for (int64_t d = 0; d < n; ++d) {
      int32_t k = pinv_lower_one(be, n, a[d]);
      if (k == (int32_t)n) fl |= 4;
      int32_t term = k - (int32_t)d;
      if (term > h) h = term;
    }
    out[b] = h;
  }
  if (flags) *flags |= fl;
}

template <typename T>
void vdev_rows(const T* alpha, const T* beta, T* out, int64_t batch, int64_t n) {
  for (int64_t b = 0; b < batch; ++b) {
    T m = osub(alpha[b * n], beta[b * n]);
    for (int64_t d = 1; d < n; ++d) {
      T v = osub(alpha[b * n + d], beta[b * n + d]);
      if (v > m) m = v;
    }
    out[b] = m;
  }
}

template <typename T>
void conv_rows(const void* f, const void* g, void* out, int64_t batch, int64_t n, int64_t sf,
               int64_t sg, bool deconv) {
  for (int64_t b = 0; b < batch; ++b) {
    const T* fr = (const T*)f + b * sf;
    const T* gr = (const T*)g + b * sg;
    T* o = (T*)out + b * n;
    if (deconv) deconv_one(fr, gr, o, n); else conv_one(fr, gr, o, n);
  }
}

template <typename T>
void dual_rows(const void* f, const void* g, void* out, int64_t batch, int64_t n, int64_t sf,
               int64_t sg, bool deconv) {
  for (int64_t b = 0; b < batch; ++b) {
    const T* fr = (const T*)f + b * sf;
    const T* gr = (const T*)g + b * sg;
    T* o = (T*)out + b * n;
    if (deconv) mindeconv_one(fr, gr, o, n); else maxconv_one(fr, gr, o, n);
  }
}

}  // namespace

// dt: 0 = int32, 1 = int64, 2 = float64.  All pointers are host pointers; rows are
// contiguous with the given element strides (stride 0 broadcasts one curve).
extern "C" {

int oracle_num_threads() { return omp_get_max_threads(); }

// Overflowing integer additions / subtractions seen since the last reset: only the debug build
// counts them (-1: this build does not check).
long long oracle_overflow_count(int reset) {
#ifdef ORACLE_CHECK_OVERFLOW
  const long long c = g_overflows;
  if (reset) g_overflows = 0;
  return c;
#else
  (void)reset;
  return -1;
#endif
}

int oracle_minplus_conv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                        int64_t stride_f, int64_t stride_g, int dt) {
  if (dt == 0) conv_rows<int32_t>(f, g, out, batch, n, stride_f, stride_g, false);
  else if (dt == 1) conv_rows<int64_t>(f, g, out, batch, n, stride_f, stride_g, false);
  else if (dt == 2) conv_rows<double>(f, g, out, batch, n, stride_f, stride_g, false);
  else return -3;
  return 0;
}

int oracle_maxplus_deconv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                          int64_t stride_f, int64_t stride_g, int dt) {
  if (dt == 0) conv_rows<int32_t>(f, g, out, batch, n, stride_f, stride_g, true);
  else if (dt == 1) conv_rows<int64_t>(f, g, out, batch, n, stride_f, stride_g, true);
  else if (dt == 2) conv_rows<double>(f, g, out, batch, n, stride_f, stride_g, true);
  else return -3;
  return 0;
}

int oracle_maxplus_conv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                        int64_t stride_f, int64_t stride_g, int dt) {
  if (dt == 0) dual_rows<int32_t>(f, g, out, batch, n, stride_f, stride_g, false);
  else if (dt == 1) dual_rows<int64_t>(f, g, out, batch, n, stride_f, stride_g, false);
  else if (dt == 2) dual_rows<double>(f, g, out, batch, n, stride_f, stride_g, false);
  else return -3;
  return 0;
}

int oracle_minplus_deconv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                          int64_t stride_f, int64_t stride_g, int dt) {
  if (dt == 0) dual_rows<int32_t>(f, g, out, batch, n, stride_f, stride_g, true);
  else if (dt == 1) dual_rows<int64_t>(f, g, out, batch, n, stride_f, stride_g, true);
  else if (dt == 2) dual_rows<double>(f, g, out, batch, n, stride_f, stride_g, true);
  else return -3;
  return 0;
}

// Outputs t_idx[0..m) of one row pair (f, g of n samples); deconv = 0 convolution, 1 deconvolution.
int oracle_product_at(const void* f, const void* g, int64_t n, const int64_t* t_idx, int64_t m,
                      void* out, int deconv, int dt) {
  for (int64_t j = 0; j < m; ++j)
    if (t_idx[j] < 0 || t_idx[j] >= n) return -2;
  if (dt == 0) product_at((const int32_t*)f, (const int32_t*)g, n, t_idx, m, (int32_t*)out, deconv != 0);
  else if (dt == 1) product_at((const int64_t*)f, (const int64_t*)g, n, t_idx, m, (int64_t*)out, deconv != 0);
  else if (dt == 2) product_at((const double*)f, (const double*)g, n, t_idx, m, (double*)out, deconv != 0);
  else return -3;
  return 0;
}

int oracle_pseudo_inverse(const void* f, int64_t n, const void* x, int64_t m, int32_t* out_idx,
                          int64_t batch, int mode, int dt) {
  if (mode != 0 && mode != 1) return -8;
  if (dt == 0) pinv_rows((const int32_t*)f, n, (const int32_t*)x, m, out_idx, batch, mode);
  else if (dt == 1) pinv_rows((const int64_t*)f, n, (const int64_t*)x, m, out_idx, batch, mode);
  else if (dt == 2) pinv_rows((const double*)f, n, (const double*)x, m, out_idx, batch, mode);
  else return -3;
  return 0;
}

int oracle_compose(const void* outer, int64_t n_outer, const int32_t* inner, int64_t n, void* out,
                   int64_t batch, int dt, int32_t* flags) {
  if (dt == 0) compose_rows((const int32_t*)outer, n_outer, inner, n, (int32_t*)out, batch, flags);
  else if (dt == 1) compose_rows((const int64_t*)outer, n_outer, inner, n, (int64_t*)out, batch, flags);
  else if (dt == 2) compose_rows((const double*)outer, n_outer, inner, n, (double*)out, batch, flags);
  else return -3;
  return 0;
}

// tmp: batch*n scratch of the value type (receives alpha^u (x) beta^u).
int oracle_gpc_step(const void* alpha_u, const void* beta_u, const void* beta_l, void* alpha_u_out,
                    void* beta_l_out, void* tmp, int64_t batch, int64_t n, int dt) {
  if (dt == 0) gpc_rows((const int32_t*)alpha_u, (const int32_t*)beta_u, (const int32_t*)beta_l,
                        (int32_t*)alpha_u_out, (int32_t*)beta_l_out, (int32_t*)tmp, batch, n);
  else if (dt == 1) gpc_rows((const int64_t*)alpha_u, (const int64_t*)beta_u, (const int64_t*)beta_l,
                             (int64_t*)alpha_u_out, (int64_t*)beta_l_out, (int64_t*)tmp, batch, n);
  else if (dt == 2) gpc_rows((const double*)alpha_u, (const double*)beta_u, (const double*)beta_l,
                             (double*)alpha_u_out, (double*)beta_l_out, (double*)tmp, batch, n);
  else return -3;
  return 0;
}

int oracle_gpc_step_lower(const void* alpha_l, const void* beta_u, const void* beta_l, void* alpha_l_out,
                          void* beta_u_out, void* tmp, int64_t batch, int64_t n, int dt) {
  if (dt == 0) gpc_lower_rows((const int32_t*)alpha_l, (const int32_t*)beta_u, (const int32_t*)beta_l,
                              (int32_t*)alpha_l_out, (int32_t*)beta_u_out, (int32_t*)tmp, batch, n);
  else if (dt == 1) gpc_lower_rows((const int64_t*)alpha_l, (const int64_t*)beta_u, (const int64_t*)beta_l,
                                   (int64_t*)alpha_l_out, (int64_t*)beta_u_out, (int64_t*)tmp, batch, n);
  else if (dt == 2) gpc_lower_rows((const double*)alpha_l, (const double*)beta_u, (const double*)beta_l,
                                   (double*)alpha_l_out, (double*)beta_u_out, (double*)tmp, batch, n);
  else return -3;
  return 0;
}

// scratch: 3*n elements of the value type
int oracle_closure(const void* f, void* out, void* scratch, int64_t batch, int64_t n, int super, int dt,
                   int32_t* flags) {
  if (dt == 0) { int32_t* s = (int32_t*)scratch; closure_rows((const int32_t*)f, (int32_t*)out, s, s + n, s + 2 * n, batch, n, super != 0, flags); }
  else if (dt == 1) { int64_t* s = (int64_t*)scratch; closure_rows((const int64_t*)f, (int64_t*)out, s, s + n, s + 2 * n, batch, n, super != 0, flags); }
  else if (dt == 2) { double* s = (double*)scratch; closure_rows((const double*)f, (double*)out, s, s + n, s + 2 * n, batch, n, super != 0, flags); }
  else return -3;
  return 0;
}

// curves: [count][batch][n]; scratch: n elements
int oracle_conv_chain(const void* curves, int64_t count, void* out, void* scratch, int64_t batch, int64_t n,
                      int dt) {
  if (count < 1) return -2;
  if (dt == 0) chain_rows((const int32_t*)curves, count, (int32_t*)out, (int32_t*)scratch, batch, n);
  else if (dt == 1) chain_rows((const int64_t*)curves, count, (int64_t*)out, (int64_t*)scratch, batch, n);
  else if (dt == 2) chain_rows((const double*)curves, count, (double*)out, (double*)scratch, batch, n);
  else return -3;
  return 0;
}

int oracle_max_hdev(const void* alpha, const void* beta, int32_t* out, int64_t batch, int64_t n,
                    int dt, int32_t* flags) {
  if (dt == 0) hdev_rows((const int32_t*)alpha, (const int32_t*)beta, out, batch, n, flags);
  else if (dt == 1) hdev_rows((const int64_t*)alpha, (const int64_t*)beta, out, batch, n, flags);
  else if (dt == 2) hdev_rows((const double*)alpha, (const double*)beta, out, batch, n, flags);
  else return -3;
  return 0;
}

int oracle_max_vdev(const void* alpha, const void* beta, void* out, int64_t batch, int64_t n, int dt) {
  if (dt == 0) vdev_rows((const int32_t*)alpha, (const int32_t*)beta, (int32_t*)out, batch, n);
  else if (dt == 1) vdev_rows((const int64_t*)alpha, (const int64_t*)beta, (int64_t*)out, batch, n);
  else if (dt == 2) vdev_rows((const double*)alpha, (const double*)beta, (double*)out, batch, n);
  else return -3;
  return 0;
}

}  // extern "C"
