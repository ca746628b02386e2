// C-ABI entry points of librtc: argument validation and launch sequencing only.
#include <hip/hip_runtime.h>

#include "rtc_internal.h"

using namespace rtc;

namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_shape(int64_t batch, int64_t n) {
  if (batch < 1 || n < 1 || n > RTC_MAX_N || batch > 0x7fffffffLL) return RTC_ERR_SHAPE;
  return RTC_OK;
}

int check_product(const void* f, const void* g, const void* out, int64_t batch, int64_t n,
                  int64_t stride_f, int64_t stride_g, int dt, const void* ws, size_t ws_bytes,
                  const int32_t* dev_flags) {
  if (f == nullptr || g == nullptr || out == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (int rc = check_shape(batch, n)) return rc;
  if ((stride_f != 0 && stride_f < n) || (stride_g != 0 && stride_g < n)) return RTC_ERR_STRIDE;
  if (!aligned(f, es) || !aligned(g, es) || !aligned(out, es) || !aligned(dev_flags, 4) ||
      !aligned(ws, 16))
    return RTC_ERR_ALIGN;
  // int64 rows need the workspace; for int32 it is optional (it enables the packed fast path)
  if (dt == RTC_I64 && (ws == nullptr || ws_bytes < tropical_workspace_bytes(batch, n, dt)))
    return RTC_ERR_WORKSPACE;
  return RTC_OK;
}

}  // namespace

extern "C" {

int rtc_minplus_conv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                     int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes,
                     int32_t* dev_flags, void* hip_stream) {
  if (int rc = check_product(f, g, out, batch, n, stride_f, stride_g, dt, ws, ws_bytes, dev_flags)) return rc;
  return validated([&] { return launch_tropical(RTC_OP_CONV, f, g, out, batch, n, stride_f, stride_g, dt, nullptr, ws, ws_bytes,
                         dev_flags, static_cast<hipStream_t>(hip_stream)); });
}

int rtc_maxplus_conv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                     int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes,
                     int32_t* dev_flags, void* hip_stream) {
  if (int rc = check_product(f, g, out, batch, n, stride_f, stride_g, dt, ws, ws_bytes, dev_flags)) return rc;
  return validated([&] { return launch_tropical(RTC_OP_MAXCONV, f, g, out, batch, n, stride_f, stride_g, dt, nullptr, ws, ws_bytes,
                         dev_flags, static_cast<hipStream_t>(hip_stream)); });
}

int rtc_minplus_deconv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                       int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes,
                       int32_t* dev_flags, void* hip_stream) {
  if (int rc = check_product(f, g, out, batch, n, stride_f, stride_g, dt, ws, ws_bytes, dev_flags)) return rc;
  return validated([&] { return launch_tropical(RTC_OP_MINDECONV, f, g, out, batch, n, stride_f, stride_g, dt, nullptr, ws, ws_bytes,
                         dev_flags, static_cast<hipStream_t>(hip_stream)); });
}

int rtc_maxplus_deconv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                       int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes,
                       int32_t* dev_flags, void* hip_stream) {
  if (int rc = check_product(f, g, out, batch, n, stride_f, stride_g, dt, ws, ws_bytes, dev_flags)) return rc;
  return validated([&] { return launch_tropical(RTC_OP_DECONV, f, g, out, batch, n, stride_f, stride_g, dt, nullptr, ws, ws_bytes,
                         dev_flags, static_cast<hipStream_t>(hip_stream)); });
}

int rtc_product_census(int op, const void* f, const void* g, int64_t batch, int64_t n, int64_t stride_f,
                       int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes, uint64_t* counts,
                       void* hip_stream) {
  if (counts == nullptr) return RTC_ERR_NULL;
  if (op != RTC_OP_CONV && op != RTC_OP_DECONV && op != RTC_OP_MAXCONV && op != RTC_OP_MINDECONV) return RTC_ERR_MODE;
  if (!aligned(counts, 8)) return RTC_ERR_ALIGN;
  // `counts` stands in for the output in the argument check (non-null, aligned); no output is written
  if (int rc = check_product(f, g, counts, batch, n, stride_f, stride_g, dt, ws, ws_bytes, nullptr)) return rc;
  static_assert(sizeof(unsigned long long) == sizeof(uint64_t), "census words");
  return validated([&] { return launch_tropical(op, f, g, nullptr, batch, n, stride_f, stride_g, dt, nullptr, ws, ws_bytes, nullptr,
                         static_cast<hipStream_t>(hip_stream), reinterpret_cast<unsigned long long*>(counts)); });
}

int rtc_product_structure(int op, const void* f, const void* g, int32_t* codes, int64_t batch, int64_t n,
                          int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* hip_stream) {
  return rtc_product_periods(op, f, g, codes, nullptr, batch, n, stride_f, stride_g, dt, hip_stream);
}

int rtc_product_periods(int op, const void* f, const void* g, int32_t* codes, int32_t* periods, int64_t batch,
                        int64_t n, int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* hip_stream) {
  if (f == nullptr || g == nullptr || codes == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (op != RTC_OP_CONV && op != RTC_OP_DECONV && op != RTC_OP_MAXCONV && op != RTC_OP_MINDECONV) return RTC_ERR_MODE;
  if (int rc = check_shape(batch, n)) return rc;
  if ((stride_f != 0 && stride_f < n) || (stride_g != 0 && stride_g < n)) return RTC_ERR_STRIDE;
  if (!aligned(f, es) || !aligned(g, es) || !aligned(codes, 4) || !aligned(periods, 4)) return RTC_ERR_ALIGN;
  return validated([&] { return launch_structure_probe(op, f, g, codes, periods, batch, n, stride_f, stride_g, dt,
                                static_cast<hipStream_t>(hip_stream)); });
}

int rtc_pseudo_inverse(const void* f, int64_t n, const void* x, int64_t m, int32_t* out_idx,
                       int64_t batch, rtc_inv_mode mode, rtc_dtype dt, void* hip_stream) {
  if (f == nullptr || x == nullptr || out_idx == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (mode != RTC_INV_LOWER && mode != RTC_INV_UPPER) return RTC_ERR_MODE;
  if (int rc = check_shape(batch, n)) return rc;
  if (m < 1 || m > RTC_MAX_N) return RTC_ERR_SHAPE;
  if (!aligned(f, es) || !aligned(x, es) || !aligned(out_idx, 4)) return RTC_ERR_ALIGN;
  return validated([&] { return launch_pseudo_inverse(f, n, x, m, out_idx, batch, mode, dt, static_cast<hipStream_t>(hip_stream)); });
}

int rtc_compose(const void* outer, int64_t n_outer, const int32_t* inner, int64_t n, void* out,
                int64_t batch, rtc_dtype dt, int32_t* dev_flags, void* hip_stream) {
  if (outer == nullptr || inner == nullptr || out == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (int rc = check_shape(batch, n)) return rc;
  if (n_outer < 1 || n_outer > RTC_MAX_N) return RTC_ERR_SHAPE;
  if (!aligned(outer, es) || !aligned(out, es) || !aligned(inner, 4) || !aligned(dev_flags, 4))
    return RTC_ERR_ALIGN;
  return validated([&] { return launch_compose(outer, n_outer, inner, n, out, batch, dt, dev_flags,
                        static_cast<hipStream_t>(hip_stream)); });
}

int rtc_gpc_step(const rtc_gpc_args* a, void* hip_stream) {
  if (a == nullptr || a->alpha_u == nullptr || a->beta_u == nullptr || a->beta_l == nullptr ||
      a->alpha_u_out == nullptr || a->beta_l_out == nullptr)
    return RTC_ERR_NULL;
  const size_t es = elem_size(a->dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (int rc = check_shape(a->batch, a->n)) return rc;
  if ((a->events_lower != nullptr || a->events_upper != nullptr) && a->gamma_u == nullptr) return RTC_ERR_NULL;
  if (a->alpha_l != nullptr && (a->alpha_l_out == nullptr || a->beta_u_out == nullptr)) return RTC_ERR_NULL;
  if ((a->events_u_lower != nullptr || a->events_u_upper != nullptr) &&
      (a->gamma_l == nullptr || a->alpha_l == nullptr))
    return RTC_ERR_NULL;
  if (a->gamma_l != nullptr && (a->n_gamma_l < 1 || a->n_gamma_l > RTC_MAX_N)) return RTC_ERR_SHAPE;
  if (a->gamma_u != nullptr && (a->n_gamma < 1 || a->n_gamma > RTC_MAX_N)) return RTC_ERR_SHAPE;
  if (!aligned(a->alpha_u, es) || !aligned(a->beta_u, es) || !aligned(a->beta_l, es) ||
      !aligned(a->alpha_u_out, es) || !aligned(a->beta_l_out, es) || !aligned(a->gamma_u, es) ||
      !aligned(a->events_lower, 4) || !aligned(a->events_upper, 4) || !aligned(a->dev_flags, 4) ||
      !aligned(a->ws, 16) || !aligned(a->alpha_l, es) || !aligned(a->alpha_l_out, es) ||
      !aligned(a->beta_u_out, es) || !aligned(a->gamma_l, es) || !aligned(a->events_u_lower, 4) ||
      !aligned(a->events_u_upper, 4))
    return RTC_ERR_ALIGN;
  const size_t need = rtc_workspace_bytes(RTC_OP_GPC, a->batch, a->n, a->dt);
  if (a->ws == nullptr || a->ws_bytes < need) return RTC_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int64_t batch = a->batch, n = a->n;
  // workspace: [c = alpha_u (x) beta_u : batch*n elements][scratch of the products]
  char* c = static_cast<char*>(a->ws);
  const size_t c_bytes = ((size_t)batch * n * es + 255) / 256 * 256;
  void* sub_ws = c + c_bytes;
  const size_t sub_bytes = a->ws_bytes - c_bytes;
  // (the whole sequence runs dry first: a launch that would not fit is reported before any is enqueued)
  return validated([&]() -> int {
  int rc = launch_tropical(RTC_OP_CONV, a->alpha_u, a->beta_u, c, batch, n, n, n, a->dt, nullptr, sub_ws,
                           sub_bytes, a->dev_flags, stream);
  if (rc != RTC_OK) return rc;
  rc = launch_tropical(RTC_OP_DECONV, c, a->beta_l, a->alpha_u_out, batch, n, n, n, a->dt, a->beta_u, sub_ws,
                       sub_bytes, a->dev_flags, stream);
  if (rc != RTC_OK) return rc;
  // beta'^l and, while its values are in registers, their event-domain images: one kernel
  // (c is free again: the segment totals of the scan go there)
  rc = launch_residual_service(a->beta_l, a->alpha_u, a->beta_l_out, batch, n, a->dt, false, stream, c, a->gamma_u,
                               a->n_gamma, a->events_lower, a->events_upper);
  if (rc != RTC_OK) return rc;
  if (a->alpha_l != nullptr) {
    // lower arrival / upper service side: alpha'^l = min((alpha^l (/) beta^u) (x) beta^l, beta^l),
    // beta'^u[D] = max(0, min_{l>=D} beta^u[l] - alpha^l[l]); the intermediate reuses c
    rc = launch_tropical(RTC_OP_DECONV, a->alpha_l, a->beta_u, c, batch, n, n, n, a->dt, nullptr, sub_ws,
                         sub_bytes, a->dev_flags, stream);
    if (rc != RTC_OK) return rc;
    rc = launch_tropical(RTC_OP_CONV, c, a->beta_l, a->alpha_l_out, batch, n, n, n, a->dt, a->beta_l, sub_ws,
                         sub_bytes, a->dev_flags, stream);
    if (rc != RTC_OK) return rc;
    rc = launch_residual_service(a->beta_u, a->alpha_l, a->beta_u_out, batch, n, a->dt, true, stream, c, a->gamma_l,
                                 a->n_gamma_l, a->events_u_lower, a->events_u_upper);
    if (rc != RTC_OK) return rc;
  }
  return RTC_OK;
  });
}

namespace {

// Layout of the closure / chain workspace: two ping-pong curves, then the product workspace.
size_t pingpong_bytes(int64_t batch, int64_t n, size_t es) { return 2 * (((size_t)batch * n * es + 255) / 256 * 256); }

int closure(const void* f, void* out, int64_t batch, int64_t n, int dt, void* ws, size_t ws_bytes,
            int32_t* dev_flags, hipStream_t stream, bool super) {
  if (f == nullptr || out == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (int rc = check_shape(batch, n)) return rc;
  if (!aligned(f, es) || !aligned(out, es) || !aligned(dev_flags, 4) || !aligned(ws, 16)) return RTC_ERR_ALIGN;
  if (ws == nullptr || ws_bytes < rtc_workspace_bytes(RTC_OP_CLOSURE, batch, n, (rtc_dtype)dt)) return RTC_ERR_WORKSPACE;
  if (dt == RTC_F64) {
    // Floating point: a k-fold sum depends on the order of its additions, so the powers are formed
    // as the definition writes them, one factor at a time from the left: h <- h (x) g, n - 2 times,
    // with g = f, g[0] = 0.  Because g[0] = 0, the candidate s = t of (h (x) g)[t] is h[t] itself:
    // every power lies below (above, for the max-plus dual) the one before it at every sample, and
    // the minimum (maximum) over all powers is the last one.  Workspace: g and two curves in turn.
    const size_t one = ((size_t)batch * n * es + 255) / 256 * 256;
    char* g = static_cast<char*>(ws);
    char* buf[2] = {g + one, g + 2 * one};
    const int64_t products = n > 2 ? n - 2 : 0;
    return validated([&]() -> int {
      int rc = launch_closure_init(f, products == 0 ? out : g, batch, n, dt, super, dev_flags, stream);
      if (rc != RTC_OK) return rc;
      const void* h = g;
      for (int64_t j = 0; j < products; ++j) {
        void* dst = (j == products - 1) ? out : buf[j & 1];
        rc = launch_tropical(super ? RTC_OP_MAXCONV : RTC_OP_CONV, h, g, dst, batch, n, n, n, dt, nullptr, nullptr, 0,
                             dev_flags, stream);
        if (rc != RTC_OK) return rc;
        h = dst;
      }
      return RTC_OK;
    });
  }
  int squarings = 0;   // after j squarings every k-fold term with k <= 2^j is covered; k <= n-1 suffices
  while (((int64_t)1 << squarings) < n - 1) ++squarings;
  const size_t half = pingpong_bytes(batch, n, es) / 2;
  char* buf[2] = {static_cast<char*>(ws), static_cast<char*>(ws) + half};
  void* sub_ws = static_cast<char*>(ws) + 2 * half;
  const size_t sub_bytes = ws_bytes - 2 * half;
  return validated([&]() -> int {
    int rc = launch_closure_init(f, squarings == 0 ? out : buf[0], batch, n, dt, super, dev_flags, stream);
    if (rc != RTC_OK) return rc;
    for (int j = 0; j < squarings; ++j) {
      const void* src = buf[j & 1];
      void* dst = (j == squarings - 1) ? out : buf[(j + 1) & 1];
      rc = launch_tropical(super ? RTC_OP_MAXCONV : RTC_OP_CONV, src, src, dst, batch, n, n, n, dt, nullptr, sub_ws,
                           sub_bytes, dev_flags, stream);
      if (rc != RTC_OK) return rc;
    }
    return RTC_OK;
  });
}

}  // namespace

int rtc_subadditive_closure(const void* f, void* out, int64_t batch, int64_t n, rtc_dtype dt, void* ws,
                            size_t ws_bytes, int32_t* dev_flags, void* hip_stream) {
  return closure(f, out, batch, n, dt, ws, ws_bytes, dev_flags, static_cast<hipStream_t>(hip_stream), false);
}

int rtc_superadditive_closure(const void* f, void* out, int64_t batch, int64_t n, rtc_dtype dt, void* ws,
                              size_t ws_bytes, int32_t* dev_flags, void* hip_stream) {
  return closure(f, out, batch, n, dt, ws, ws_bytes, dev_flags, static_cast<hipStream_t>(hip_stream), true);
}

int rtc_conv_chain(const void* curves, int64_t count, void* out, int64_t batch, int64_t n, rtc_dtype dt,
                   void* ws, size_t ws_bytes, int32_t* dev_flags, void* hip_stream) {
  if (curves == nullptr || out == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (int rc = check_shape(batch, n)) return rc;
  if (count < 1 || count > 65536) return RTC_ERR_SHAPE;
  if (!aligned(curves, es) || !aligned(out, es) || !aligned(dev_flags, 4) || !aligned(ws, 16)) return RTC_ERR_ALIGN;
  if (ws == nullptr || ws_bytes < rtc_workspace_bytes(RTC_OP_CHAIN, batch, n, dt)) return RTC_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const size_t curve_bytes = (size_t)batch * n * es;
  const char* base = static_cast<const char*>(curves);
  if (count == 1) return validated([&] { return launch_copy(base, out, batch * n, dt, stream); });
  const size_t half = pingpong_bytes(batch, n, es) / 2;
  char* buf[2] = {static_cast<char*>(ws), static_cast<char*>(ws) + half};
  void* sub_ws = static_cast<char*>(ws) + 2 * half;
  const size_t sub_bytes = ws_bytes - 2 * half;
  return validated([&]() -> int {
    const void* acc = base;
    for (int64_t k = 1; k < count; ++k) {
      void* dst = (k == count - 1) ? out : buf[k & 1];
      int rc = launch_tropical(RTC_OP_CONV, acc, base + k * curve_bytes, dst, batch, n, n, n, dt, nullptr, sub_ws,
                               sub_bytes, dev_flags, stream);
      if (rc != RTC_OK) return rc;
      acc = dst;
    }
    return RTC_OK;
  });
}

int rtc_max_hdev(const void* alpha, const void* beta, int32_t* out, int64_t batch, int64_t n,
                 rtc_dtype dt, int32_t* dev_flags, void* hip_stream) {
  if (alpha == nullptr || beta == nullptr || out == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (int rc = check_shape(batch, n)) return rc;
  if (!aligned(alpha, es) || !aligned(beta, es) || !aligned(out, 4) || !aligned(dev_flags, 4))
    return RTC_ERR_ALIGN;
  return validated([&] { return launch_max_hdev(alpha, beta, out, batch, n, dt, dev_flags, static_cast<hipStream_t>(hip_stream)); });
}

int rtc_max_deviations(const void* alpha, const void* beta, int32_t* out_h, void* out_v, int64_t batch, int64_t n,
                       rtc_dtype dt, int32_t* dev_flags, void* hip_stream) {
  if (alpha == nullptr || beta == nullptr || out_h == nullptr || out_v == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (int rc = check_shape(batch, n)) return rc;
  if (!aligned(alpha, es) || !aligned(beta, es) || !aligned(out_h, 4) || !aligned(out_v, es) || !aligned(dev_flags, 4))
    return RTC_ERR_ALIGN;
  return validated([&] { return launch_max_hdev(alpha, beta, out_h, batch, n, dt, dev_flags, static_cast<hipStream_t>(hip_stream), out_v); });
}

int rtc_validate_monotone(const void* f, int64_t batch, int64_t n, int64_t stride, rtc_dtype dt,
                          int32_t* first_bad, int32_t* dev_flags, void* hip_stream) {
  if (f == nullptr || dev_flags == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (int rc = check_shape(batch, n)) return rc;
  if (stride != 0 && stride < n) return RTC_ERR_STRIDE;
  if (!aligned(f, es) || !aligned(first_bad, 4) || !aligned(dev_flags, 4)) return RTC_ERR_ALIGN;
  return validated([&] { return launch_validate_monotone(f, batch, n, stride, dt, first_bad, dev_flags, static_cast<hipStream_t>(hip_stream)); });
}

int rtc_max_vdev(const void* alpha, const void* beta, void* out, int64_t batch, int64_t n,
                 rtc_dtype dt, void* hip_stream) {
  if (alpha == nullptr || beta == nullptr || out == nullptr) return RTC_ERR_NULL;
  const size_t es = elem_size(dt);
  if (es == 0) return RTC_ERR_DTYPE;
  if (int rc = check_shape(batch, n)) return rc;
  if (!aligned(alpha, es) || !aligned(beta, es) || !aligned(out, es)) return RTC_ERR_ALIGN;
  return validated([&] { return launch_max_vdev(alpha, beta, out, batch, n, dt, static_cast<hipStream_t>(hip_stream)); });
}

size_t rtc_workspace_bytes(int op, int64_t batch, int64_t n, rtc_dtype dt) {
  const size_t es = elem_size(dt);
  if (es == 0 || check_shape(batch, n) != RTC_OK) return 0;
  const size_t prod = tropical_workspace_bytes(batch, n, dt);
  switch (op) {
    case RTC_OP_CONV:
    case RTC_OP_DECONV:
    case RTC_OP_MAXCONV:
    case RTC_OP_MINDECONV:
      return prod;
    case RTC_OP_GPC:
      return ((size_t)batch * n * es + 255) / 256 * 256 + prod;
    case RTC_OP_CLOSURE:
      if (dt == RTC_F64) return 3 * (((size_t)batch * n * es + 255) / 256 * 256);   // g and two powers in turn
      return 2 * (((size_t)batch * n * es + 255) / 256 * 256) + prod;
    case RTC_OP_CHAIN:
      return 2 * (((size_t)batch * n * es + 255) / 256 * 256) + prod;
    default:
      return 0;
  }
}

int rtc_set_packed_min_work(double batch_times_n_squared) {
  if (!(batch_times_n_squared >= 0.0)) return RTC_ERR_SHAPE;
  rtc::g_packed_min_work = batch_times_n_squared;
  return RTC_OK;
}

int rtc_set_packed_small_n(int64_t n) {
  if (n < 0) return RTC_ERR_SHAPE;
  rtc::g_packed_small_n = n;
  return RTC_OK;
}

int rtc_set_small_problem_items(int64_t items) {
  if (items < 0) return RTC_ERR_SHAPE;
  rtc::g_small_items = items;
  return RTC_OK;
}

int rtc_set_rebase_wide(int mode) {
  if (mode < 0 || mode > 2) return RTC_ERR_MODE;
  rtc::g_rebase_wide = mode;
  return RTC_OK;
}

int rtc_set_structure_paths(int enabled) {
  rtc::g_structure_paths = enabled != 0;
  return RTC_OK;
}

const char* rtc_strerror(int status) {
  switch (status) {
    case RTC_OK: return "ok";
    case RTC_ERR_NULL: return "required pointer is NULL";
    case RTC_ERR_SHAPE: return "batch or n out of range";
    case RTC_ERR_DTYPE: return "unknown dtype";
    case RTC_ERR_ALIGN: return "pointer not aligned to its element size";
    case RTC_ERR_STRIDE: return "stride must be 0 or >= n";
    case RTC_ERR_WORKSPACE: return "workspace missing or too small";
    case RTC_ERR_HIP: return "HIP runtime error while enqueueing";
    case RTC_ERR_MODE: return "unknown mode";
    default: return "unknown status";
  }
}

int rtc_selftest_half_minmax(uint32_t* mismatches, void* hip_stream) {
  if (mismatches == nullptr) return RTC_ERR_NULL;
  if (!aligned(mismatches, 4)) return RTC_ERR_ALIGN;
  return validated([&] { return launch_selftest_half_minmax(mismatches, static_cast<hipStream_t>(hip_stream)); });
}

int rtc_device_info(int* cu_count, int* clock_khz, int* lds_bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return RTC_ERR_HIP;
  int v = 0;
  if (cu_count) {
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return RTC_ERR_HIP;
    *cu_count = v;
  }
  if (clock_khz) {
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeClockRate, dev) != hipSuccess) return RTC_ERR_HIP;
    *clock_khz = v;
  }
  if (lds_bytes) {
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return RTC_ERR_HIP;
    *lds_bytes = v;
  }
  return RTC_OK;
}

}  // extern "C"
