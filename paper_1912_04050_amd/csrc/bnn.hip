// Binary convolution layer for gfx950: channel packing, filter-bank preparation and the
// xor / popcount convolution with the integrated batch-norm threshold, binarisation and output
// packing (the paper's binary convolution operation, channel compression, layer integration,
// workload optimisation and branch-free selection sections).
//
// Mapping.  One wave64 per workgroup.  The 64 lanes are 64 consecutive filters k; the wave owns
// TM consecutive output pixels of one output row.  An activation word is then the same for all
// lanes, so it lives in a scalar register and is the scalar source of v_xor_b32; a lane's
// filter word is the vector source.  Per (pixel, word) the kernel issues v_xor_b32 +
// v_bcnt_u32_b32 (popcount with accumulate): 2 VALU instructions per 32 binary
// multiply-accumulates per lane, nothing else in the inner loop.  The TM pixels share one strip
// of (TM-1) stride + S input pixels per filter row, loaded once into scalar registers.  The
// paper's "one thread computes 8 filters and packs a byte" becomes "one wavefront computes 64
// filters and a ballot packs two words": the 64 binarised results of a pixel are the 64 bits of
// the wave's compare mask.
//
// Image borders: a filter row outside the image is skipped (the same for all pixels of the
// strip); a strip pixel left or right of the image is read as an all-zero word, and what the
// zero word wrongly contributed, popcount(w[k][r][s][:]), is taken off again in the epilogue
// from the per-(tap, filter) table that bnn_pack_weights appends to the filter bank.
#include <hip/hip_runtime.h>

#include "bnn.h"
#include "rtc_internal.h"

namespace bnn {
namespace {

constexpr int kProfileKind = 32;   // rtc_profile_read() kind of the convolution kernel

inline int hip_status() { return hipGetLastError() == hipSuccess ? BNN_OK : BNN_ERR_HIP; }

// ---- channel packing ------------------------------------------------------------------------

// One wave per (row, block of 64 channels): coalesced reads, the compare mask is the packing.
template <typename T>
__global__ __launch_bounds__(64) void pack_channels_kernel(const T* __restrict__ x, uint32_t* __restrict__ words,
                                                           int64_t rows, int C, int Cw, int cblocks) {
  const int64_t row = blockIdx.x / cblocks;
  const int cb = blockIdx.x % cblocks;
  const int c = cb * 64 + threadIdx.x;
  bool bit = false;
  if (c < C) bit = x[row * C + c] > (T)0;
  const unsigned long long mask = __ballot(bit);
  if (threadIdx.x < 2) {
    const int j = cb * 2 + threadIdx.x;
    if (j < Cw) words[row * Cw + j] = (uint32_t)(threadIdx.x ? mask >> 32 : mask);
  }
}

// ---- filter bank ------------------------------------------------------------------------------

// Layout: word (tap, cw, k) at (tap * Cw + cw) * Kp + k, Kp = K rounded up to 64 (zero filters
// beyond K), then the table pop[tap][k] = sum_cw popcount(word) at R*S*Cw*Kp + tap * Kp + k.
__global__ __launch_bounds__(256) void pack_weights_kernel(const int8_t* __restrict__ w, uint32_t* __restrict__ packed,
                                                           int K, int taps, int C, int Cw, int Kp) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;     // (tap, cw, k), k fastest
  const int64_t total = (int64_t)taps * Cw * Kp;
  if (idx >= total) return;
  const int k = (int)(idx % Kp);
  const int cw = (int)((idx / Kp) % Cw);
  const int tap = (int)(idx / ((int64_t)Kp * Cw));
  uint32_t word = 0;
  if (k < K) {
    const int8_t* src = w + ((int64_t)k * taps + tap) * C + cw * 32;
    const int m = min(32, C - cw * 32);
    for (int i = 0; i < m; ++i) word |= (src[i] > 0 ? 1u : 0u) << i;
  }
  packed[idx] = word;
}

__global__ __launch_bounds__(256) void weight_popcount_kernel(uint32_t* __restrict__ packed, int taps, int Cw, int Kp) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;     // (tap, k)
  if (idx >= (int64_t)taps * Kp) return;
  const int k = (int)(idx % Kp), tap = (int)(idx / Kp);
  uint32_t total = 0;
  for (int cw = 0; cw < Cw; ++cw) total += __popc(packed[((int64_t)tap * Cw + cw) * Kp + k]);
  packed[(int64_t)taps * Cw * Kp + idx] = total;
}

// ---- convolution ------------------------------------------------------------------------------

struct ConvArgs {
  const uint32_t* x;       // [N][H][W][Cw]
  const uint32_t* w;       // filter bank, see pack_weights_kernel
  const float* xi;         // [K] or null
  const float* gamma;      // [K] or null
  int32_t* out_x1;         // [N][Ho][Wo][K] or null
  uint32_t* out_x4;        // [N][Ho][Wo][Kw] or null
  int32_t H, W, C, Cw, K, Kp, Kw, R, pad, Ho, Wo, kblocks, wtiles;
};

// S = filter width, STRIDE, QC = words of a pixel handled per pass (divides Cw), TM = output
// pixels per wave.
template <int S, int STRIDE, int QC, int TM>
__global__ __launch_bounds__(64) void bconv_kernel(const ConvArgs p) {
  constexpr int PS = (TM - 1) * STRIDE + S;    // input pixels of the strip
  const int lane = threadIdx.x;
  uint32_t b = blockIdx.x;
  const int kb = b % p.kblocks; b /= p.kblocks;
  const int wt = b % p.wtiles; b /= p.wtiles;
  const int ho = b % p.Ho;
  const int n = b / p.Ho;
  const int k = kb * 64 + lane;
  const int wo0 = wt * TM;
  const int wi0 = wo0 * STRIDE - p.pad;
  const uint32_t* __restrict__ xw = p.x;
  const uint32_t* __restrict__ ww = p.w;

  uint32_t acc[TM];
#pragma unroll
  for (int j = 0; j < TM; ++j) acc[j] = 0;

  // word offsets of the strip's pixels inside an input row (clamped into the row: the loads
  // below are unconditional, a pixel outside the image is zeroed after the load)
  uint32_t poff[PS];
  bool pin[PS];
#pragma unroll
  for (int i = 0; i < PS; ++i) {
    const int wi = wi0 + i;
    pin[i] = wi >= 0 && wi < p.W;
    poff[i] = (uint32_t)(pin[i] ? wi : 0) * (uint32_t)p.Cw;
  }
  const uint32_t wstep = (uint32_t)p.Kp;   // words between consecutive (tap, cw) rows of the filter bank

  int rows_inside = 0;
  for (int r = 0; r < p.R; ++r) {
    const int hi = ho * STRIDE - p.pad + r;
    if (hi < 0 || hi >= p.H) continue;           // wave-uniform
    ++rows_inside;
    const uint32_t* __restrict__ xrow = xw + ((int64_t)n * p.H + hi) * p.W * p.Cw;
    const uint32_t* __restrict__ wrow = ww + (int64_t)r * S * p.Cw * p.Kp;   // wave-uniform; the lane adds k
    for (int c0 = 0; c0 < p.Cw; c0 += QC) {
      uint32_t a[PS][QC];                        // wave-uniform: scalar registers
#pragma unroll
      for (int i = 0; i < PS; ++i) {
        const uint32_t* __restrict__ src = xrow + (poff[i] + (uint32_t)c0);
#pragma unroll
        for (int q = 0; q < QC; ++q) {
          const uint32_t v = src[q];
          a[i][q] = pin[i] ? v : 0u;
        }
      }
#pragma unroll
      for (int s = 0; s < S; ++s) {
        const uint32_t* __restrict__ wtap = wrow + (uint32_t)(s * p.Cw + c0) * wstep;
        uint32_t wv[QC];
#pragma unroll
        for (int q = 0; q < QC; ++q) wv[q] = (wtap + q * wstep)[k];
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
          for (int q = 0; q < QC; ++q) acc[j] += __popc(a[j * STRIDE + s][q] ^ wv[q]);
      }
    }
  }

  // epilogue: x1 = Len - 2 popcount, Len = C x (taps inside the image); then the integrated layer
  const uint32_t* __restrict__ pop = ww + (int64_t)p.R * S * p.Cw * p.Kp;
  const bool touches_border = wi0 < 0 || wi0 + PS > p.W;   // wave-uniform
  const float xi = (p.out_x4 != nullptr && k < p.K) ? p.xi[k] : 0.f;
  const float gamma = (p.out_x4 != nullptr && k < p.K) ? p.gamma[k] : 0.f;
  unsigned long long mine = 0;
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int wo = wo0 + j;
    if (wo >= p.Wo) break;                       // wave-uniform
    int cols_inside = S;
    uint32_t wrong = 0;
    if (touches_border) {
      cols_inside = 0;
#pragma unroll
      for (int s = 0; s < S; ++s) {
        const int wi = wo * STRIDE - p.pad + s;
        if (wi >= 0 && wi < p.W) { ++cols_inside; continue; }
        for (int r = 0; r < p.R; ++r) {
          const int hi = ho * STRIDE - p.pad + r;
          if (hi >= 0 && hi < p.H) wrong += pop[(int64_t)(r * S + s) * p.Kp + k];
        }
      }
    }
    const int32_t x1 = p.C * rows_inside * cols_inside - 2 * (int32_t)(acc[j] - wrong);
    const int64_t pixel = ((int64_t)n * p.Ho + ho) * p.Wo + wo;
    if (p.out_x1 != nullptr && k < p.K) p.out_x1[pixel * p.K + k] = x1;
    if (p.out_x4 != nullptr) {
      const float v = (float)x1;
      const bool A = v < xi, B = gamma > 0.f, Cq = v == xi;
      const bool bit = k < p.K && ((A != B) || Cq);
      const unsigned long long mask = __ballot(bit);
      if (lane == 2 * j || lane == 2 * j + 1) mine = mask;
    }
  }
  if (p.out_x4 != nullptr) {
    // lanes 2j and 2j+1 hold the mask of pixel j: its low and high word
    const int j = lane >> 1, half = lane & 1;
    const int word = kb * 2 + half;
    if (j < TM && wo0 + j < p.Wo && word < p.Kw) {
      const int64_t pixel = ((int64_t)n * p.Ho + ho) * p.Wo + wo0 + j;
      p.out_x4[pixel * p.Kw + word] = (uint32_t)(half ? mine >> 32 : mine);
    }
  }
}

template <int S, int STRIDE, int QC, int TM>
void launch_conv(const ConvArgs& a, uint32_t blocks, hipStream_t stream) {
  rtc::prof_begin(kProfileKind, stream);
  hipLaunchKernelGGL((bconv_kernel<S, STRIDE, QC, TM>), dim3(blocks), dim3(64), 0, stream, a);
  rtc::prof_end(stream);
}

template <int S, int STRIDE, int QC>
void launch_conv_tm(const ConvArgs& a, int tm, uint32_t blocks, hipStream_t stream) {
  if (tm == 7) launch_conv<S, STRIDE, QC, 7>(a, blocks, stream);
  else launch_conv<S, STRIDE, QC, 8>(a, blocks, stream);
}

template <int S, int STRIDE>
void launch_conv_qc(const ConvArgs& a, int qc, int tm, uint32_t blocks, hipStream_t stream) {
  if (qc == 4) launch_conv_tm<S, STRIDE, 4>(a, tm, blocks, stream);
  else if (qc == 2) launch_conv_tm<S, STRIDE, 2>(a, tm, blocks, stream);
  else launch_conv_tm<S, STRIDE, 1>(a, tm, blocks, stream);
}

template <int S>
void launch_conv_stride(const ConvArgs& a, int stride, int qc, int tm, uint32_t blocks, hipStream_t stream) {
  if (stride == 1) launch_conv_qc<S, 1>(a, qc, tm, blocks, stream);
  else launch_conv_qc<S, 2>(a, qc, tm, blocks, stream);
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

constexpr int64_t kMaxDim = 1 << 20;

}  // namespace
}  // namespace bnn

extern "C" {

int bnn_pack_channels(const void* x, bnn_value_type type, uint32_t* words, int64_t rows, int64_t C,
                      void* hip_stream) {
  using namespace bnn;
  if (x == nullptr || words == nullptr) return BNN_ERR_NULL;
  if (type != BNN_VALUE_INT8 && type != BNN_VALUE_FLOAT) return BNN_ERR_DTYPE;
  if (rows < 1 || C < 1 || C > kMaxDim) return BNN_ERR_SHAPE;
  if (!aligned(words, 4) || (type == BNN_VALUE_FLOAT && !aligned(x, 4))) return BNN_ERR_ALIGN;
  const int64_t cblocks = (C + 63) / 64, Cw = (C + 31) / 32;
  if (rows * cblocks > 0x7fffffffLL) return BNN_ERR_SHAPE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const dim3 grid((uint32_t)(rows * cblocks));
  if (type == BNN_VALUE_INT8)
    hipLaunchKernelGGL(pack_channels_kernel<int8_t>, grid, dim3(64), 0, stream, static_cast<const int8_t*>(x), words,
                       rows, (int)C, (int)Cw, (int)cblocks);
  else
    hipLaunchKernelGGL(pack_channels_kernel<float>, grid, dim3(64), 0, stream, static_cast<const float*>(x), words,
                       rows, (int)C, (int)Cw, (int)cblocks);
  return hip_status();
}

size_t bnn_weight_words(int64_t K, int64_t R, int64_t S, int64_t C) {
  using namespace bnn;
  if (K < 1 || R < 1 || S < 1 || C < 1 || K > kMaxDim || C > kMaxDim || R > 64 || S > 64) return 0;
  const int64_t Kp = (K + 63) / 64 * 64, Cw = (C + 31) / 32;
  return (size_t)(R * S * Cw * Kp + R * S * Kp);
}

int bnn_pack_weights(const int8_t* w, uint32_t* packed, int64_t K, int64_t R, int64_t S, int64_t C,
                     void* hip_stream) {
  using namespace bnn;
  if (w == nullptr || packed == nullptr) return BNN_ERR_NULL;
  const size_t words = bnn_weight_words(K, R, S, C);
  if (words == 0 || words > 0x7fffffffULL) return BNN_ERR_SHAPE;
  if (!aligned(packed, 4)) return BNN_ERR_ALIGN;
  const int64_t Kp = (K + 63) / 64 * 64, Cw = (C + 31) / 32, taps = R * S;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(pack_weights_kernel, dim3((uint32_t)((taps * Cw * Kp + 255) / 256)), dim3(256), 0, stream, w,
                     packed, (int)K, (int)taps, (int)C, (int)Cw, (int)Kp);
  hipLaunchKernelGGL(weight_popcount_kernel, dim3((uint32_t)((taps * Kp + 255) / 256)), dim3(256), 0, stream, packed,
                     (int)taps, (int)Cw, (int)Kp);
  return hip_status();
}

int bnn_binary_conv2d(const uint32_t* x, const uint32_t* packed, const float* xi, const float* gamma,
                      int32_t* out_x1, uint32_t* out_x4, int64_t N, int64_t H, int64_t W, int64_t C,
                      int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad, void* hip_stream) {
  using namespace bnn;
  if (x == nullptr || packed == nullptr || (out_x1 == nullptr && out_x4 == nullptr)) return BNN_ERR_NULL;
  if (out_x4 != nullptr && (xi == nullptr || gamma == nullptr)) return BNN_ERR_NULL;
  if (N < 1 || H < 1 || W < 1 || C < 1 || K < 1 || R < 1 || S < 1 || stride < 1 || pad < 0) return BNN_ERR_SHAPE;
  if (H > kMaxDim || W > kMaxDim || C > kMaxDim || K > kMaxDim || N > kMaxDim || R > 64 || pad > 64) return BNN_ERR_SHAPE;
  if (S != 1 && S != 3 && S != 5) return BNN_ERR_UNSUPPORTED;
  if (stride != 1 && stride != 2) return BNN_ERR_UNSUPPORTED;
  if (H + 2 * pad < R || W + 2 * pad < S) return BNN_ERR_SHAPE;
  if (!aligned(x, 4) || !aligned(packed, 4) || !aligned(xi, 4) || !aligned(gamma, 4) || !aligned(out_x1, 4) ||
      !aligned(out_x4, 4))
    return BNN_ERR_ALIGN;
  const int64_t Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - S) / stride + 1;
  const int64_t Cw = (C + 31) / 32, Kp = (K + 63) / 64 * 64, Kw = (K + 31) / 32;
  // every index the kernel forms in 32 bits, and the popcount accumulator itself
  if (R * S * C > 0x3fffffffLL || bnn_weight_words(K, R, S, C) > 0x7fffffffULL) return BNN_ERR_SHAPE;
  // pixels per wave: the one of 7 / 8 that wastes fewer slots of an output row
  const int tm = ((Wo + 6) / 7 * 7 < (Wo + 7) / 8 * 8) ? 7 : 8;
  const int64_t wtiles = (Wo + tm - 1) / tm, kblocks = Kp / 64;
  const int64_t blocks = N * Ho * wtiles * kblocks;
  if (blocks > 0x7fffffffLL) return BNN_ERR_SHAPE;
  const int qc = Cw % 4 == 0 ? 4 : Cw % 2 == 0 ? 2 : 1;
  ConvArgs a;
  a.x = x; a.w = packed; a.xi = xi; a.gamma = gamma; a.out_x1 = out_x1; a.out_x4 = out_x4;
  a.H = (int32_t)H; a.W = (int32_t)W; a.C = (int32_t)C; a.Cw = (int32_t)Cw; a.K = (int32_t)K; a.Kp = (int32_t)Kp;
  a.Kw = (int32_t)Kw; a.R = (int32_t)R; a.pad = (int32_t)pad; a.Ho = (int32_t)Ho; a.Wo = (int32_t)Wo;
  a.kblocks = (int32_t)kblocks; a.wtiles = (int32_t)wtiles;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (S == 1) launch_conv_stride<1>(a, (int)stride, qc, tm, (uint32_t)blocks, stream);
  else if (S == 3) launch_conv_stride<3>(a, (int)stride, qc, tm, (uint32_t)blocks, stream);
  else launch_conv_stride<5>(a, (int)stride, qc, tm, (uint32_t)blocks, stream);
  return hip_status();
}

const char* bnn_strerror(int status) {
  switch (status) {
    case BNN_OK: return "ok";
    case BNN_ERR_NULL: return "required pointer is NULL";
    case BNN_ERR_SHAPE: return "invalid or too large shape";
    case BNN_ERR_DTYPE: return "unknown value type";
    case BNN_ERR_ALIGN: return "misaligned pointer";
    case BNN_ERR_UNSUPPORTED: return "filter width must be 1, 3 or 5 and stride 1 or 2";
    case BNN_ERR_HIP: return "HIP runtime error while enqueueing";
    default: return "unknown status";
  }
}

}  // extern "C"
