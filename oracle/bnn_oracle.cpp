// CPU oracle for the binary convolution layer of the paper (binary convolution operation,
// channel compression, layer integration).
//
// TEST INFRASTRUCTURE ONLY.  Slow, literal loops over the definitions; shares no code with the
// HIP path and must never be called from the product path.
//
// Values are +1 / -1 (int8).  Tensors are NHWC, filters [K][R][S][C].
//
//   binary convolution        x1[n][ho][wo][k] = sum over the taps (r, s) that fall inside the
//                             image and all channels c of x[n][hi][wi][c] * w[k][r][s][c]
//                             (the dot product that the paper's xor / popcount identity
//                             A.B = Len - 2 popcount(xor(a, b)) evaluates; taps in the zero
//                             padding contribute nothing)
//   layer integration         x4 = 1 if (x1 >= xi and gamma > 0) or (x1 <= xi and gamma < 0),
//                             else 0: the four cases of the integrated convolution + batch
//                             normalisation + binarisation; xi and the comparison are fp32
//   batch-norm chain          x2 = x1 + b, x3 = gamma (x2 - mu) / sigma + beta, x4 = [x3 >= 0]
//                             (unfused reference in fp64, used by the pins of xi only)
//   channel packing           bit (c mod 32) of word (c div 32) is set iff channel c is +1
//                             (resp. x4 = 1); unused high bits of the last word are 0
//   packed dot product        Len - 2 popcount(xor) over packed words
//   bit-plane input layer     s = sum_{i=1..8} 2^(i-1) <I_i . W>, I_i the i-th bit-plane of an
//                             8-bit input read as +1 (bit set) / -1 (bit clear)
//
// Readings where the paper is silent: zero padding (out-of-image taps add nothing), bit order
// of the packing (least significant bit first), threshold comparison in fp32, gamma = 0 is
// outside the domain (reported as an error), bit-planes in the same +1 / -1 encoding as every
// other binary tensor.
//
// Pins (tests/test_bnn_oracle_pins.py, all CPU): torch.nn.functional.conv2d on the same +1 / -1
// tensors in float64 (exact), the xor / popcount identity against the plain dot product, the
// boolean form (A xor B) or C against the four cases over the whole truth table, the unfused
// batch-norm chain against the threshold form, a hand-packed bit pattern.
#include <cstdint>
#include <cstddef>

namespace {

inline int64_t out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad) { return (in + 2 * pad - k) / stride + 1; }

}  // namespace

extern "C" {

int oracle_bnn_conv2d(const int8_t* x, const int8_t* w, int32_t* out, int64_t N, int64_t H, int64_t W, int64_t C,
                      int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad) {
  if (N < 1 || H < 1 || W < 1 || C < 1 || K < 1 || R < 1 || S < 1 || stride < 1 || pad < 0) return -2;
  const int64_t Ho = out_dim(H, R, stride, pad), Wo = out_dim(W, S, stride, pad);
  if (Ho < 1 || Wo < 1) return -2;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t ho = 0; ho < Ho; ++ho)
      for (int64_t wo = 0; wo < Wo; ++wo)
        for (int64_t k = 0; k < K; ++k) {
          int32_t sum = 0;
          for (int64_t r = 0; r < R; ++r)
            for (int64_t s = 0; s < S; ++s) {
              const int64_t hi = ho * stride - pad + r, wi = wo * stride - pad + s;
              if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
              const int8_t* xp = x + ((n * H + hi) * W + wi) * C;
              const int8_t* wp = w + ((k * R + r) * S + s) * C;
              for (int64_t c = 0; c < C; ++c) sum += (int32_t)xp[c] * (int32_t)wp[c];
            }
          out[((n * Ho + ho) * Wo + wo) * K + k] = sum;
        }
  return 0;
}

// s = sum_i 2^(i-1) <I_i . W> for an 8-bit input x (uint8, NHWC)
int oracle_bnn_bitplane_conv2d(const uint8_t* x, const int8_t* w, int32_t* out, int64_t N, int64_t H, int64_t W,
                               int64_t C, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad) {
  if (N < 1 || H < 1 || W < 1 || C < 1 || K < 1 || R < 1 || S < 1 || stride < 1 || pad < 0) return -2;
  const int64_t Ho = out_dim(H, R, stride, pad), Wo = out_dim(W, S, stride, pad);
  if (Ho < 1 || Wo < 1) return -2;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t ho = 0; ho < Ho; ++ho)
      for (int64_t wo = 0; wo < Wo; ++wo)
        for (int64_t k = 0; k < K; ++k) {
          int32_t total = 0;
          for (int plane = 1; plane <= 8; ++plane) {
            int32_t conv = 0;   // <I_plane . W>
            for (int64_t r = 0; r < R; ++r)
              for (int64_t s = 0; s < S; ++s) {
                const int64_t hi = ho * stride - pad + r, wi = wo * stride - pad + s;
                if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                const uint8_t* xp = x + ((n * H + hi) * W + wi) * C;
                const int8_t* wp = w + ((k * R + r) * S + s) * C;
                for (int64_t c = 0; c < C; ++c) conv += (((xp[c] >> (plane - 1)) & 1) ? 1 : -1) * (int32_t)wp[c];
              }
            total += (1 << (plane - 1)) * conv;
          }
          out[((n * Ho + ho) * Wo + wo) * K + k] = total;
        }
  return 0;
}

// the four cases of the integrated layer; rows = output pixels, K filters
int oracle_bnn_binarize(const int32_t* x1, const float* xi, const float* gamma, uint8_t* x4, int64_t rows, int64_t K) {
  for (int64_t k = 0; k < K; ++k)
    if (!(gamma[k] > 0.0f) && !(gamma[k] < 0.0f)) return -4;
  for (int64_t m = 0; m < rows; ++m)
    for (int64_t k = 0; k < K; ++k) {
      const float v = (float)x1[m * K + k];
      uint8_t bit;
      if (gamma[k] > 0.0f) bit = v >= xi[k] ? 1 : 0;
      else bit = v <= xi[k] ? 1 : 0;
      x4[m * K + k] = bit;
    }
  return 0;
}

// unfused chain in fp64: x4 = [gamma (x1 + b - mu) / sigma + beta >= 0]
int oracle_bnn_batchnorm_sign(const int32_t* x1, const double* b, const double* mu, const double* sigma,
                              const double* gamma, const double* beta, uint8_t* x4, int64_t rows, int64_t K) {
  for (int64_t m = 0; m < rows; ++m)
    for (int64_t k = 0; k < K; ++k) {
      const double x2 = (double)x1[m * K + k] + b[k];
      const double x3 = gamma[k] * ((x2 - mu[k]) / sigma[k]) + beta[k];
      x4[m * K + k] = x3 >= 0.0 ? 1 : 0;
    }
  return 0;
}

// bits: [rows][C] with 1 for +1 (or x4 = 1), anything else for -1 (or 0); words: [rows][ceil(C/32)]
int oracle_bnn_pack(const int8_t* bits, uint32_t* words, int64_t rows, int64_t C) {
  const int64_t Cw = (C + 31) / 32;
  for (int64_t m = 0; m < rows; ++m)
    for (int64_t j = 0; j < Cw; ++j) {
      uint32_t word = 0;
      for (int64_t i = 0; i < 32; ++i) {
        const int64_t c = j * 32 + i;
        if (c < C && bits[m * C + c] == 1) word |= (uint32_t)1 << i;
      }
      words[m * Cw + j] = word;
    }
  return 0;
}

// A.B = Len - 2 popcount(xor(a, b)) for vectors of `len` elements packed as above
int64_t oracle_bnn_dot_packed(const uint32_t* a, const uint32_t* b, int64_t len) {
  int64_t differing = 0;
  for (int64_t j = 0; j < (len + 31) / 32; ++j) {
    uint32_t v = a[j] ^ b[j];
    while (v) { differing += v & 1u; v >>= 1; }
  }
  return len - 2 * differing;
}

}  // extern "C"
