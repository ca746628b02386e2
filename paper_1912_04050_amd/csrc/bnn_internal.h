// Declarations shared by the translation units of the binary convolution layer.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "bnn.h"

namespace bnn {

// Thresholds of the integrated layer in the integer domain.  For an integer x1 (exact in fp32
// while |x1| <= 2^24, which the entry point guarantees) and v = (float)x1:
//   gamma > 0:  (A xor B) or C = not (v < xi) = not (x1 < ceil(xi))
//   otherwise:  (A xor B) or C = (v <= xi)    = x1 < floor(xi) + 1
// so the decision is `(x1 < T) xor (gamma > 0)` with T = ceil(xi) resp. floor(xi) + 1, clamped to
// +-2^30 (infinite thresholds) and -2^30 for a NaN (every comparison with it is false).
__device__ __forceinline__ int32_t integer_threshold(float xi, bool positive) {
  if (xi != xi) return -(1 << 30);
  const float t = positive ? ceilf(xi) : floorf(xi) + 1.0f;
  return (int32_t)fminf(fmaxf(t, -1073741824.0f), 1073741824.0f);
}

// ---- matrix-core path (bnn_mfma.hip) ----------------------------------------------------------
// Layers with 3 x 3 filters, stride 1, padding 1, C a multiple of 32 (at least 128) and K a
// multiple of 64 can run on the matrix cores: +1 / -1 as int8, v_mfma_i32_32x32x32_i8.  The filter
// bank then carries, behind the packed words, the filters once more as int8 in the order in which
// the instruction's B operand wants them.
struct MfmaArgs {
  const uint32_t* x;       // packed activations [N][H][W][Cw]
  const int8_t* wbytes;    // int8 filter fragments, see mfma_bank_bytes
  const float* xi;         // [K] or null
  const float* gamma;      // [K] or null
  int32_t* out_x1;         // [N][H][W][K] or null
  uint32_t* out_x4;        // [N][H][W][K / 32] or null
  int32_t N, H, W, Cw, K;
};

bool mfma_shape(int64_t K, int64_t R, int64_t S, int64_t C);            // the filter bank carries int8 fragments
size_t mfma_bank_bytes(int64_t K, int64_t R, int64_t S, int64_t C);      // 0 when !mfma_shape
bool mfma_slots_fit(int64_t H, int64_t W);                               // the staged pixel range fits the kernel
void launch_pack_weights_mfma(const int8_t* w, int8_t* bank, int64_t K, int64_t C, hipStream_t stream);
// false when the shape does not fit the kernel (the caller then takes another one)
// tiles: 3 or 4 pixel tiles of 32 per wave, 0 = the launcher chooses
bool launch_bconv_mfma(const MfmaArgs& a, hipStream_t stream, int tiles = 0);

}  // namespace bnn
