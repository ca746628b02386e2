/* Binary convolution layer of the paper on AMD MI355X (gfx950); exported by the same shared
 * library as rtc.h.
 *
 * Tensors hold +1 / -1 values, NHWC, packed along the channel dimension (the paper's channel
 * compression): channel c of a pixel is bit (c mod 32) of its word (c div 32), set for +1; a
 * pixel has ceil(C / 32) words and the unused high bits of its last word are 0.
 *
 * Conventions
 *   - All data pointers are DEVICE pointers; the caller owns every buffer, the library never
 *     allocates.  `hip_stream` is a hipStream_t passed as void*; calls only enqueue work.
 *   - Return value: BNN_OK or a negative bnn_status; on a negative status nothing was launched.
 *   - Outputs must not alias inputs.
 */
#ifndef BNN_H
#define BNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BNN_OK = 0,
  BNN_ERR_NULL = -1,        /* a required pointer is NULL */
  BNN_ERR_SHAPE = -2,       /* a dimension < 1, an empty output, or sizes beyond the 32-bit grid / index range */
  BNN_ERR_DTYPE = -3,       /* unknown bnn_value_type */
  BNN_ERR_ALIGN = -4,       /* a pointer is not aligned to its element size */
  BNN_ERR_UNSUPPORTED = -5, /* kernel width S not in {1, 3, 5} or stride not in {1, 2} */
  BNN_ERR_HIP = -7          /* the HIP runtime reported an error while enqueueing */
} bnn_status;

typedef enum { BNN_VALUE_INT8 = 0, BNN_VALUE_FLOAT = 1 } bnn_value_type;

/* Channel compression (the paper's data layout and bit packing sections): rows x C values ->
 * rows x ceil(C/32) words, bit set iff the value is > 0 (so +1 / -1 tensors pack to their
 * signs).  x: [rows][C] of int8 or float; words: [rows][ceil(C/32)]. */
int bnn_pack_channels(const void* x, bnn_value_type type, uint32_t* words, int64_t rows, int64_t C,
                      void* hip_stream);

/* Number of 32-bit words of the filter bank in the kernel's own layout (the paper prepares its
 * compressed model format offline; so does this): the packed filters, transposed so that the 64
 * filters of a wavefront sit side by side, followed by one popcount per (tap, filter) that the
 * kernel uses at image borders; for layers that the matrix cores can take (3 x 3 filters, C a
 * multiple of 32 and at least 128, K a multiple of 64) the filters follow once more as int8, in
 * the order of that instruction's operand.  0 on invalid sizes. */
size_t bnn_weight_words(int64_t K, int64_t R, int64_t S, int64_t C);

/* w: [K][R][S][C] int8 of +1 / -1  ->  packed: bnn_weight_words(K, R, S, C) words. */
int bnn_pack_weights(const int8_t* w, uint32_t* packed, int64_t K, int64_t R, int64_t S, int64_t C,
                     void* hip_stream);

/* Binary convolution (the paper's binary convolution operation, A.B = Len - 2 popcount(xor))
 * with the integrated batch normalisation + binarisation + packing (layer integration, workload
 * optimisation and branch-free selection sections).
 *   x1[n][ho][wo][k] = sum over taps (r, s) inside the image and channels c of x * w
 *                      (zero padding `pad` on every side: taps outside add nothing),
 *                      Ho = (H + 2 pad - R) / stride + 1, Wo likewise
 *   x4 = (A xor B) or C,  A = x1 < xi[k], B = gamma[k] > 0, C = x1 = xi[k]   (fp32 comparison;
 *        gamma[k] = 0 is outside the paper's domain and behaves like gamma < 0)
 * x:       packed activations [N][H][W][ceil(C/32)]
 * packed:  from bnn_pack_weights
 * out_x1:  optional int32 [N][Ho][Wo][K]
 * out_x4:  optional packed [N][Ho][Wo][ceil(K/32)] (needs xi and gamma, float [K])
 * At least one output must be given.  S must be 1, 3 or 5 and stride 1 or 2 (R is free). */
int bnn_binary_conv2d(const uint32_t* x, const uint32_t* packed, const float* xi, const float* gamma,
                      int32_t* out_x1, uint32_t* out_x4, int64_t N, int64_t H, int64_t W, int64_t C,
                      int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad, void* hip_stream);

/* Planner knobs (results do not depend on them; process-wide, not thread-safe): output pixels
 * per wavefront (7, 8 or 13; 13 only where stride is 1; tiles of 26 were measured slower) and blocks of 64
 * filters per wavefront
 * (1 or 2; 2 only for pixels of a multiple of 4 words and an even number of blocks).
 * 0 = choose automatically.  A value that does not apply to a shape is ignored for that shape. */
int bnn_set_planner(int tile_pixels, int filter_blocks);

/* Matrix-core path for 3 x 3, stride 1, pad 1 layers with C a multiple of 32 (>= 128) and K a
 * multiple of 64 (results do not depend on it; process-wide, not thread-safe): 0 = where the
 * planner expects it to be faster, 1 = wherever the shape allows, -1 = never; 3 or 4 = as 1, with
 * that many tiles of 32 pixels per wave instead of the planner's choice between the two (tests). */
int bnn_set_matrix_path(int mode);

/* 1 if bnn_binary_conv2d would run this layer on the matrix cores under the current setting of
 * bnn_set_matrix_path (given 16-byte aligned filter bank), else 0 (also for invalid sizes).  For
 * reports: which kernel a measured time belongs to. */
int bnn_matrix_path_applies(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                            int64_t stride, int64_t pad);

/* Static description of a status code. */
const char* bnn_strerror(int status);

#ifdef __cplusplus
}
#endif

#endif /* BNN_H */
