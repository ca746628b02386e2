// Binary convolution layer for gfx950: channel packing, filter-bank preparation and the
// xor / popcount convolution with the integrated batch-norm threshold, binarisation and output
// packing (the paper's binary convolution operation, channel compression, layer integration,
// workload optimisation and branch-free selection sections).
//
// Mapping.  The 64 lanes of a wave are 64 consecutive filters k; the wave owns TM consecutive
// output pixels of one output row.  An activation word is then the same for all lanes and a
// lane's filter word its own, and per (pixel, word) the kernels issue v_xor_b32 + v_bcnt_u32_b32
// (popcount with accumulate): 2 VALU instructions per 32 binary multiply-accumulates per lane,
// nothing else in the inner loop.  The TM pixels share one strip of (TM-1) stride + S input
// pixels per filter row.  The paper's "one thread computes 8 filters and packs a byte" becomes
// "one wavefront computes 64 filters and a ballot packs two words": the 64 binarised results of a
// pixel are the 64 bits of the wave's compare mask.
//
// Three kernels differ in how the strip reaches the lanes:
//   bconv_resident_kernel (+ _half)  pixels of 1, 2 or 4 words: filters live in registers, the
//                                    strip is fetched one tile ahead by a coalesced vector load
//                                    and broadcast through a wave-private LDS line
//   bconv_lds_kernel                 pixels of a multiple of 4 words: 4 waves share a strip staged
//                                    once in LDS, filter words stream from the transposed bank
//   bconv_kernel                     everything else: the strip sits in scalar registers and is
//                                    the scalar source of v_xor_b32
//
// Image borders: a filter row outside the image is skipped (it only lowers Len, i.e. the tile's
// threshold); a strip pixel left or right of the image is read as an all-zero word, and what the
// zero word wrongly contributed, popcount(w[k][r][s][:]), is taken off again in the epilogue
// from the per-(tap, filter) table that bnn_pack_weights appends to the filter bank.
#include <hip/hip_runtime.h>

#include "bnn.h"
#include "bnn_internal.h"
#include "rtc_internal.h"

namespace bnn {
namespace {

constexpr int kProfileKind = 32;   // rtc_profile_read() kind of the convolution kernel

inline int hip_status() { return rtc::hip_ok() == RTC_OK ? BNN_OK : BNN_ERR_HIP; }   // this thread's own launches only

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
  int32_t N, H, W, C, Cw, K, Kp, Kw, R, pad, Ho, Wo, kblocks, wtiles;
  int32_t tiles_per_wave, waves_per_image;   // resident-filter kernel only
};

// acc += popcount(v) as the one instruction v_bcnt_u32_b32 (popcount with accumulate).  Written
// as inline assembly so that the compiler keeps the accumulation a chain: left to itself it may
// re-associate the sum into separate popcounts and three-operand adds, which costs registers
// (and with them occupancy) for nothing.
__device__ __forceinline__ void popcount_accumulate(uint32_t& acc, uint32_t v) {
  asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(v));
}

// v with lane LANE replaced by the wave-uniform value s (v_writelane_b32: one VALU instruction).
template <int LANE>
__device__ __forceinline__ uint32_t write_lane(uint32_t v, uint32_t s) {
  asm("v_writelane_b32 %0, %1, %2" : "+v"(v) : "s"(s), "n"(LANE));
  return v;
}

// the same for a lane index that is a constant only after loop unrolling (0..51)
__device__ __forceinline__ uint32_t write_lane_of(uint32_t v, uint32_t s, int lane) {
  switch (lane) {
#define BNN_LANE(L) case L: return write_lane<L>(v, s);
    BNN_LANE(0) BNN_LANE(1) BNN_LANE(2) BNN_LANE(3) BNN_LANE(4) BNN_LANE(5) BNN_LANE(6) BNN_LANE(7)
    BNN_LANE(8) BNN_LANE(9) BNN_LANE(10) BNN_LANE(11) BNN_LANE(12) BNN_LANE(13) BNN_LANE(14) BNN_LANE(15)
    BNN_LANE(16) BNN_LANE(17) BNN_LANE(18) BNN_LANE(19) BNN_LANE(20) BNN_LANE(21) BNN_LANE(22) BNN_LANE(23)
    BNN_LANE(24) BNN_LANE(25) BNN_LANE(26) BNN_LANE(27) BNN_LANE(28) BNN_LANE(29) BNN_LANE(30) BNN_LANE(31)
    BNN_LANE(32) BNN_LANE(33) BNN_LANE(34) BNN_LANE(35) BNN_LANE(36) BNN_LANE(37) BNN_LANE(38) BNN_LANE(39)
    BNN_LANE(40) BNN_LANE(41) BNN_LANE(42) BNN_LANE(43) BNN_LANE(44) BNN_LANE(45) BNN_LANE(46) BNN_LANE(47)
    BNN_LANE(48) BNN_LANE(49) BNN_LANE(50) BNN_LANE(51)
#undef BNN_LANE
    default: return v;
  }
}

// Per-lane constants of the integrated layer for the 64 filters of one block.
struct Decision {
  int32_t T;                       // x1 < T decides (see integer_threshold)
  unsigned long long posmask;      // lanes with gamma > 0
  unsigned long long okmask;       // lanes whose filter exists
  bool lane_ok;
};

__device__ __forceinline__ Decision make_decision(const ConvArgs& p, int k, int S) {
  Decision d;
  const bool fused = p.out_x4 != nullptr;
  d.lane_ok = k < p.K;
  const bool positive = fused && d.lane_ok && p.gamma[k] > 0.f;
  d.T = fused && d.lane_ok ? integer_threshold(p.xi[k], positive) : 0;
  d.posmask = __ballot(positive);
  d.okmask = __ballot(d.lane_ok);
  return d;
}

// Epilogue of one tile of TM output pixels and one block of 64 filters: x1 = Len - 2 popcount
// with Len = C x (taps inside the image) and the popcounts that zeroed border pixels wrongly
// added taken off; optional store of x1; the integrated layer's bit, its 64-lane compare mask
// being the two packed output words of the pixel.  `interior`: every tap of every pixel of the
// tile lies inside the image.
template <int S, int STRIDE, int TM>
__device__ __forceinline__ void finish_tile(const ConvArgs& p, const Decision& d, const uint32_t (&acc)[TM], int n,
                                            int ho, int wo0, int kb, int k, int rows_inside, bool interior) {
  const int lane = threadIdx.x & 63;
  const uint32_t* __restrict__ pop = p.w + (int64_t)p.R * S * p.Cw * p.Kp;
  const int64_t pixel0 = ((int64_t)n * p.Ho + ho) * p.Wo + wo0;
  const int hi0 = ho * STRIDE - p.pad;
  uint32_t mine = 0;
  // Pixels all of whose columns lie inside the image need no correction (filter rows outside
  // were skipped, not zeroed): x1 = Len - 2 popcount with Len = C S rows_inside, so
  // x1 < T  <=>  popcount > U = floor((Len - T) / 2): one integer compare.  Only the one or two
  // pixels of a border tile whose columns reach outside take the long way.
  (void)interior;
  const int32_t U = (p.C * rows_inside * S - d.T) >> 1;       // arithmetic shift = floor for either sign
  constexpr int PS = (TM - 1) * STRIDE + S;
  const int wi0 = wo0 * STRIDE - p.pad;
  const bool tile_cols_inside = wi0 >= 0 && wi0 + PS <= p.W;  // wave-uniform
  if (tile_cols_inside && p.out_x1 == nullptr) {
    // the common case, straight-line (pixels beyond the end of the output row are computed too
    // and never stored)
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      const unsigned long long less = __ballot((int32_t)acc[j] > U);
      const unsigned long long mask = (less ^ d.posmask) & d.okmask;
      mine = write_lane_of(mine, (uint32_t)mask, 2 * j);
      mine = write_lane_of(mine, (uint32_t)(mask >> 32), 2 * j + 1);
    }
  } else
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int wi_first = (wo0 + j) * STRIDE - p.pad;
    const bool cols_inside_all = wi_first >= 0 && wi_first + S <= p.W;    // wave-uniform
    unsigned long long less;                     // lanes with x1 < T
    if (cols_inside_all && p.out_x1 == nullptr) {
      less = __ballot((int32_t)acc[j] > U);
    } else if (wo0 + j < p.Wo) {
      int cols_inside = 0;
      uint32_t wrong = 0;
#pragma unroll
      for (int s = 0; s < S; ++s) {
        const int wi = wi_first + s;
        if (wi >= 0 && wi < p.W) { ++cols_inside; continue; }
        for (int r = 0; r < p.R; ++r)
          if (hi0 + r >= 0 && hi0 + r < p.H) wrong += pop[(uint32_t)(r * S + s) * (uint32_t)p.Kp + k];
      }
      const int32_t x1 = p.C * rows_inside * cols_inside - 2 * (int32_t)(acc[j] - wrong);
      if (p.out_x1 != nullptr && d.lane_ok) p.out_x1[(pixel0 + j) * p.K + k] = x1;
      less = __ballot(x1 < d.T);
    } else {
      less = 0;                                  // beyond the end of the output row: never stored
    }
    const unsigned long long mask = (less ^ d.posmask) & d.okmask;
    mine = write_lane_of(mine, (uint32_t)mask, 2 * j);
    mine = write_lane_of(mine, (uint32_t)(mask >> 32), 2 * j + 1);
  }
  if (p.out_x4 != nullptr) {
    // lanes 2j and 2j+1 hold the low and high word of pixel j
    const int j = lane >> 1, word = kb * 2 + (lane & 1);
    if (j < TM && wo0 + j < p.Wo && word < p.Kw) p.out_x4[(pixel0 + j) * p.Kw + word] = mine;
  }
}

// One row of the strip into scalar registers: QC words of each of the PS pixels from word c0 of
// the pixel on; pixels left or right of the image read as zero words.
template <int PS, int QC>
__device__ __forceinline__ void load_strip(uint32_t (&a)[PS][QC], const uint32_t* __restrict__ xrow, int wi0, int c0,
                                           int Cw, int W, bool cols_interior) {
  if (cols_interior) {
#pragma unroll
    for (int i = 0; i < PS; ++i) {
      const uint32_t* __restrict__ src = xrow + ((uint32_t)(wi0 + i) * (uint32_t)Cw + (uint32_t)c0);
#pragma unroll
      for (int q = 0; q < QC; ++q) a[i][q] = src[q];
    }
  } else {
#pragma unroll
    for (int i = 0; i < PS; ++i) {
      const int wi = wi0 + i;
      const bool in = wi >= 0 && wi < W;
      const uint32_t* __restrict__ src = xrow + ((uint32_t)(in ? wi : 0) * (uint32_t)Cw + (uint32_t)c0);
#pragma unroll
      for (int q = 0; q < QC; ++q) {
        const uint32_t v = src[q];               // unconditional (the address is clamped), zeroed afterwards
        a[i][q] = in ? v : 0u;
      }
    }
  }
}

// General kernel.  S = filter width, STRIDE, QC = words of a pixel per pass (divides Cw), TM =
// output pixels per wave, KB = blocks of 64 filters per wave (each scalar activation word then
// serves KB vector instructions pairs).
template <int S, int STRIDE, int QC, int TM, int KB>
__global__ __launch_bounds__(64) void bconv_kernel(
    const uint32_t* __restrict__ x, const uint32_t* __restrict__ w, const float* __restrict__ xi,
    const float* __restrict__ gamma, int32_t* __restrict__ out_x1, uint32_t* __restrict__ out_x4, const ConvArgs dims) {
  // the pointers travel as restrict-qualified kernel parameters (so that loads of the read-only
  // operands stay scalar loads even though the kernel also stores), the sizes in `dims`
  ConvArgs p = dims;
  p.x = x; p.w = w; p.xi = xi; p.gamma = gamma; p.out_x1 = out_x1; p.out_x4 = out_x4;
  constexpr int PS = (TM - 1) * STRIDE + S;      // input pixels of the strip
  const int lane = threadIdx.x;
  uint32_t b = blockIdx.x;
  // tiles fastest, filter blocks slowest: the waves in flight at any time share a few filter
  // blocks, whose words they then find in the vector caches
  const int wt = b % p.wtiles; b /= p.wtiles;
  const int ho = b % p.Ho; b /= p.Ho;
  const int n = b % p.N;
  const int kb0 = (b / p.N) * KB;
  const int wo0 = wt * TM;
  const int wi0 = wo0 * STRIDE - p.pad;
  const bool cols_interior = wi0 >= 0 && wi0 + PS <= p.W;    // wave-uniform
  const uint32_t wstep = (uint32_t)p.Kp;         // words between consecutive (tap, cw) rows of the filter bank

  uint32_t acc[KB][TM];
#pragma unroll
  for (int u = 0; u < KB; ++u)
#pragma unroll
    for (int j = 0; j < TM; ++j) acc[u][j] = 0;

  int rows_inside = 0;
  for (int r = 0; r < p.R; ++r) {
    const int hi = ho * STRIDE - p.pad + r;
    if (hi < 0 || hi >= p.H) continue;           // wave-uniform
    ++rows_inside;
    const uint32_t* __restrict__ xrow = p.x + ((int64_t)n * p.H + hi) * p.W * p.Cw;
    const uint32_t* __restrict__ wrow = p.w + (int64_t)r * S * p.Cw * p.Kp + kb0 * 64;
    for (int c0 = 0; c0 < p.Cw; c0 += QC) {
      uint32_t a[PS][QC];                        // wave-uniform: scalar registers
      load_strip<PS, QC>(a, xrow, wi0, c0, p.Cw, p.W, cols_interior);
#pragma unroll
      for (int s = 0; s < S; ++s) {
        const uint32_t* __restrict__ wtap = wrow + (uint32_t)(s * p.Cw + c0) * wstep;
        uint32_t wv[KB][QC];
#pragma unroll
        for (int u = 0; u < KB; ++u)
#pragma unroll
          for (int q = 0; q < QC; ++q) wv[u][q] = (wtap + (q * wstep + u * 64))[lane];
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
          for (int q = 0; q < QC; ++q)
#pragma unroll
            for (int u = 0; u < KB; ++u) popcount_accumulate(acc[u][j], a[j * STRIDE + s][q] ^ wv[u][q]);
      }
    }
  }

  const bool interior = cols_interior && rows_inside == p.R;
#pragma unroll
  for (int u = 0; u < KB; ++u) {
    const int k = (kb0 + u) * 64 + lane;
    const Decision d = make_decision(p, k, S);
    finish_tile<S, STRIDE, TM>(p, d, acc[u], n, ho, wo0, kb0 + u, k, rows_inside, interior);
  }
}

// Kernel for wide pixels (Cw a multiple of 4).  A workgroup of 4 waves owns one tile of TM
// output pixels and 4 KB blocks of 64 filters (one KB-group per wave).  The input strip of the
// tile -- every filter row inside the image, PS pixels, all Cw words -- is staged once in LDS
// with coalesced 16-byte loads (scalar loads would fetch a 64-byte line per pixel for 16 bytes of
// use and thrash the small scalar cache); every lane of a wave then reads the same LDS address
// (a broadcast, free of bank conflicts) and xors it with its own filter word.
template <int S, int STRIDE, int TM, int KB>
__global__ __launch_bounds__(256) void bconv_lds_kernel(
    const uint32_t* __restrict__ x, const uint32_t* __restrict__ w, const float* __restrict__ xi,
    const float* __restrict__ gamma, int32_t* __restrict__ out_x1, uint32_t* __restrict__ out_x4, const ConvArgs dims) {
  // the pointers travel as restrict-qualified kernel parameters (so that loads of the read-only
  // operands stay scalar loads even though the kernel also stores), the sizes in `dims`
  ConvArgs p = dims;
  p.x = x; p.w = w; p.xi = xi; p.gamma = gamma; p.out_x1 = out_x1; p.out_x4 = out_x4;
  extern __shared__ __align__(16) uint32_t strip[];          // [rows inside][PS][Cw]
  constexpr int PS = (TM - 1) * STRIDE + S;
  constexpr int QC = 4;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t b = blockIdx.x;
  const int wt = b % p.wtiles; b /= p.wtiles;
  const int ho = b % p.Ho; b /= p.Ho;
  const int n = b % p.N;
  const int kgroup = b / p.N;
  const int wo0 = wt * TM;
  const int wi0 = wo0 * STRIDE - p.pad;
  const int r_lo = max(0, p.pad - ho * STRIDE);
  const int r_hi = min(p.R, p.H + p.pad - ho * STRIDE);
  const int rows_inside = max(r_hi - r_lo, 0);
  const int cw4 = p.Cw / QC;

  // stage the strip: element e = (row rr, strip pixel i, group of 4 words c4), c4 fastest
  const int staged = rows_inside * PS * cw4;
  for (int e = tid; e < staged; e += 256) {
    const int c4 = e % cw4;
    const int i = (e / cw4) % PS;
    const int rr = e / (cw4 * PS);
    const int wi = wi0 + i, hi = ho * STRIDE - p.pad + r_lo + rr;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (wi >= 0 && wi < p.W)
      v = *reinterpret_cast<const u32x4*>(p.x + (((int64_t)n * p.H + hi) * p.W + wi) * p.Cw + c4 * QC);
    reinterpret_cast<u32x4*>(strip)[e] = v;
  }
  __syncthreads();

  const int kb0 = (kgroup * 4 + wave) * KB;
  if (kb0 >= p.kblocks) return;                  // whole wave, after the only barrier
  const uint32_t wstep = (uint32_t)p.Kp;
  uint32_t acc[KB][TM];
#pragma unroll
  for (int u = 0; u < KB; ++u)
#pragma unroll
    for (int j = 0; j < TM; ++j) acc[u][j] = 0;

  for (int rr = 0; rr < rows_inside; ++rr) {
    const uint32_t* __restrict__ wrow = p.w + (int64_t)(r_lo + rr) * S * p.Cw * p.Kp + kb0 * 64;
    const u32x4* __restrict__ srow = reinterpret_cast<const u32x4*>(strip) + rr * PS * cw4;
    for (int c4 = 0; c4 < cw4; ++c4) {
      u32x4 a[PS];                               // the same value in every lane
#pragma unroll
      for (int i = 0; i < PS; ++i) a[i] = srow[i * cw4 + c4];
#pragma unroll
      for (int s = 0; s < S; ++s) {
        const uint32_t* __restrict__ wtap = wrow + (uint32_t)(s * p.Cw + c4 * QC) * wstep;
        uint32_t wv[KB][QC];
#pragma unroll
        for (int u = 0; u < KB; ++u)
#pragma unroll
          for (int q = 0; q < QC; ++q) wv[u][q] = (wtap + (q * wstep + u * 64))[lane];
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
          for (int q = 0; q < QC; ++q)
#pragma unroll
            for (int u = 0; u < KB; ++u) popcount_accumulate(acc[u][j], a[j * STRIDE + s][q] ^ wv[u][q]);
      }
    }
  }

  const bool interior = wi0 >= 0 && wi0 + PS <= p.W && rows_inside == p.R;
#pragma unroll
  for (int u = 0; u < KB; ++u) {
    const int k = (kb0 + u) * 64 + lane;
    const Decision d = make_decision(p, k, S);
    finish_tile<S, STRIDE, TM>(p, d, acc[u], n, ho, wo0, kb0 + u, k, rows_inside, interior);
  }
}

// Filters small enough to live in registers (R * S * CW <= 36 words per lane): the wave loads
// its 64 filters once and then streams over `tiles_per_wave` consecutive (output row, strip)
// tiles of one image, which is how the paper uses a thread's private memory for layers of few
// channels.  A strip row is PS * CW <= 64 contiguous words: lane i fetches word i with one
// coalesced vector load, issued one tile ahead so that its latency hides behind the current
// tile's arithmetic; the row then passes through a wave-private LDS line, from which every lane
// reads the same 16 bytes at a time (a broadcast), so each lane holds the whole strip.
template <int R, int S, int STRIDE, int CW, int TM>
__global__ __launch_bounds__(64) void bconv_resident_kernel(
    const uint32_t* __restrict__ x, const uint32_t* __restrict__ w, const float* __restrict__ xi,
    const float* __restrict__ gamma, int32_t* __restrict__ out_x1, uint32_t* __restrict__ out_x4, const ConvArgs dims) {
  ConvArgs p = dims;
  p.x = x; p.w = w; p.xi = xi; p.gamma = gamma; p.out_x1 = out_x1; p.out_x4 = out_x4;
  constexpr int PS = (TM - 1) * STRIDE + S;
  constexpr int WORDS = PS * CW;                 // words of one strip row
  constexpr int QUADS = (WORDS + 3) / 4;
  if (WORDS > 64) return;                        // one lane per strip word: the host never launches such a shape
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  __shared__ __align__(16) uint32_t line[R][64];
  const int lane = threadIdx.x;
  uint32_t b = blockIdx.x;
  const int kb = b % p.kblocks; b /= p.kblocks;
  const int chunk = b % p.waves_per_image;
  const int n = b / p.waves_per_image;
  const int k = kb * 64 + lane;
  const uint32_t* __restrict__ ximg = p.x + (int64_t)n * p.H * p.W * CW;

  uint32_t wreg[R][S][CW];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
      for (int q = 0; q < CW; ++q) wreg[r][s][q] = (p.w + (uint32_t)((r * S + s) * CW + q) * (uint32_t)p.Kp)[k];
  const Decision d = make_decision(p, k, S);

  // lane i's word of each strip row of the tile (ho, wt); 0 outside the image.  Offsets inside an
  // image fit 32 bits (checked by the entry point).
  const int lane_pixel = lane / CW, lane_word = lane % CW;
  const uint32_t row_words = (uint32_t)p.W * CW;
  auto fetch = [&](uint32_t (&dst)[R], int ho, int wt) {
    const int wi = wt * TM * STRIDE - p.pad + lane_pixel;
    const bool col_ok = lane < WORDS && (uint32_t)wi < (uint32_t)p.W;
    const uint32_t col_off = (uint32_t)wi * CW + lane_word;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int hi = ho * STRIDE - p.pad + r;
      uint32_t v = 0;
      if (col_ok && (uint32_t)hi < (uint32_t)p.H) v = ximg[(uint32_t)hi * row_words + col_off];
      dst[r] = v;
    }
  };

  const int total_tiles = p.Ho * p.wtiles;
  const int t_begin = chunk * p.tiles_per_wave;
  const int t_end = min(t_begin + p.tiles_per_wave, total_tiles);
  if (t_begin >= t_end) return;
  int ho = t_begin / p.wtiles, wt = t_begin % p.wtiles;   // advanced incrementally below
  uint32_t cur[R], nxt[R];
  fetch(cur, ho, wt);
  for (int t = t_begin; t < t_end; ++t) {
    int ho_next = ho, wt_next = wt + 1;
    if (wt_next == p.wtiles) { wt_next = 0; ++ho_next; }
    if (t + 1 < t_end) fetch(nxt, ho_next, wt_next);

    const int wo0 = wt * TM;
    const int wi0 = wo0 * STRIDE - p.pad;
    const int hi0 = ho * STRIDE - p.pad;
#pragma unroll
    for (int r = 0; r < R; ++r) line[r][lane] = cur[r];
    __syncthreads();                             // one wave: orders the LDS writes before the broadcast reads

    uint32_t acc[TM];
#pragma unroll
    for (int j = 0; j < TM; ++j) acc[j] = 0;
    int rows_inside = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int hi = hi0 + r;
      if (hi < 0 || hi >= p.H) continue;         // wave-uniform
      ++rows_inside;
      u32x4 a[QUADS];                            // the same value in every lane
#pragma unroll
      for (int v = 0; v < QUADS; ++v) a[v] = reinterpret_cast<const u32x4*>(line[r])[v];
#pragma unroll
      for (int s = 0; s < S; ++s)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
          for (int q = 0; q < CW; ++q) {
            const int word = (j * STRIDE + s) * CW + q;
            acc[j] += __popc(a[word / 4][word % 4] ^ wreg[r][s][q]);   // the compiler's own schedule measured 5 % faster here
          }
    }
    __syncthreads();                             // reads done before the next tile's writes
    const bool interior = wi0 >= 0 && wi0 + PS <= p.W && rows_inside == R;
    finish_tile<S, STRIDE, TM>(p, d, acc, n, ho, wo0, kb, k, rows_inside, interior);
#pragma unroll
    for (int r = 0; r < R; ++r) cur[r] = nxt[r];
    ho = ho_next; wt = wt_next;
  }
}

// At most 32 filters: the two halves of the wave work on two different tiles with the same 32
// filters, which is possible because the strip reaches the lanes through LDS (each half reads its
// own 32 words of the line) and not through scalar registers.  The 64-bit compare mask of pixel
// j then holds tile A's packed word in its low half and tile B's in its high half.  No filter
// row is skipped (the halves may sit in different output rows): rows and columns outside the
// image are read as zero words and corrected alike.  Stride 1, WORDS = PS * CW <= 32.
// PAIR (one word per pixel of at most 16 channels, S = 3): the upper half of every activation and
// filter word is padding, zero in both, so the taps (r, 0) and (r, 1) share one xor + popcount:
// the strip is staged a second time with each word's right neighbour in its upper half, the
// filters pair their taps the same way, and a filter row costs two instruction pairs per pixel
// instead of three.
template <int R, int S, int CW, int TM, bool PAIR>
__global__ __launch_bounds__(64) void bconv_resident_half_kernel(
    const uint32_t* __restrict__ x, const uint32_t* __restrict__ w, const float* __restrict__ xi,
    const float* __restrict__ gamma, int32_t* __restrict__ out_x1, uint32_t* __restrict__ out_x4, const ConvArgs dims) {
  ConvArgs p = dims;
  p.x = x; p.w = w; p.xi = xi; p.gamma = gamma; p.out_x1 = out_x1; p.out_x4 = out_x4;
  constexpr int PS = TM - 1 + S;
  constexpr int WORDS = PS * CW;
  constexpr int QUADS = (WORDS + 3) / 4;
  if (WORDS > 32) return;                        // the host never launches such a shape
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  static_assert(!PAIR || (CW == 1 && S == 3), "pairing is for one half-filled word per pixel and three taps per row");
  __shared__ __align__(16) uint32_t line[R][64];
  __shared__ __align__(16) uint32_t linep[PAIR ? R : 1][64];   // word i | word i + 1 << 16
  const int lane = threadIdx.x, half = lane >> 5, l32 = lane & 31;
  const int chunk = blockIdx.x % p.waves_per_image;
  const int n = blockIdx.x / p.waves_per_image;
  const int k = l32;
  const uint32_t* __restrict__ ximg = p.x + (int64_t)n * p.H * p.W * CW;
  const uint32_t* __restrict__ pop = p.w + (int64_t)R * S * CW * p.Kp;

  uint32_t wreg[R][S][CW];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
      for (int q = 0; q < CW; ++q) wreg[r][s][q] = (p.w + (uint32_t)((r * S + s) * CW + q) * (uint32_t)p.Kp)[k];
  uint32_t wpair[R];                             // PAIR: taps (r, 0) and (r, 1) in one word
#pragma unroll
  for (int r = 0; r < R; ++r) wpair[r] = PAIR ? wreg[r][0][0] | (wreg[r][S > 1 ? 1 : 0][0] << 16) : 0u;
  const Decision d = make_decision(p, k, S);
  uint32_t popv[R][S];                           // popcount of each tap of this lane's filter (border corrections)
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int s = 0; s < S; ++s) popv[r][s] = pop[(uint32_t)(r * S + s) * (uint32_t)p.Kp + k];

  // this lane's word of each strip row of its half's tile; 0 outside the image or without a tile
  const int lane_pixel = l32 / CW, lane_word = l32 % CW;
  const uint32_t row_words = (uint32_t)p.W * CW;   // offsets inside an image fit 32 bits (checked by the entry point)
  auto fetch = [&](uint32_t (&dst)[R], int ho_l, int wt_l, bool tile_ok) {
    const int wi = wt_l * TM - p.pad + lane_pixel;
    const bool col_ok = tile_ok && l32 < WORDS && (uint32_t)wi < (uint32_t)p.W;
    const uint32_t col_off = (uint32_t)wi * CW + lane_word;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int hi = ho_l - p.pad + r;
      uint32_t v = 0;
      if (col_ok && (uint32_t)hi < (uint32_t)p.H) v = ximg[(uint32_t)hi * row_words + col_off];
      dst[r] = v;
    }
  };
  auto advance = [&](int& ho, int& wt) { if (++wt == p.wtiles) { wt = 0; ++ho; } };

  const int total_tiles = p.Ho * p.wtiles;
  const int t_begin = chunk * p.tiles_per_wave;
  const int t_end = min(t_begin + p.tiles_per_wave, total_tiles);
  if (t_begin >= t_end) return;
  int hoA = t_begin / p.wtiles, wtA = t_begin % p.wtiles;
  int hoB = hoA, wtB = wtA;
  advance(hoB, wtB);
  uint32_t cur[R], nxt[R];
  fetch(cur, half ? hoB : hoA, half ? wtB : wtA, half == 0 || t_begin + 1 < t_end);
  for (int t = t_begin; t < t_end; t += 2) {
    const bool has_b = t + 1 < t_end;            // wave-uniform
    int hoA2 = hoB, wtA2 = wtB;
    advance(hoA2, wtA2);
    int hoB2 = hoA2, wtB2 = wtA2;
    advance(hoB2, wtB2);
    if (t + 2 < t_end) fetch(nxt, half ? hoB2 : hoA2, half ? wtB2 : wtA2, half == 0 || t + 3 < t_end);

#pragma unroll
    for (int r = 0; r < R; ++r) {
      line[r][lane] = cur[r];
      // (the neighbour of a half's last lane belongs to the other tile: no pixel of a tile reads that far)
      if constexpr (PAIR) linep[r][lane] = cur[r] | ((uint32_t)__shfl_down((int)cur[r], 1) << 16);
    }
    __syncthreads();                             // one wave: orders the LDS writes before the reads
    uint32_t acc[TM];
#pragma unroll
    for (int j = 0; j < TM; ++j) acc[j] = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      u32x4 a[QUADS];                            // the same value in every lane of a half
#pragma unroll
      for (int v = 0; v < QUADS; ++v) a[v] = reinterpret_cast<const u32x4*>(&line[r][half * 32])[v];
      if constexpr (PAIR) {
        u32x4 ap[QUADS];
#pragma unroll
        for (int v = 0; v < QUADS; ++v) ap[v] = reinterpret_cast<const u32x4*>(&linep[r][half * 32])[v];
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          popcount_accumulate(acc[j], ap[j / 4][j % 4] ^ wpair[r]);
          popcount_accumulate(acc[j], a[(j + 2) / 4][(j + 2) % 4] ^ wreg[r][2][0]);
        }
      } else {
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
          for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int q = 0; q < CW; ++q) {
              const int word = (j + s) * CW + q;
              popcount_accumulate(acc[j], a[word / 4][word % 4] ^ wreg[r][s][q]);
            }
      }
    }
    __syncthreads();                             // reads done before the next pair's writes

    // Per lane (the halves sit on different tiles): filter rows outside the image were read as
    // zero words, which added popcount(w) of their taps; with those taken off,
    // x1 = C S rows_in - 2 (popcount - wrong_rows), so for pixels whose columns all lie inside
    // x1 < T  <=>  popcount > U = floor((C S rows_in + 2 wrong_rows - T) / 2): one compare.
    const int ho_l = half ? hoB : hoA, wo0_l = (half ? wtB : wtA) * TM;
    const bool tile_ok = half == 0 || has_b;
    const int64_t pixel0_l = ((int64_t)n * p.Ho + ho_l) * p.Wo + wo0_l;
    bool row_in[R];
    int rows_in = 0;
    uint32_t wrong_rows = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      row_in[r] = ho_l - p.pad + r >= 0 && ho_l - p.pad + r < p.H;
      rows_in += row_in[r] ? 1 : 0;
#pragma unroll
      for (int s = 0; s < S; ++s) wrong_rows += row_in[r] ? 0u : popv[r][s];
    }
    const int32_t U = (p.C * rows_in * S + 2 * (int32_t)wrong_rows - d.T) >> 1;
    uint32_t mine = 0;
    const int wi0A = wtA * TM - p.pad, wi0B = wtB * TM - p.pad;
    const bool tiles_cols_inside = wi0A >= 0 && wi0A + PS <= p.W && (!has_b || (wi0B >= 0 && wi0B + PS <= p.W));
    if (tiles_cols_inside && p.out_x1 == nullptr) {
      // the common case, straight-line
#pragma unroll
      for (int j = 0; j < TM; ++j) {
        const unsigned long long less = __ballot((int32_t)acc[j] > U);
        const unsigned long long mask = (less ^ d.posmask) & d.okmask;
        mine = write_lane_of(mine, (uint32_t)mask, 2 * j);
        mine = write_lane_of(mine, (uint32_t)(mask >> 32), 2 * j + 1);
      }
    } else
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      const int wiA = wtA * TM + j - p.pad, wiB = wtB * TM + j - p.pad;
      const bool cols_all = wiA >= 0 && wiA + S <= p.W && (!has_b || (wiB >= 0 && wiB + S <= p.W));   // wave-uniform
      unsigned long long less;                   // lanes with x1 < T
      if (cols_all && p.out_x1 == nullptr) {
        less = __ballot((int32_t)acc[j] > U);
      } else {
        const int wo = wo0_l + j;
        int cols_in = 0;
        uint32_t wrong = wrong_rows;
#pragma unroll
        for (int s = 0; s < S; ++s) {
          const int wi = wo - p.pad + s;
          const bool col_in = wi >= 0 && wi < p.W;
          cols_in += col_in ? 1 : 0;
#pragma unroll
          for (int r = 0; r < R; ++r) wrong += (!col_in && row_in[r]) ? popv[r][s] : 0u;
        }
        const int32_t x1 = p.C * rows_in * cols_in - 2 * (int32_t)(acc[j] - wrong);
        if (p.out_x1 != nullptr && d.lane_ok && tile_ok && wo < p.Wo) p.out_x1[(pixel0_l + j) * p.K + k] = x1;
        less = __ballot(x1 < d.T);
      }
      const unsigned long long mask = (less ^ d.posmask) & d.okmask;
      mine = write_lane_of(mine, (uint32_t)mask, 2 * j);
      mine = write_lane_of(mine, (uint32_t)(mask >> 32), 2 * j + 1);
    }
    if (p.out_x4 != nullptr && lane < 2 * TM) {
      // lane 2j holds tile A's word of pixel j, lane 2j+1 tile B's (Kw = 1)
      const int j = lane >> 1, which = lane & 1;
      const int ho_w = which ? hoB : hoA, wo_w = (which ? wtB : wtA) * TM + j;
      if ((which == 0 || has_b) && wo_w < p.Wo) p.out_x4[((int64_t)n * p.Ho + ho_w) * p.Wo + wo_w] = mine;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) cur[r] = nxt[r];
    hoA = hoA2; wtA = wtA2; hoB = hoB2; wtB = wtB2;
  }
}

// ---- launch selection -------------------------------------------------------------------------

template <int S, int STRIDE, int QC, int TM, int KB>
void launch_general(const ConvArgs& a, uint32_t blocks, hipStream_t stream) {
  rtc::prof_begin(kProfileKind, stream);
  RTC_LAUNCH((bconv_kernel<S, STRIDE, QC, TM, KB>), dim3(blocks), dim3(64), 0, stream, a.x, a.w, a.xi, a.gamma,
                     a.out_x1, a.out_x4, a);
  rtc::prof_end(stream);
}

// Instantiated scalar-strip variants (the fallback for pixels whose word count is not a multiple
// of 4, or whose strip does not fit LDS): tiles of 7 / 8 pixels, one block of filters.
template <int S>
bool launch_general_s(const ConvArgs& a, int stride, int qc, int tm, uint32_t blocks, hipStream_t stream) {
#define BNN_GENERAL(ST, QQ, TT)                                            \
  if (stride == ST && qc == QQ && tm == TT) {                              \
    launch_general<S, ST, QQ, TT, 1>(a, blocks, stream);                   \
    return true;                                                           \
  }
  BNN_GENERAL(1, 4, 7) BNN_GENERAL(1, 4, 8) BNN_GENERAL(1, 2, 7) BNN_GENERAL(1, 2, 8) BNN_GENERAL(1, 1, 7) BNN_GENERAL(1, 1, 8)
  BNN_GENERAL(2, 4, 7) BNN_GENERAL(2, 4, 8) BNN_GENERAL(2, 2, 7) BNN_GENERAL(2, 2, 8) BNN_GENERAL(2, 1, 7) BNN_GENERAL(2, 1, 8)
#undef BNN_GENERAL
  return false;
}

template <int S, int STRIDE, int TM, int KB>
void launch_lds_one(const ConvArgs& a, uint32_t blocks, size_t lds_bytes, hipStream_t stream) {
  rtc::prof_begin(kProfileKind, stream);
  RTC_LAUNCH((bconv_lds_kernel<S, STRIDE, TM, KB>), dim3(blocks), dim3(256), lds_bytes, stream, a.x, a.w, a.xi,
                     a.gamma, a.out_x1, a.out_x4, a);
  rtc::prof_end(stream);
}

template <int S>
bool launch_lds_s(const ConvArgs& a, int stride, int tm, int kb, uint32_t blocks, size_t lds_bytes, hipStream_t stream) {
#define BNN_LDS(ST, TT, KK)                                                \
  if (stride == ST && tm == TT && kb == KK) {                              \
    launch_lds_one<S, ST, TT, KK>(a, blocks, lds_bytes, stream);           \
    return true;                                                           \
  }
  BNN_LDS(1, 7, 1) BNN_LDS(1, 8, 1) BNN_LDS(1, 13, 1) BNN_LDS(1, 7, 2) BNN_LDS(1, 8, 2) BNN_LDS(1, 13, 2)
  BNN_LDS(2, 7, 1) BNN_LDS(2, 8, 1) BNN_LDS(2, 7, 2) BNN_LDS(2, 8, 2)
#undef BNN_LDS
  return false;
}

template <int R, int S, int STRIDE, int CW, int TM>
void launch_resident_one(const ConvArgs& a, uint32_t blocks, hipStream_t stream) {
  rtc::prof_begin(kProfileKind, stream);
  RTC_LAUNCH((bconv_resident_kernel<R, S, STRIDE, CW, TM>), dim3(blocks), dim3(64), 0, stream, a.x, a.w, a.xi,
                     a.gamma, a.out_x1, a.out_x4, a);
  rtc::prof_end(stream);
}

// true when a resident-filter instantiation exists for the shape (and it was launched)
bool launch_resident(const ConvArgs& a, int R, int S, int stride, int tm, uint32_t blocks, hipStream_t stream) {
  const int cw = a.Cw;
#define BNN_RESIDENT_TM(RR, SS, ST, CC, TT)                                \
  if (R == RR && S == SS && cw == CC && stride == ST && tm == TT) {        \
    launch_resident_one<RR, SS, ST, CC, TT>(a, blocks, stream);            \
    return true;                                                           \
  }
#define BNN_RESIDENT(RR, SS, CC)                                           \
  BNN_RESIDENT_TM(RR, SS, 1, CC, 7) BNN_RESIDENT_TM(RR, SS, 1, CC, 8) BNN_RESIDENT_TM(RR, SS, 1, CC, 13) \
  BNN_RESIDENT_TM(RR, SS, 2, CC, 7) BNN_RESIDENT_TM(RR, SS, 2, CC, 8)
  BNN_RESIDENT(1, 1, 1) BNN_RESIDENT(1, 1, 2) BNN_RESIDENT(1, 1, 4)
  BNN_RESIDENT(3, 3, 1) BNN_RESIDENT(3, 3, 2) BNN_RESIDENT(3, 3, 4)
  BNN_RESIDENT(5, 5, 1)
#undef BNN_RESIDENT
#undef BNN_RESIDENT_TM
  return false;
}

template <int R, int S, int CW, int TM>
void launch_resident_half_one(const ConvArgs& a, uint32_t blocks, hipStream_t stream) {
  rtc::prof_begin(kProfileKind, stream);
  if constexpr (CW == 1 && S == 3) {
    if (a.C <= 16) {                              // half-filled words: two taps per instruction pair
      RTC_LAUNCH((bconv_resident_half_kernel<R, S, CW, TM, true>), dim3(blocks), dim3(64), 0, stream, a.x, a.w, a.xi,
                 a.gamma, a.out_x1, a.out_x4, a);
      rtc::prof_end(stream);
      return;
    }
  }
  RTC_LAUNCH((bconv_resident_half_kernel<R, S, CW, TM, false>), dim3(blocks), dim3(64), 0, stream, a.x, a.w, a.xi, a.gamma,
                     a.out_x1, a.out_x4, a);
  rtc::prof_end(stream);
}

// the two-tiles-per-wave form for at most 32 filters; true when an instantiation exists
bool launch_resident_half(const ConvArgs& a, int R, int S, int tm, uint32_t blocks, hipStream_t stream) {
  const int cw = a.Cw;
#define BNN_HALF(RR, SS, CC, TT)                                           \
  if (R == RR && S == SS && cw == CC && tm == TT) {                        \
    launch_resident_half_one<RR, SS, CC, TT>(a, blocks, stream);           \
    return true;                                                           \
  }
  BNN_HALF(3, 3, 1, 7) BNN_HALF(3, 3, 1, 8) BNN_HALF(3, 3, 1, 13) BNN_HALF(3, 3, 2, 7) BNN_HALF(3, 3, 2, 8) BNN_HALF(3, 3, 2, 13)
  BNN_HALF(1, 1, 1, 7) BNN_HALF(1, 1, 1, 8) BNN_HALF(1, 1, 1, 13) BNN_HALF(5, 5, 1, 7) BNN_HALF(5, 5, 1, 8) BNN_HALF(5, 5, 1, 13)
#undef BNN_HALF
  return false;
}

// Output pixels per wave: the candidate that leaves the fewest idle slots in an output row of
// Wo pixels (ties: the wider tile).
std::atomic<int> g_force_tm{0}, g_force_kb{0};   // planner overrides, see bnn_set_planner
std::atomic<int> g_matrix_path{0};        // see bnn_set_matrix_path

int pick_tm(int64_t Wo, bool allow13) {
  if (g_force_tm == 7 || g_force_tm == 8 || (g_force_tm == 13 && allow13)) return g_force_tm;
  int best = 8;
  int64_t best_slots = (Wo + 7) / 8 * 8;
  const int cands[2] = {7, 13};
  for (int c : cands) {
    if (c == 13 && !allow13) continue;
    const int64_t slots = (Wo + c - 1) / c * c;
    if (slots < best_slots || (slots == best_slots && c > best)) { best = c; best_slots = slots; }
  }
  return best;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

constexpr int64_t kMaxDim = 1 << 20;
// below this many output pixels the matrix-core kernel's 512-pixel workgroups leave the chip idle
constexpr int64_t kMatrixMinPixels = 4096;

// The planner's choice for a layer (the launcher can still decline: rows of more than 127 pixels
// and images of very few pixels need more LDS slots than the kernel stages).
bool matrix_path_wanted(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S, int64_t stride,
                        int64_t pad) {
  return g_matrix_path >= 0 && mfma_shape(K, R, S, C) && stride == 1 && pad == 1 &&
         (g_matrix_path > 0 || N * H * W >= kMatrixMinPixels);
}

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
    RTC_LAUNCH(pack_channels_kernel<int8_t>, grid, dim3(64), 0, stream, static_cast<const int8_t*>(x), words,
                       rows, (int)C, (int)Cw, (int)cblocks);
  else
    RTC_LAUNCH(pack_channels_kernel<float>, grid, dim3(64), 0, stream, static_cast<const float*>(x), words,
                       rows, (int)C, (int)Cw, (int)cblocks);
  return hip_status();
}

size_t bnn_weight_words(int64_t K, int64_t R, int64_t S, int64_t C) {
  using namespace bnn;
  if (K < 1 || R < 1 || S < 1 || C < 1 || K > kMaxDim || C > kMaxDim || R > 64 || S > 64) return 0;
  const int64_t Kp = (K + 63) / 64 * 64, Cw = (C + 31) / 32;
  // (a multiple of 4 words, so the int8 fragments that may follow start on a 16-byte boundary)
  return (size_t)(R * S * Cw * Kp + R * S * Kp) + mfma_bank_bytes(K, R, S, C) / 4;
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
  RTC_LAUNCH(pack_weights_kernel, dim3((uint32_t)((taps * Cw * Kp + 255) / 256)), dim3(256), 0, stream, w,
                     packed, (int)K, (int)taps, (int)C, (int)Cw, (int)Kp);
  RTC_LAUNCH(weight_popcount_kernel, dim3((uint32_t)((taps * Kp + 255) / 256)), dim3(256), 0, stream, packed,
                     (int)taps, (int)Cw, (int)Kp);
  if (mfma_shape(K, R, S, C))
    launch_pack_weights_mfma(w, reinterpret_cast<int8_t*>(packed + taps * Cw * Kp + taps * Kp), K, C, stream);
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
  // offsets inside one image and inside the filter bank are formed in 32 bits
  // |x1| <= R S C must convert to fp32 exactly (the threshold comparison is an fp32 one)
  if (R * S * C > (1 << 24) || bnn_weight_words(K, R, S, C) > 0x7fffffffULL || H * W * Cw > 0x7fffffffLL) return BNN_ERR_SHAPE;
  const int64_t kblocks = Kp / 64;
  const int qc = Cw % 4 == 0 ? 4 : Cw % 2 == 0 ? 2 : 1;
  ConvArgs a;
  a.x = x; a.w = packed; a.xi = xi; a.gamma = gamma; a.out_x1 = out_x1; a.out_x4 = out_x4;
  a.N = (int32_t)N; a.H = (int32_t)H; a.W = (int32_t)W; a.C = (int32_t)C; a.Cw = (int32_t)Cw; a.K = (int32_t)K; a.Kp = (int32_t)Kp;
  a.Kw = (int32_t)Kw; a.R = (int32_t)R; a.pad = (int32_t)pad; a.Ho = (int32_t)Ho; a.Wo = (int32_t)Wo;
  a.kblocks = (int32_t)kblocks;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  // many channels and filters, 3 x 3, same-size output: a dense contraction for the matrix cores
  if (matrix_path_wanted(N, H, W, C, K, R, S, stride, pad) && aligned(packed, 16)) {
    MfmaArgs m;
    m.x = x; m.wbytes = reinterpret_cast<const int8_t*>(packed + R * S * Cw * Kp + R * S * Kp);
    m.xi = xi; m.gamma = gamma; m.out_x1 = out_x1; m.out_x4 = out_x4;
    m.N = (int32_t)N; m.H = (int32_t)H; m.W = (int32_t)W; m.Cw = (int32_t)Cw; m.K = (int32_t)K;
    const int mode = g_matrix_path;
    if (launch_bconv_mfma(m, stream, mode == 3 || mode == 4 ? mode : 0)) return hip_status();
  }
  // few channels: the filters stay in registers and a wave streams over several tiles, enough
  // of them that a launch has about 32K waves (measured: better than 8K or 16K)
  const bool resident_shape = R == S && Cw <= 4 && (Cw & (Cw - 1)) == 0 && R * S * Cw <= 36;
  if (resident_shape) {
    int tm = pick_tm(Wo, stride == 1);
    if (((tm - 1) * stride + S) * Cw > 64) tm = 7;          // one lane per word of a strip row
    const int64_t wtiles = (Wo + tm - 1) / tm;
    const int64_t tiles_per_image = Ho * wtiles;
    int64_t tpw = (N * tiles_per_image * kblocks + 32767) / 32768;
    if (tpw > tiles_per_image) tpw = tiles_per_image;
    if (tpw > 64) tpw = 64;
    const int64_t wpi = (tiles_per_image + tpw - 1) / tpw;
    if (N * wpi * kblocks > 0x7fffffffLL) return BNN_ERR_SHAPE;
    a.wtiles = (int32_t)wtiles; a.tiles_per_wave = (int32_t)tpw; a.waves_per_image = (int32_t)wpi;
    if (K <= 32 && stride == 1 && (tm - 1 + S) * Cw <= 32 && g_force_kb != 1) {
      // at most 32 filters: two tiles per wave, one per half (the knob's value 1 asks for the plain form)
      const int64_t tpw2 = (tpw + 1) / 2 * 2;
      const int64_t wpi2 = (tiles_per_image + tpw2 - 1) / tpw2;
      ConvArgs h = a;
      h.tiles_per_wave = (int32_t)tpw2; h.waves_per_image = (int32_t)wpi2;
      if (launch_resident_half(h, (int)R, (int)S, tm, (uint32_t)(N * wpi2), stream)) return hip_status();
    }
    if (((tm - 1) * stride + S) * Cw <= 64 &&
        launch_resident(a, (int)R, (int)S, (int)stride, tm, (uint32_t)(N * wpi * kblocks), stream))
      return hip_status();
  }
  // wide pixels: the strip goes through LDS, 4 waves = 4 groups of KB filter blocks per tile
  if (qc == 4 && aligned(x, 16)) {
    const int tm = pick_tm(Wo, stride == 1);
    // one block of filters per wave measured faster than two (registers, occupancy); two only on request,
    // and only when no wave would own half a pair
    const int kb = g_force_kb == 2 && kblocks % 2 == 0 ? 2 : 1;
    const int ps = (tm - 1) * (int)stride + (int)S;
    const size_t lds_bytes = (size_t)R * ps * Cw * 4;
    const int64_t wtiles = (Wo + tm - 1) / tm;
    const int64_t kgroups = (kblocks + 4 * kb - 1) / (4 * kb);
    const int64_t blocks = N * Ho * wtiles * kgroups;
    if (blocks > 0x7fffffffLL) return BNN_ERR_SHAPE;
    a.wtiles = (int32_t)wtiles; a.tiles_per_wave = 0; a.waves_per_image = 0;
    if (lds_bytes <= 64 * 1024) {
      bool launched;
      if (S == 1) launched = launch_lds_s<1>(a, (int)stride, tm, kb, (uint32_t)blocks, lds_bytes, stream);
      else if (S == 3) launched = launch_lds_s<3>(a, (int)stride, tm, kb, (uint32_t)blocks, lds_bytes, stream);
      else launched = launch_lds_s<5>(a, (int)stride, tm, kb, (uint32_t)blocks, lds_bytes, stream);
      if (launched) return hip_status();
    }
  }
  const int tm = pick_tm(Wo, false);
  const int64_t wtiles = (Wo + tm - 1) / tm;
  const int64_t blocks = N * Ho * wtiles * kblocks;
  if (blocks > 0x7fffffffLL) return BNN_ERR_SHAPE;
  a.wtiles = (int32_t)wtiles; a.tiles_per_wave = 0; a.waves_per_image = 0;
  bool launched;
  if (S == 1) launched = launch_general_s<1>(a, (int)stride, qc, tm, (uint32_t)blocks, stream);
  else if (S == 3) launched = launch_general_s<3>(a, (int)stride, qc, tm, (uint32_t)blocks, stream);
  else launched = launch_general_s<5>(a, (int)stride, qc, tm, (uint32_t)blocks, stream);
  if (!launched) return BNN_ERR_UNSUPPORTED;
  return hip_status();
}

int bnn_set_planner(int tile_pixels, int filter_blocks) {
  if ((tile_pixels != 0 && tile_pixels != 7 && tile_pixels != 8 && tile_pixels != 13) || filter_blocks < 0 ||
      filter_blocks > 2)
    return BNN_ERR_SHAPE;
  bnn::g_force_tm = tile_pixels;
  bnn::g_force_kb = filter_blocks;
  return BNN_OK;
}

int bnn_set_matrix_path(int mode) {
  if (mode < -1 || mode == 2 || mode > 4) return BNN_ERR_SHAPE;
  bnn::g_matrix_path = mode;
  return BNN_OK;
}

int bnn_matrix_path_applies(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S, int64_t stride,
                            int64_t pad) {
  using namespace bnn;
  if (N < 1 || H < 1 || W < 1 || C < 1 || K < 1 || R < 1 || S < 1) return 0;
  return matrix_path_wanted(N, H, W, C, K, R, S, stride, pad) && mfma_slots_fit(H, W) ? 1 : 0;
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
