// Binary convolution on the matrix cores of gfx950 (the paper's binary convolution operation and
// layer integration sections; the instruction choice is this machine's, not the paper's).
//
// A binary dot product is a dense contraction: with +1 / -1 stored as int8, x1 = sum x w is
// what v_mfma_i32_32x32x32_i8 accumulates, 32768 multiply-accumulates per instruction against 64
// per v_xor_b32 + v_bcnt_u32_b32 pair on the vector ALU.  The price is the unpacking of bits to
// bytes, which is paid once per staged value and amortised over the filters (activations) resp.
// done when the filter bank is prepared (filters).
//
// Mapping.  Output pixels are numbered q = (n H + y) W + x over the whole batch (stride 1 and
// padding 1 keep the output the size of the input).  A workgroup of 4 waves owns 128 MT
// consecutive pixels and 64 consecutive filters; wave w owns the pixel tiles
// [32 (w MT + mt), +32), mt < MT, and both 32-filter tiles: 2 MT accumulator tiles of 16 registers.
// Per word of channels (32 channels = one K step of the instruction):
//   * the words of the input pixels that the workgroup's taps touch are unpacked to bytes in LDS,
//     16 bytes per pixel in each of two planes (channels 0..15 and 16..31 of the word), so that
//     consecutive lanes read consecutive 16-byte pieces.  LDS slots follow the PADDED image: slot
//     t(n, y, x) = (n (H + 1) + y) (W + 1) + x, so every image row is followed by one slot and
//     every image by one row of slots that hold zeros.  The tap (dy, dx) of any pixel is then the
//     slot t + dy (W + 1) + dx, also at the borders, where it is one of the zero slots -- zero
//     padding: such taps add nothing -- and no lane needs a mask;
//   * the filter fragments of this channel word (18 KB: 9 taps x 2 tiles of 32 filters) are
//     copied to LDS as they are;
//   * for each of the 9 taps a lane reads the 16 bytes of "its" pixel shifted by the tap
//     (row i = lane % 32 of the A operand, channels 16 (lane / 32) ... + 15) and, once per tap,
//     the 16 bytes of filter lane % 32 for the same channels (B operand).
// Both stagings go through registers two channel words ahead and through one of two LDS buffers
// one word ahead: while the matrix instructions of word cw read one buffer, word cw + 1 is
// unpacked into the other and word cw + 2 is on its way from memory; one barrier per word.
// The contraction sums over (tap, channel) in any order, so only the pairing of A and B bytes
// matters: both use lane / 32 for the half and the byte index for the channel.
// Result layout of the instruction (checked on the device): register r of lane l holds row
// 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32.  Columns are filters, so the 64-lane compare mask
// of register r IS the packed output word of two pixels (rows ... and ... + 4): the ballot packs.
#include <hip/hip_runtime.h>

#include "bnn_internal.h"
#include "rtc_internal.h"

namespace bnn {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kProfileKind = 32;    // the convolution kernel's kind in the timing record
constexpr int kPitch = 16;          // bytes per staged pixel and half (16 channels)
constexpr int kMinChannels = 128;   // below that the vector-ALU kernels keep their filters in registers (64 channels on
                                    // a 52 x 52 map, 128 filters, batch 256: 0.132 ms here against 0.107 ms there)

// 4 bits -> 4 bytes of +1 (bit set) / -1, or 4 zero bytes.  The multiplication puts bit j of the
// nibble at bit 8 j (the partial products n << 0, 7, 14, 21 do not collide there); the byte
// permute then looks every byte up in the table {0: 0xFF, 1: 0x01}.  `zero` = 0x0C0C0C0C together
// with n = 0 makes every selector 12, which yields 0x00; `zero` = 0 changes nothing.
__device__ __forceinline__ uint32_t nibble_to_signs(uint32_t n, uint32_t zero) {
  const uint32_t spread = (__umul24(n, 0x204081u) & 0x01010101u) | zero;
  return __builtin_amdgcn_perm(0x000001FFu, 0x000001FFu, spread);
}

// ---- filter fragments -------------------------------------------------------------------------
// bank[((((fg Cw + cw) 9 + tap) 2 + nt) 64 + lane) 16 + j] = w[fg 64 + nt 32 + lane % 32][tap][cw 32 + 16 (lane / 32) + j]
__global__ __launch_bounds__(256) void pack_weights_mfma_kernel(const int8_t* __restrict__ w, int8_t* __restrict__ bank,
                                                                int K, int C, int Cw) {
  const int64_t frag = (int64_t)blockIdx.x * 256 + threadIdx.x;      // one 16-byte fragment per thread
  const int64_t total = (int64_t)(K / 64) * Cw * 9 * 2 * 64;
  if (frag >= total) return;
  const int lane = (int)(frag % 64);
  const int nt = (int)((frag / 64) % 2);
  const int tap = (int)((frag / 128) % 9);
  const int cw = (int)((frag / (128 * 9)) % Cw);
  const int fg = (int)(frag / ((int64_t)128 * 9 * Cw));
  const int k = fg * 64 + nt * 32 + lane % 32;
  const int8_t* src = w + ((int64_t)k * 9 + tap) * C + cw * 32 + 16 * (lane / 32);
  int8_t* dst = bank + frag * 16;
#pragma unroll
  for (int j = 0; j < 16; ++j) dst[j] = src[j] > 0 ? (int8_t)1 : (int8_t)-1;
}

// ---- convolution ------------------------------------------------------------------------------
constexpr int kTilesPerWave = 4;                     // MT: pixel tiles of 32 per wave
constexpr int kStageRounds = 3;                      // staged slots per thread and channel word
constexpr int kMaxSlots = 256 * kStageRounds;
constexpr int kFragBytes = 9 * 2 * 64 * 16;          // filter fragments of one (filter group, channel word)
constexpr int kFragChunks = kFragBytes / 16;         // in 16-byte pieces: 1152 = 4.5 per thread
constexpr int kFragRounds = (kFragChunks + 255) / 256;

// slot of pixel q in the padded numbering
__device__ __forceinline__ int64_t padded_slot(int64_t q, int H, int W) {
  const int64_t row = q / W;                         // n H + y
  const int x = (int)(q - row * W);
  const int64_t n = row / H;
  const int y = (int)(row - n * H);
  return (n * (H + 1) + y) * (W + 1) + x;
}

// QC: channel words that a thread fetches per staged pixel at a time (4 where a pixel's words
// allow 16-byte loads: a word-by-word walk would pull every pixel's cache line in again for each
// word).
template <int MT, int QC>
__global__ __launch_bounds__(256, 2) void bconv_mfma_kernel(const MfmaArgs a, int fgroups, int plane) {
  typedef uint32_t xwords __attribute__((ext_vector_type(QC)));
  extern __shared__ __align__(16) unsigned char lds[];
  // two buffers of [filter fragments of a channel word][unpacked pixels: two planes]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = lane & 31, h = lane >> 5;
  const int W = a.W, H = a.H, Cw = a.Cw, PW = W + 1, PH = H + 1;
  const int64_t total = (int64_t)a.N * H * W;
  constexpr int kWgPixels = 4 * MT * 32;
  const int fg = blockIdx.x % fgroups;
  const int64_t P0 = (int64_t)(blockIdx.x / fgroups) * kWgPixels;
  const int64_t Plast = P0 + kWgPixels - 1 < total ? P0 + kWgPixels - 1 : total - 1;
  const int64_t slot0 = padded_slot(P0, H, W) - (PW + 1);
  const int slots = (int)(padded_slot(Plast, H, W) + (PW + 1) + 1 - slot0);   // <= kMaxSlots (launcher)

  // the lane's pixel of each of the wave's tiles (pixels beyond the last one read the last one's
  // data; their results are not stored)
  int lds_pix[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int64_t q = P0 + (wave * MT + mt) * 32 + i;
    if (q > Plast) q = Plast;
    lds_pix[mt] = (int)(padded_slot(q, H, W) - slot0 - 1) * kPitch + plane * h;     // the tap (0, -1)
  }

  v16i acc[MT][2];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc[mt][0][r] = 0; acc[mt][1][r] = 0; }
  }

  // what a thread stages per channel word: up to kStageRounds slots and kFragRounds 16-byte pieces
  // of the filter fragments (in the last round the upper half of the threads repeats the lower
  // half's pieces)
  const uint32_t* xsrc[kStageRounds];
  bool xreal[kStageRounds];
  int xdst[kStageRounds];
#pragma unroll
  for (int j = 0; j < kStageRounds; ++j) {
    int s = threadIdx.x + 256 * j;
    if (s > slots - 1) s = slots - 1;
    const int64_t t = slot0 + s;
    const int64_t prow = t >= 0 ? t / PW : -1;
    const int x = (int)(t - prow * PW);
    const int64_t n = prow >= 0 ? prow / PH : 0;
    const int y = (int)(prow - n * PH);
    xreal[j] = prow >= 0 && x < W && y < H && n < a.N;
    xsrc[j] = a.x + (xreal[j] ? ((n * H + y) * W + x) * Cw : 0);
    xdst[j] = s * kPitch;
  }
  const v4i* wsrc = reinterpret_cast<const v4i*>(a.wbytes + (int64_t)fg * Cw * kFragBytes);
  xwords xr[kStageRounds];
  // Fetches are never conditional (a word index past the end is clamped: the values are then
  // staged into a buffer that nobody reads), so that the loop body below is one basic block in
  // which the compiler can place the staging between the matrix instructions.
  auto fetch_x = [&](int cw) {                 // the QC words from cw on (cw a multiple of QC)
    const int c = cw < Cw - QC ? cw : Cw - QC;
#pragma unroll
    for (int j = 0; j < kStageRounds; ++j) xr[j] = *reinterpret_cast<const xwords*>(xsrc[j] + c);
  };
  // The filter fragments need no unpacking: they go from memory straight into LDS
  // (global_load_lds_dwordx4: lane l of a wave writes 16 bytes at the wave's LDS base + 16 l), one
  // wave per run of 64 pieces; the copy is complete for everybody after the copying wave's
  // s_waitcnt vmcnt(0) and the workgroup's barrier.
  auto stage_w = [&](int cw, unsigned char* buf) {
    const int c = cw < Cw - 1 ? cw : Cw - 1;
#pragma unroll
    for (int j = 0; j < kFragRounds; ++j) {
      const int piece0 = 256 * j + 64 * wave;            // (wave-uniform)
      if (piece0 < kFragChunks)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(wsrc + c * kFragChunks + piece0 + lane),
                                         (__attribute__((address_space(3))) void*)(buf + piece0 * 16), 16, 0, 0);
    }
  };

  // Two LDS buffers: while the matrix instructions of channel word cw read one, the word cw + 1
  // (fetched into registers an iteration earlier) is unpacked into the other, so a wave's own
  // staging runs under its own matrix instructions and an iteration needs one barrier: the buffer
  // written in iteration cw was last read in iteration cw - 1, which every wave has left.
  // (A staging round beyond the workgroup's slots repeats its last slot: same bytes, same place.)
  const int buf_bytes = kFragBytes + 2 * plane;
  auto stage = [&](int sub, unsigned char* buf) {       // word `sub` of the fetched QC words
    unsigned char* const bA = buf + kFragBytes;
#pragma unroll
    for (int j = 0; j < kStageRounds; ++j) {
      uint32_t word = xr[j][sub];
      if (!xreal[j]) word = 0u;                               // a padding slot: zeros
      const uint32_t zero = xreal[j] ? 0u : 0x0C0C0C0Cu;
      uint4 lo, hi;
      lo.x = nibble_to_signs(word & 15u, zero);         lo.y = nibble_to_signs((word >> 4) & 15u, zero);
      lo.z = nibble_to_signs((word >> 8) & 15u, zero);  lo.w = nibble_to_signs((word >> 12) & 15u, zero);
      hi.x = nibble_to_signs((word >> 16) & 15u, zero); hi.y = nibble_to_signs((word >> 20) & 15u, zero);
      hi.z = nibble_to_signs((word >> 24) & 15u, zero); hi.w = nibble_to_signs(word >> 28, zero);
      *reinterpret_cast<uint4*>(bA + xdst[j]) = lo;
      *reinterpret_cast<uint4*>(bA + plane + xdst[j]) = hi;
    }
  };
  stage_w(0, lds);
  fetch_x(0);
  stage(0, lds);
  if constexpr (QC == 1) fetch_x(1);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  for (int cq = 0; cq < Cw; cq += QC) {
#pragma unroll
    for (int sub = 0; sub < QC; ++sub) {
      const int cw = cq + sub;
      const unsigned char* const curB = lds + (cw & 1) * buf_bytes;
      const unsigned char* const curA = curB + kFragBytes;
      stage_w(cw + 1, lds + ((cw + 1) & 1) * buf_bytes);
      stage((sub + 1) % QC, lds + ((cw + 1) & 1) * buf_bytes);
      if ((sub + 2) % QC == 0) fetch_x(cw + 2);          // (decided at compile time)
      // operands of tap t + 1 are requested before the matrix instructions of tap t
      v4i bq[2][2], aq[2][MT];
      auto read_tap = [&](int tap, int buf) {
        bq[buf][0] = *reinterpret_cast<const v4i*>(curB + ((tap * 2 + 0) * 64 + lane) * 16);
        bq[buf][1] = *reinterpret_cast<const v4i*>(curB + ((tap * 2 + 1) * 64 + lane) * 16);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          aq[buf][mt] = *reinterpret_cast<const v4i*>(curA + lds_pix[mt] + (tap / 3 - 1) * PW * kPitch + (tap % 3) * kPitch);
      };
      read_tap(0, 0);
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        if (tap + 1 < 9) read_tap(tap + 1, (tap + 1) & 1);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          acc[mt][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aq[tap & 1][mt], bq[tap & 1][0], acc[mt][0], 0, 0, 0);
          acc[mt][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aq[tap & 1][mt], bq[tap & 1][1], acc[mt][1], 0, 0, 0);
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's share of the next word's fragments has landed
      __syncthreads();                       // reads of this word done, the next word's buffer complete
    }
  }

  // epilogue: x1 as it is, and / or the integrated layer's bit, packed by the ballot
  const int Kw = a.K / 32;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int k = fg * 64 + nt * 32 + i;
    int32_t T = 0;
    bool positive = false;
    if (a.out_x4 != nullptr) {
      positive = a.gamma[k] > 0.f;
      T = integer_threshold(a.xi[k], positive);
    }
    const unsigned long long posmask = __ballot(positive);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r / 4) + 4 * h + (r % 4);
        const int64_t q = P0 + (wave * MT + mt) * 32 + row;
        const int32_t x1 = acc[mt][nt][r];
        if (a.out_x1 != nullptr && q < total) a.out_x1[q * a.K + k] = x1;
        if (a.out_x4 != nullptr) {
          const unsigned long long mask = __ballot(x1 < T) ^ posmask;
          // lanes 0..31 hold the pixel of row (h = 0), lanes 32..63 the one four rows further
          if (i == 0 && q < total) a.out_x4[q * Kw + fg * 2 + nt] = (uint32_t)(h ? mask >> 32 : mask);
        }
      }
    }
  }
}

}  // namespace

bool mfma_shape(int64_t K, int64_t R, int64_t S, int64_t C) {
  return R == 3 && S == 3 && C % 32 == 0 && C >= kMinChannels && K % 64 == 0;
}

size_t mfma_bank_bytes(int64_t K, int64_t R, int64_t S, int64_t C) {
  return mfma_shape(K, R, S, C) ? (size_t)K * 9 * C : 0;
}

void launch_pack_weights_mfma(const int8_t* w, int8_t* bank, int64_t K, int64_t C, hipStream_t stream) {
  const int64_t frags = (K / 64) * (C / 32) * 9 * 2 * 64;
  RTC_LAUNCH(pack_weights_mfma_kernel, dim3((uint32_t)((frags + 255) / 256)), dim3(256), 0, stream, w, bank, (int)K,
             (int)C, (int)(C / 32));
}

// Upper bound of the padded slots that a workgroup's pixels and their taps span: its pixels, one
// slot per end of an image row and one row of slots per end of an image that lie between its
// first and last pixel, and a padded row + 1 on either side.  (It sizes the LDS buffers: two
// workgroups per CU need it tight.)
static int64_t slot_bound(int64_t H, int64_t W) {
  constexpr int kWgPixels = 4 * kTilesPerWave * 32;
  const int64_t row_ends = (kWgPixels - 1) / W + 1, image_ends = (kWgPixels - 1) / (H * W) + 1;
  return kWgPixels + row_ends + image_ends * (W + 1) + 2 * (W + 2) + 1;
}

bool mfma_slots_fit(int64_t H, int64_t W) { return slot_bound(H, W) <= kMaxSlots; }

namespace {

template <int MT>
bool launch_tiles(const MfmaArgs& a, int64_t total, int64_t fgroups, size_t lds_bytes, int plane, hipStream_t stream) {
  constexpr int kWgPixels = 4 * MT * 32;
  const int64_t blocks = (total + kWgPixels - 1) / kWgPixels * fgroups;
  if (blocks > 0x7fffffffLL) return false;
  // more dynamic LDS than the default limit of a kernel: ask for it once per process
  static const bool lds_ok = [] {
    constexpr int kMaxLds = 2 * (kFragBytes + 2 * ((kMaxSlots * kPitch + 255) / 256 * 256 + 128));
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&bconv_mfma_kernel<MT, 4>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) == hipSuccess &&
           hipFuncSetAttribute(reinterpret_cast<const void*>(&bconv_mfma_kernel<MT, 1>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) == hipSuccess;
  }();
  if (!lds_ok) return false;
  rtc::prof_begin(kProfileKind, stream);
  if (a.Cw % 4 == 0 && reinterpret_cast<uintptr_t>(a.x) % 16 == 0)
    RTC_LAUNCH((bconv_mfma_kernel<MT, 4>), dim3((uint32_t)blocks), dim3(256), lds_bytes, stream, a, (int)fgroups, plane);
  else
    RTC_LAUNCH((bconv_mfma_kernel<MT, 1>), dim3((uint32_t)blocks), dim3(256), lds_bytes, stream, a, (int)fgroups, plane);
  rtc::prof_end(stream);
  return true;
}

}  // namespace

bool launch_bconv_mfma(const MfmaArgs& a, hipStream_t stream, int tiles) {
  const int64_t total = (int64_t)a.N * a.H * a.W;
  if (!mfma_slots_fit(a.H, a.W)) return false;               // long rows or tiny images: another kernel
  const int64_t slot_bound = bnn::slot_bound(a.H, a.W);
  // the two halves of the staged pixels (channels 0..15 and 16..31 of the word) lie in two planes
  // an odd multiple of 128 bytes apart: the 16 lanes that the LDS serves per cycle then hit 16
  // different bank groups whether they belong to one half or to both
  const int plane = (int)((slot_bound * kPitch + 255) / 256 * 256 + 128);
  const size_t lds_bytes = 2 * ((size_t)kFragBytes + 2 * (size_t)plane);       // two buffers
  const int64_t fgroups = a.K / 64;
  // Workgroups of one size run in rounds of one per slot (two slots per CU), and a partly filled
  // last round costs about as much as a full one.  Three tiles per wave instead of four (a round
  // then costs about 3.3 / 4.3 of a full-size one: prologue, epilogue and the filter fragments do
  // not shrink) win where they save a round's worth: conv6 of the detector trunk at batch 256,
  // 680 workgroups of four tiles = 2 rounds against 904 of three = 2 cheaper ones (74 -> 69 us);
  // conv5, conv7 and conv8 stay with four (measured 0 to 3 % slower with three).  Cutting a layer
  // into whole rounds of full-size workgroups plus a second launch of smaller ones for the rest was
  // measured too and not kept (conv8 3 % quicker, conv5 and conv6 4 to 6 % slower: the second
  // launch waits for the first to drain).
  static const int cus = [] {                                 // (the devices of a process are alike)
    int device = 0, count = 0;
    if (hipGetDevice(&device) != hipSuccess ||
        hipDeviceGetAttribute(&count, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess)
      return 0;
    return count;
  }();
  const int64_t slots = 2 * (int64_t)(cus > 0 ? cus : 256);
  auto cost = [&](int mt) {
    const int64_t wgs = (total + 128 * mt - 1) / (128 * mt) * fgroups;
    return (double)((wgs + slots - 1) / slots) * (mt + 0.3);
  };
  if (tiles == 3 || (tiles != 4 && cost(3) < cost(4))) return launch_tiles<3>(a, total, fgroups, lds_bytes, plane, stream);
  return launch_tiles<4>(a, total, fgroups, lds_bytes, plane, stream);
}

}  // namespace bnn
