// Tropical (min,+) / (max,-) products on the vector ALUs of gfx950.
//
//   min-plus convolution     out[t] = min_{0<=s<=t}     f[s]   + g[t-s]
//   max-plus deconvolution   out[t] = max_{0<=u<=n-1-t} f[t+u] - g[u]
//
// Both are instances of one triangular product
//   out'[t] = REDUCE_{0<=s<=t} COMBINE(b'[t-s], a[s])
// with (a, b') = (f, g), COMBINE = +, REDUCE = min for the convolution, and
// (a, b') = (g, f reversed), COMBINE = window - uniform, REDUCE = max, output stored
// reversed, for the deconvolution (substitute t -> n-1-t).
//
// Mapping to the machine (one wave64 per workgroup, no barriers between waves):
//   * a wave owns a tile of W = 64*R consecutive outputs; lane l owns the R consecutive
//     outputs t0 + l*R .. t0 + l*R + R-1 and keeps their running reductions in VGPRs;
//   * the operand indexed by s is wave-uniform: it is fetched with scalar loads and used
//     as the SGPR source of the VALU add/sub, so it costs no vector issue slot;
//   * the operand indexed by t-s is a sliding window: per block of R steps a lane needs
//     one new aligned group of R values, read from an LDS copy of the window with
//     16-byte reads.  Groups are stored with a 16-byte skew per group so that the 64 lanes
//     (whose groups are consecutive) hit distinct banks;
//   * per (lane, step, output) the inner loop is exactly one add/sub and one min/max.
// The s range of a tile is cut into segments so that a launch has enough equally sized work
// items; partial results of one tile are merged with atomic min/max (exact and order-free).
// On the diagonal (s-block overlapping the tile) block j only concerns lanes > j, which run
// under an exec mask; each lane's own R x R triangle is finished by a short epilogue.
//
// Packed 16-bit path (int32 arithmetic only).  A common slope rho is removed from both
// operands: with ad[s] = a[s] - rho*s and bd[i] = b'[i] -/+ rho*i (minus for the convolution,
// plus for the deconvolution, whose window operand is the reversed, hence falling, f) every
// candidate equals COMBINE(bd[t-s], ad[s]) +/- rho*t, so the trend is put back once per output.
// Per chunk of 1024 steps the detrended values are re-based to the chunk / window minimum;
// when range(ad chunk) + range(bd window) <= 65534 every candidate of that (tile, chunk) fits
// an unsigned 16-bit lane, and two output halves of a 2048-wide tile are computed at once with
// v_pk_add_u16 + v_pk_min_u16 (v_pk_sub_u16 + v_pk_max_u16 for the deconvolution), both
// saturating: one VALU instruction per pair-op instead of 1.5.
// Positions that do not exist (window index < 0, s >= n) are staged as a poison value that
// saturates and never wins, so the packed kernel needs neither exec masks nor a triangle epilogue.
// The decision is made per (row, tile, chunk) from precomputed block minima / maxima; chunks
// that do not qualify are done by the 32-bit kernel, which evaluates the same predicate and
// skips exactly the chunks the packed kernel owns.  Results are exact in both cases.
// (tropical_packed.h also has the flavour for chunks that fit 15 bits, where the packed
// three-operand half-float minimum / maximum acts as an exact integer min3 / max3: 0.75 VALU
// instructions per pair-op.)
//
// Other row-dependent paths, each chosen per row pair on the device, all with bit-identical
// results: rows of exploitable convexity or periodicity (tropical_structured.h); int64 rows
// narrowed to 32 bits by their minima or with the pair's common slope removed (the probe kernels
// of tropical_prepare.h), or re-based per chunk (tropical_rebased.h); the 64-bit kernel takes what
// is left.  Problems with too few work items to fill the chip use the same kernel with small
// tiles (kSmallR).
#include <hip/hip_runtime.h>

#include <limits>
#include <type_traits>

#include "rtc_internal.h"
#include "tropical_common.h"
#include "tropical_generic.h"
#include "tropical_packed.h"
#include "tropical_prepare.h"
#include "tropical_structured.h"
#include "tropical_rebased.h"

namespace rtc {

std::atomic<int64_t> g_packed_small_n{4096};   // rows up to this length use the narrower packed tiles
std::atomic<bool> g_structure_paths{true};     // rows of exploitable convexity / periodicity take their own kernels
std::atomic<int64_t> g_small_items{RTC_DEFAULT_SMALL_PROBLEM_ITEMS};   // problems with fewer work items than this get the small tiles, see kSmallR
std::atomic<int> g_rebase_wide{2};             // int64 rows beyond 32 bits: 0 64-bit kernel, 1 also re-based per chunk, 2 also common slope removed

namespace {

template <typename T, typename OutT, int OP, int R, bool ATOMIC>
__global__ __launch_bounds__(64) void tropical_kernel(const TropicalArgs p) {
  __shared__ __align__(16) unsigned char lds[lds_bytes<T, R>()];
  tropical_body<T, OutT, OP, R, ATOMIC>(p, lds, blockIdx.x);
}

// The same work for a launch most of whose rows are expected to be handled elsewhere (the 64-bit
// kernel behind the range probe): `parts` workgroups per row, each looks at its row's selector
// once and either leaves or walks every parts-th item of the row (items are numbered rows
// fastest).  A full grid of workgroups that only find out that they have nothing to do costs
// ~15 us of dispatch per call.
template <typename T, typename OutT, int OP, int R>
__global__ __launch_bounds__(64) void tropical_rows_kernel(const TropicalArgs p, uint32_t items_per_row, uint32_t parts) {
  __shared__ __align__(16) unsigned char lds[lds_bytes<T, R>()];
  const uint32_t row = blockIdx.x % (uint32_t)p.batch, part = blockIdx.x / (uint32_t)p.batch;
  if (p.sel != nullptr && p.sel[row] != p.sel_want) return;
  for (uint32_t j = part; j < items_per_row; j += parts)
    tropical_body<T, OutT, OP, R, true>(p, lds, j * (uint32_t)p.batch + row);
}

// One launch for an int32 product with the packed path: the first n_packed workgroups are
// items of the packed kernel, the rest are items of the 32-bit kernel (which skip the chunks
// the packed items own).  Issuing both kinds together keeps the machine full whatever share of
// the chunks qualifies for 16 bits.
// RP = accumulators per lane of the packed items (their tiles are 128 RP outputs wide).
template <typename OutT, int OP, int RP>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(4, 4))) void fused_kernel(const TropicalArgs pk, const TropicalArgs pg,
                                                   uint32_t n_packed) {
  static_assert(lds_bytes<int32_t, RP>() <= lds_bytes<int32_t, kPkR>(), "the 32-bit layout is the larger one");
  __shared__ __align__(16) unsigned char lds[lds_bytes<int32_t, kPkR>()];
  if (blockIdx.x < n_packed) packed_body<OutT, OP, RP>(pk, lds, blockIdx.x);
  else tropical_body<int32_t, OutT, OP, kPkR, true>(pg, lds, blockIdx.x - n_packed);
}

template <typename T> struct RFor { static constexpr int value = 16; };

// Identity of the reduction as a host value (used to pre-fill outputs merged by atomics).
template <typename T, int OP> T host_identity() {
  if (std::numeric_limits<T>::has_infinity)
    return op_max(OP) ? -std::numeric_limits<T>::infinity() : std::numeric_limits<T>::infinity();
  return op_max(OP) ? std::numeric_limits<T>::lowest() : std::numeric_limits<T>::max();
}

struct Plan {
  int n_tiles, fold_width, seg;
  bool atomic;
  int64_t items;
};

// Cut the triangular iteration space (tiles of `width` outputs, chunks of `chunk` steps) into
// about RTC_TARGET_ITEMS work items of equal length.
Plan make_plan(int64_t batch, int64_t n, int width, int chunk) {
  Plan pl;
  pl.n_tiles = (int)((n + width - 1) / width);
  const double total_steps = (double)batch * (double)n * (pl.n_tiles + 1) * 0.5;
  // Measured on MI355X: items shorter than two chunks pay noticeably for their fixed cost
  // (staging, atomics), items much longer than that leave a ragged tail at the end of the launch.
  int64_t seg = (int64_t)(total_steps / (double)RTC_TARGET_ITEMS);
  seg = seg / chunk * chunk;
  if (seg < 2 * chunk) seg = total_steps / (2.0 * chunk) >= 8192.0 ? 2 * chunk : chunk;
  const int64_t span = ((int64_t)pl.n_tiles * width + chunk - 1) / chunk * chunk;  // longest s range, rounded up
  if (seg >= span) seg = span;
  pl.seg = (int)seg;
  auto nseg = [&](int k) { const int64_t e = (int64_t)(k + 1) * width; return (int)(((e < n ? e : n) + seg - 1) / seg); };
  pl.fold_width = 0;
  for (int k_lo = 0; k_lo <= pl.n_tiles - 1 - k_lo; ++k_lo) {
    const int k_hi = pl.n_tiles - 1 - k_lo;
    const int w = nseg(k_hi) + (k_lo != k_hi ? nseg(k_lo) : 0);
    if (w > pl.fold_width) pl.fold_width = w;
  }
  pl.atomic = nseg(pl.n_tiles - 1) > 1;
  pl.items = batch * (int64_t)((pl.n_tiles + 1) / 2) * pl.fold_width;
  return pl;
}

template <typename T, int R> Plan make_plan(int64_t batch, int64_t n) {
  using TL = Tile<T, R>;
  return make_plan(batch, n, TL::kW, TL::kChunk);
}

// Accumulators per lane of the generic kernel: 16, or 4 for problems so small that 16 would give
// fewer work items than the chip has CUs (a single pair of 4096 samples: 10 items of 1024 x 1024
// candidates, 67 us; with tiles of 256 outputs and chunks of 256 steps 136 items that finish in a
// sixth of that, although each candidate costs more instructions).
constexpr int kSmallR = 4;

// Starting value of an output that work items merge into with atomics: the identity of the
// reduction, or, for a min-type product with a fused cap, the cap itself -- an item whose partial
// result still equals the identity skips its merge (it saw no candidate), so an output whose
// every candidate legitimately equals the largest value of the type must already hold
// min(identity, cap) = cap.  (Under a max-type reduction the skipped value is the smallest of the
// type, which a min with the cap leaves as it is.)
template <typename OutT, int OP>
void launch_fill(OutT* out, const OutT* cap, int64_t count, hipStream_t stream) {
  const int64_t want = (count + 2047) / 2048;
  const int blocks = (int)(want < 65535 ? want : 65535);
  if (cap != nullptr && !op_max(OP))
    RTC_LAUNCH(copy_rows_kernel<OutT>, dim3(blocks), dim3(256), 0, stream, cap, out, count);
  else
    RTC_LAUNCH(fill_kernel<OutT>, dim3(blocks), dim3(256), 0, stream, out, count, host_identity<OutT, OP>());
}

// One launch of the generic kernel.  `force_atomic` is set when several kernels contribute to
// one output (the output is then already filled with the identity).
template <typename T, typename OutT, int OP, int R>
int run_product_r(const T* a, int64_t stride_a, const T* b, int64_t stride_b, OutT* out, const OutT* cap,
                  const int32_t* sel, int sel_want, int64_t batch, int64_t n, hipStream_t stream,
                  bool prefilled, bool force_atomic, const int64_t* out_base) {
  const Plan pl = make_plan<T, R>(batch, n);
  if (pl.items > 0x7fffffffLL) return RTC_ERR_SHAPE;
  TropicalArgs args = {};
  args.a = a; args.b = b; args.out = out; args.cap = cap; args.sel = sel;
  args.stride_a = stride_a; args.stride_b = stride_b; args.sel_want = sel_want;
  args.n = (int32_t)n; args.batch = (int32_t)batch;
  args.n_tiles = pl.n_tiles; args.fold_width = pl.fold_width; args.seg = pl.seg;
  args.out_base = out_base;
  constexpr int dtype_code = std::is_same<T, int32_t>::value ? RTC_I32 : std::is_same<T, int64_t>::value ? RTC_I64 : RTC_F64;
  if (pl.atomic || force_atomic) {
    if (!prefilled) launch_fill<OutT, OP>(out, cap, batch * n, stream);
    prof_begin(RTC_PROFILE_KIND(dtype_code, 0, OP), stream, sel != nullptr);
    if (sel != nullptr && sizeof(T) == 8 && pl.items > 8192) {
      const uint32_t items_per_row = (uint32_t)(pl.items / batch);
      uint32_t parts = (uint32_t)(4096 / batch);
      if (parts < 1) parts = 1;
      if (parts > items_per_row) parts = items_per_row;
      RTC_LAUNCH((tropical_rows_kernel<T, OutT, OP, R>), dim3((uint32_t)batch * parts), dim3(64), 0, stream,
                         args, items_per_row, parts);
    } else {
      RTC_LAUNCH((tropical_kernel<T, OutT, OP, R, true>), dim3((uint32_t)pl.items), dim3(64), 0,
                         stream, args);
    }
  } else {
    prof_begin(RTC_PROFILE_KIND(dtype_code, 0, OP), stream);
    RTC_LAUNCH((tropical_kernel<T, OutT, OP, R, false>), dim3((uint32_t)pl.items), dim3(64), 0,
                       stream, args);
  }
  prof_end(stream);
  return hip_ok();
}

template <typename T, typename OutT, int OP>
int run_product(const T* a, int64_t stride_a, const T* b, int64_t stride_b, OutT* out, const OutT* cap,
                const int32_t* sel, int sel_want, int64_t batch, int64_t n, hipStream_t stream,
                bool prefilled, bool force_atomic, const int64_t* out_base) {
  if (make_plan<T, RFor<T>::value>(batch, n).items < g_small_items && n > Tile<T, kSmallR>::kW)
    return run_product_r<T, OutT, OP, kSmallR>(a, stride_a, b, stride_b, out, cap, sel, sel_want, batch, n, stream,
                                               prefilled, force_atomic, out_base);
  return run_product_r<T, OutT, OP, RFor<T>::value>(a, stride_a, b, stride_b, out, cap, sel, sel_want, batch, n,
                                                    stream, prefilled, force_atomic, out_base);
}

// Layout of the packed path's arrays inside the workspace.
struct PackLayout {
  int64_t npad, nchunk, nsub, nblk;
  size_t off_apk, off_apk_s, off_bd, off_ab, off_ar, off_ab_s, off_ar_s, off_bmn, off_bmx, off_rho, off_ok, off_sel, off_jstar, off_period, off_F, off_dbl, bytes;
};

PackLayout pack_layout(int64_t batch, int64_t n) {
  PackLayout L;
  L.nchunk = (n + kPkChunk - 1) / kPkChunk;
  L.npad = L.nchunk * kPkChunk;
  L.nsub = L.nchunk * kPkSubs;
  L.nblk = (n + kPkBlock - 1) / kPkBlock;
  size_t o = 0;
  auto take = [&](size_t elems) { const size_t at = o; o += (elems * 4 + 255) / 256 * 256; return at; };
  L.off_apk = take((size_t)batch * (L.npad + 16));     // rows of npad + 16 words, see prep_kernel
  L.off_apk_s = take((size_t)batch * (L.npad + 16));
  L.off_bd = take((size_t)batch * ((n + 3) & ~(int64_t)3));   // row pitch: a multiple of 16 bytes
  L.off_ab = take((size_t)batch * L.nchunk);
  L.off_ar = take((size_t)batch * L.nchunk);
  L.off_ab_s = take((size_t)batch * L.nsub);
  L.off_ar_s = take((size_t)batch * L.nsub);
  L.off_bmn = take((size_t)batch * L.nblk);
  L.off_bmx = take((size_t)batch * L.nblk);
  L.off_rho = take((size_t)batch);
  L.off_ok = take((size_t)batch);
  L.off_sel = take((size_t)batch);   // per-row selector of int32 products (int64 products keep their own)
  L.off_jstar = take(bracket_jstar_elems(batch, n));   // anchor optima of the bracket path
  L.off_period = take((size_t)batch);                  // period per row of the periodic path
  L.off_F = take((size_t)batch * n * 2);               // its scan F, [batch][n] of the rows' own type
  L.off_dbl = take((size_t)batch * n * 2);             // second fp64 copy of wide int64 rows (the first one shares F)
  L.bytes = o;
  return L;
}

// rtc_product_census: which arithmetic would do how much.  One workgroup per (row, tile of 2048
// outputs), its threads over the chunks of the tile; the unit is one sub-chunk (128 steps) of one
// such tile.  counts: [0] 15-bit flavour on the chunk base, [1] 15-bit flavour on sub-chunk bases,
// [2] 16-bit saturating flavour, [3] 32-bit items, [4] rows that other kernels do.
__global__ __launch_bounds__(64) void census_kernel(PackAux x, const int32_t* __restrict__ sel, int n, int batch,
                                                    int plain_kind, unsigned long long* __restrict__ counts) {
  const int row = blockIdx.x % batch, T2 = blockIdx.x / batch;
  const int s_end = min((T2 + 1) * kPkW, n);
  unsigned long long c[RTC_CENSUS_COUNTS] = {};
  for (int ch = threadIdx.x; ch * kPkChunk < s_end; ch += 64) {
    const int left = s_end - ch * kPkChunk;
    const int valid = min((left + kPkSub - 1) / kPkSub, kPkSubs);
    const int mask = (1 << valid) - 1;
    if (sel != nullptr && sel[row] != 1) { c[4] += valid; continue; }
    if (x.apk == nullptr) { c[plain_kind] += valid; continue; }   // no packed path in this call
    int32_t gb, br;
    const int plan = chunk_plan(x, row, T2, ch, n, &gb, &br);
    const int taken = __builtin_popcount(plan & mask);
    if (plan & kPlanNarrow) c[(plan & kPlanWhole) ? 0 : 1] += taken; else c[2] += taken;
    c[3] += valid - taken;
  }
#pragma unroll
  for (int k = 0; k < RTC_CENSUS_COUNTS; ++k) {
    unsigned long long v = c[k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    if (threadIdx.x == 0 && v != 0) atomicAdd(&counts[k], v);
  }
}

// The census of a product that runs without the packed path: every row (with `sel`: every row
// whose selector is 1) counts under `kind`, the others under [4].
int launch_plain_census(const int32_t* sel, int kind, int64_t batch, int64_t n, unsigned long long* counts,
                        hipStream_t stream) {
  PackAux none = {};
  const int64_t n_t2 = (n + kPkW - 1) / kPkW;
  if (batch * n_t2 > 0x7fffffffLL) return RTC_ERR_SHAPE;
  RTC_LAUNCH(census_kernel, dim3((uint32_t)(batch * n_t2)), dim3(64), 0, stream, none, sel, (int)n, (int)batch,
                     kind, counts);
  return hip_ok();
}

// int32 product with the packed fast path.  f32 / g32 are int32 rows (the caller's own,
// or the narrowed copies of int64 rows); pack_ok / rho were written by the probe and the output
// is already filled with the identity.  `sel` (optional) restricts both kernels to rows with
// sel[row] == 1.
template <typename OutT, int OP>
int run_packed(const int32_t* f32, int64_t stride_f, const int32_t* g32, int64_t stride_g, OutT* out,
               const OutT* cap, const int32_t* sel, const int64_t* out_base, int64_t batch, int64_t n, char* wsp,
               const PackLayout& L, hipStream_t stream, unsigned long long* census) {
  PackAux aux;
  aux.apk = reinterpret_cast<uint32_t*>(wsp + L.off_apk);
  aux.apk_s = reinterpret_cast<uint32_t*>(wsp + L.off_apk_s);
  aux.ab_s = reinterpret_cast<int32_t*>(wsp + L.off_ab_s);
  aux.ar_s = reinterpret_cast<int32_t*>(wsp + L.off_ar_s);
  aux.bd = reinterpret_cast<int32_t*>(wsp + L.off_bd);
  aux.ab = reinterpret_cast<int32_t*>(wsp + L.off_ab);
  aux.ar = reinterpret_cast<int32_t*>(wsp + L.off_ar);
  aux.bmn = reinterpret_cast<int32_t*>(wsp + L.off_bmn);
  aux.bmx = reinterpret_cast<int32_t*>(wsp + L.off_bmx);
  aux.rho = reinterpret_cast<int32_t*>(wsp + L.off_rho);
  aux.pack_ok = reinterpret_cast<int32_t*>(wsp + L.off_ok);
  aux.npad = (int32_t)L.npad; aux.nchunk = (int32_t)L.nchunk; aux.nsub = (int32_t)L.nsub;
  aux.nblk = (int32_t)L.nblk;
  if (batch * L.nchunk > 0x7fffffffLL) return RTC_ERR_SHAPE;
  // uniform operand: f for the convolution, g for the deconvolution; window operand: the other
  RTC_LAUNCH(prep_kernel, dim3((uint32_t)(batch * L.nchunk)), dim3(kPrepThreads), 0, stream,
                     op_sub(OP) ? g32 : f32, op_sub(OP) ? stride_g : stride_f, op_sub(OP) ? f32 : g32,
                     op_sub(OP) ? stride_f : stride_g, (int)n, op_sub(OP), op_sub(OP) != op_max(OP), (int)L.npad, (int)L.nchunk, (int)L.nblk,
                     aux.rho, aux.pack_ok, const_cast<uint32_t*>(aux.apk), const_cast<uint32_t*>(aux.apk_s),
                     const_cast<int32_t*>(aux.ab_s), const_cast<int32_t*>(aux.ar_s), (int)L.nsub,
                     const_cast<int32_t*>(aux.bd), const_cast<int32_t*>(aux.ab), const_cast<int32_t*>(aux.ar),
                     const_cast<int32_t*>(aux.bmn), const_cast<int32_t*>(aux.bmx));
  RTC_LAUNCH(decide_kernel, dim3((uint32_t)batch), dim3(kDecideThreads), 0, stream, aux, (int)n,
                     const_cast<int32_t*>(aux.pack_ok));
  if (census != nullptr) {
    const int64_t n_t2 = (n + kPkW - 1) / kPkW;
    if (batch * n_t2 > 0x7fffffffLL) return RTC_ERR_SHAPE;
    RTC_LAUNCH(census_kernel, dim3((uint32_t)(batch * n_t2)), dim3(64), 0, stream, aux, sel, (int)n, (int)batch,
                       3, census);
    return hip_ok();
  }
  // short rows: tiles of 1024 outputs halve the candidates wasted on the diagonal
  const bool small_tiles = n <= g_packed_small_n;
  const Plan pk = make_plan(batch, n, small_tiles ? kPkW / 2 : kPkW, kPkChunk);
  const Plan pg = make_plan<int32_t, kPkR>(batch, n);
  if (pk.items + pg.items > 0x7fffffffLL) return RTC_ERR_SHAPE;
  TropicalArgs ak = {};
  ak.out = out; ak.cap = cap; ak.sel = sel; ak.sel_want = 1; ak.out_base = out_base;
  ak.n = (int32_t)n; ak.batch = (int32_t)batch;
  ak.n_tiles = pk.n_tiles; ak.fold_width = pk.fold_width; ak.seg = pk.seg;
  ak.use_aux = 1; ak.aux = aux;
  // the 32-bit items work on the caller's rows and skip the chunks owned by the packed items
  TropicalArgs ag = ak;
  ag.a = op_sub(OP) ? g32 : f32; ag.stride_a = op_sub(OP) ? stride_g : stride_f;
  ag.b = op_sub(OP) ? f32 : g32; ag.stride_b = op_sub(OP) ? stride_f : stride_g;
  ag.n_tiles = pg.n_tiles; ag.fold_width = pg.fold_width; ag.seg = pg.seg;
  prof_begin(RTC_PROFILE_KIND(RTC_I32, 1, OP), stream);
  if (small_tiles)
    RTC_LAUNCH((fused_kernel<OutT, OP, kPkR / 2>), dim3((uint32_t)(pk.items + pg.items)), dim3(64), 0,
                       stream, ak, ag, (uint32_t)pk.items);
  else
    RTC_LAUNCH((fused_kernel<OutT, OP, kPkR>), dim3((uint32_t)(pk.items + pg.items)), dim3(64), 0,
                       stream, ak, ag, (uint32_t)pk.items);
  prof_end(stream);
  return hip_ok();
}

}  // namespace

std::atomic<double> g_packed_min_work{(double)RTC_DEFAULT_PACKED_MIN_WORK};   // batch * n^2 from which the packed path is used

namespace {

bool packed_worthwhile(int64_t batch, int64_t n) {
  return (double)batch * (double)n * (double)n >= g_packed_min_work;
}

template <typename T, int OP>
int run_typed(const void* f, const void* g, void* out, int64_t batch, int64_t n, int64_t stride_f,
              int64_t stride_g, const void* cap, void* ws, size_t ws_bytes, int32_t* dev_flags,
              hipStream_t stream, unsigned long long* census) {
  // convolution: uniform operand f, window g.  deconvolution: uniform g, window f (reversed).
  const T* a = static_cast<const T*>(op_sub(OP) ? g : f);
  const T* b = static_cast<const T*>(op_sub(OP) ? f : g);
  const int64_t sa = op_sub(OP) ? stride_g : stride_f;
  const int64_t sb = op_sub(OP) ? stride_f : stride_g;
  if constexpr (std::is_same<T, int32_t>::value) {
    const PackLayout L = pack_layout(batch, n);
    // tiny problems are launch-bound: the extra kernels of the packed path would only cost
    if (ws != nullptr && ws_bytes >= L.bytes && packed_worthwhile(batch, n)) {
      char* wsp = static_cast<char*>(ws);
      int32_t* sel = reinterpret_cast<int32_t*>(wsp + L.off_sel);
      RTC_LAUNCH(probe_kernel<int32_t>, dim3((uint32_t)batch), dim3(1024), 0, stream,
                         static_cast<const int32_t*>(f), stride_f, static_cast<const int32_t*>(g), stride_g,
                         (int)n, g_structure_paths ? OP : OP | kProbeGeneralOnly,
                         reinterpret_cast<int32_t*>(wsp + L.off_ok),
                         reinterpret_cast<int32_t*>(wsp + L.off_rho), sel, dev_flags);
      if (g_structure_paths)
        launch_period<int32_t>(static_cast<const int32_t*>(f), stride_f, static_cast<const int32_t*>(g), stride_g, sel,
                             reinterpret_cast<int32_t*>(wsp + L.off_period),
                             reinterpret_cast<int32_t*>(wsp + L.off_ok), batch, n, OP, stream);
      if (census == nullptr)
        launch_fill<int32_t, OP>(static_cast<int32_t*>(out), static_cast<const int32_t*>(cap), batch * n, stream);
      // general rows (selector 1): packed + 32-bit items; rows of exploitable convexity: structured_kernel
      const int rc = run_packed<int32_t, OP>(static_cast<const int32_t*>(f), stride_f,
                                             static_cast<const int32_t*>(g), stride_g, static_cast<int32_t*>(out),
                                             static_cast<const int32_t*>(cap), sel, nullptr, batch, n, wsp, L,
                                             stream, census);
      if (rc != RTC_OK || !g_structure_paths || census != nullptr) return rc;
      return launch_structured<int32_t, OP>(static_cast<const int32_t*>(f), stride_f,
                                            static_cast<const int32_t*>(g), stride_g, static_cast<int32_t*>(out),
                                            static_cast<const int32_t*>(cap), sel,
                                            reinterpret_cast<int32_t*>(wsp + L.off_jstar),
                                            reinterpret_cast<const int32_t*>(wsp + L.off_period),
                                            reinterpret_cast<int32_t*>(wsp + L.off_F), batch, n, stream);
    }
  }
  // no packed path: the 32-bit kernel (counts[3]), or the fp64 kernel (counts[4]), does every row
  if (census != nullptr)
    return launch_plain_census(nullptr, std::is_same<T, int32_t>::value ? 3 : 4, batch, n, census, stream);
  if (dev_flags != nullptr && std::numeric_limits<T>::is_integer) {
    RTC_LAUNCH(probe_kernel<T>, dim3((uint32_t)batch), dim3(1024), 0, stream,
                       static_cast<const T*>(f), stride_f, static_cast<const T*>(g), stride_g, (int)n,
                       OP, (int32_t*)nullptr, (int32_t*)nullptr, (int32_t*)nullptr, dev_flags);
  }
  return run_product<T, T, OP>(a, sa, b, sb, static_cast<T*>(out), static_cast<const T*>(cap),
                                   nullptr, 0, batch, n, stream, false, false, nullptr);
}

// Bytes of the narrowed copies + selector that precede the packed-path arrays for int64 rows.
size_t narrow_base_offset(int64_t batch, int64_t n) {
  return ((size_t)(2 * batch * n + batch) * sizeof(int32_t) + 255) / 256 * 256;
}
constexpr int kProbeMaxSegs = 16;   // segments per row of the two-pass range probe
size_t narrow_partial_offset(int64_t batch, int64_t n) {
  return narrow_base_offset(batch, n) + ((size_t)batch * 2 * sizeof(int64_t) + 255) / 256 * 256;   // [base, slope] per row
}
size_t narrow_tables_offset(int64_t batch, int64_t n) {
  return narrow_partial_offset(batch, n) + ((size_t)batch * kProbeMaxSegs * kProbePartial * sizeof(int64_t) + 255) / 256 * 256;
}
size_t narrow_bytes(int64_t batch, int64_t n) {
  return narrow_tables_offset(batch, n) + (wide_table_elems(batch, n) * sizeof(int64_t) + 255) / 256 * 256;
}

template <int OP>
int run_i64(const void* f, const void* g, void* out, int64_t batch, int64_t n, int64_t stride_f,
            int64_t stride_g, const void* cap, void* ws, int32_t* dev_flags, hipStream_t stream,
            unsigned long long* census) {
  // workspace: [f32: batch*n][g32: batch*n][narrow_ok: batch][out_base: 2*batch int64][probe partials]
  // [block tables of the re-based path][packed-path arrays]
  int32_t* f32 = static_cast<int32_t*>(ws);
  int32_t* g32 = f32 + batch * n;
  int32_t* ok = g32 + batch * n;
  int64_t* base = reinterpret_cast<int64_t*>(static_cast<char*>(ws) + narrow_base_offset(batch, n));
  char* wsp = static_cast<char*>(ws) + narrow_bytes(batch, n);
  const PackLayout L = pack_layout(batch, n);
  // long rows and few of them: several workgroups per row, extrema in a first pass
  int segs = 1;
  while (segs < kProbeMaxSegs && batch * segs < 512 && n / (2 * segs) >= 4096) segs *= 2;
  int64_t* partial = reinterpret_cast<int64_t*>(static_cast<char*>(ws) + narrow_partial_offset(batch, n));
  const bool structure = packed_worthwhile(batch, n) && g_structure_paths;
  if (segs > 1)
    RTC_LAUNCH(probe_partial_kernel, dim3((uint32_t)(batch * segs)), dim3(1024), 0, stream,
                       static_cast<const int64_t*>(f), stride_f, static_cast<const int64_t*>(g), stride_g, (int)n,
                       structure, segs, partial);
  RTC_LAUNCH(probe_narrow_kernel, dim3((uint32_t)(batch * segs)), dim3(1024), 0, stream,
                     static_cast<const int64_t*>(f), stride_f, static_cast<const int64_t*>(g), stride_g,
                     (int)n, OP, structure, f32, g32, ok, base,
                     reinterpret_cast<int32_t*>(wsp + L.off_ok),
                     reinterpret_cast<int32_t*>(wsp + L.off_rho), dev_flags, segs,
                     segs > 1 ? partial : (const int64_t*)nullptr, g_rebase_wide >= 2);
  if (structure)
    launch_period<int64_t>(static_cast<const int64_t*>(f), stride_f, static_cast<const int64_t*>(g), stride_g, ok,
                           reinterpret_cast<int32_t*>(wsp + L.off_period),
                             reinterpret_cast<int32_t*>(wsp + L.off_ok), batch, n, OP, stream);
  // rows still with the 64-bit kernel (selector 0): those whose values vary slowly enough go to the
  // re-based 32-bit items instead
  int64_t* tab = reinterpret_cast<int64_t*>(static_cast<char*>(ws) + narrow_tables_offset(batch, n));
  const int nb = wide_blocks(n);
  const Plan pw = make_plan<int32_t, kWideR>(batch, n);
  // (not for problems so small that the launches themselves are the cost: their rows stay with
  // the 64-bit kernel, which the same criterion gives small tiles)
  const int64_t small_items = g_small_items;
  const bool small = make_plan<int64_t, RFor<int64_t>::value>(batch, n).items < (small_items < 256 ? small_items : 256);
  const bool rebase = g_rebase_wide >= 1 && n > kWideBlock && pw.items <= 0x7fffffffLL && !small;
  if (rebase) {
    RTC_LAUNCH(wide_tables_kernel<OP>, dim3((uint32_t)batch), dim3(kWideThreads), 0, stream,
                       static_cast<const int64_t*>(f), stride_f, static_cast<const int64_t*>(g), stride_g, ok, tab,
                       tab + (size_t)batch * nb * 4, reinterpret_cast<double*>(wsp + L.off_F),
                       reinterpret_cast<double*>(wsp + L.off_dbl), (int)n, nb, g_rebase_wide >= 2);
  }
  // Several kernels see every row; the selector makes each row run in exactly one family.
  // The output is filled once with the identity, before all of them.
  if (census != nullptr) {   // rows with selector 1: packed + 32-bit items, or 32-bit items alone; the rest: other kernels
    if (packed_worthwhile(batch, n))
      return run_packed<int64_t, OP>(f32, n, g32, n, static_cast<int64_t*>(out), static_cast<const int64_t*>(cap),
                                     ok, base, batch, n, wsp, L, stream, census);
    return launch_plain_census(ok, 3, batch, n, census, stream);
  }
  launch_fill<int64_t, OP>(static_cast<int64_t*>(out), static_cast<const int64_t*>(cap), batch * n, stream);
  int rc;
  if (packed_worthwhile(batch, n)) {
    rc = run_packed<int64_t, OP>(f32, n, g32, n, static_cast<int64_t*>(out), static_cast<const int64_t*>(cap),
                                 ok, base, batch, n, wsp, L, stream, nullptr);
  } else {
    rc = run_product<int32_t, int64_t, OP>(op_sub(OP) ? g32 : f32, n, op_sub(OP) ? f32 : g32, n,
                                           static_cast<int64_t*>(out), static_cast<const int64_t*>(cap), ok, 1,
                                           batch, n, stream, true, true, base);
  }
  if (rc != RTC_OK) return rc;
  const int64_t* a = static_cast<const int64_t*>(op_sub(OP) ? g : f);
  const int64_t* b = static_cast<const int64_t*>(op_sub(OP) ? f : g);
  rc = run_product<int64_t, int64_t, OP>(a, op_sub(OP) ? stride_g : stride_f, b,
                                         op_sub(OP) ? stride_f : stride_g, static_cast<int64_t*>(out),
                                         static_cast<const int64_t*>(cap), ok, 0, batch, n, stream, true, true,
                                         nullptr);
  if (rc != RTC_OK) return rc;
  if (rebase) {
    TropicalArgs args = {};
    args.a = a; args.b = b; args.out = out; args.cap = cap; args.sel = ok; args.sel_want = kSelRebased;
    args.stride_a = op_sub(OP) ? stride_g : stride_f; args.stride_b = op_sub(OP) ? stride_f : stride_g;
    args.n = (int32_t)n; args.batch = (int32_t)batch;
    args.n_tiles = pw.n_tiles; args.fold_width = pw.fold_width; args.seg = pw.seg;
    const uint32_t items_per_row = (uint32_t)(pw.items / batch);
    uint32_t parts = (uint32_t)(4096 / batch);
    if (parts < 1) parts = 1;
    if (parts > items_per_row) parts = items_per_row;
    prof_begin(RTC_PROFILE_KIND(RTC_I64, 0, OP), stream, true);
    RTC_LAUNCH(rebased_rows_kernel<OP>, dim3((uint32_t)batch * parts), dim3(64), 0, stream, args, tab,
                       tab + (size_t)batch * nb * 4, nb, items_per_row, parts);
    prof_end(stream);
    if (int hrc = hip_ok()) return hrc;
    // ... and the pairs within +-2^51 that did not qualify: the fp64 kernel on the double copies
    // (uniform operand a, window operand b, as wide_tables_kernel wrote them)
    rc = run_product<double, int64_t, OP>(reinterpret_cast<const double*>(wsp + L.off_F), n,
                                          reinterpret_cast<const double*>(wsp + L.off_dbl), n,
                                          static_cast<int64_t*>(out), static_cast<const int64_t*>(cap), ok,
                                          kSelDouble, batch, n, stream, true, true, nullptr);
    if (rc != RTC_OK) return rc;
  }
  if (!structure) return RTC_OK;
  // rows of exploitable convexity (selector 2 / 3), on the caller's own 64-bit rows
  return launch_structured<int64_t, OP>(static_cast<const int64_t*>(f), stride_f,
                                        static_cast<const int64_t*>(g), stride_g, static_cast<int64_t*>(out),
                                        static_cast<const int64_t*>(cap), ok,
                                        reinterpret_cast<int32_t*>(wsp + L.off_jstar),
                                        reinterpret_cast<const int32_t*>(wsp + L.off_period),
                                        reinterpret_cast<int64_t*>(wsp + L.off_F), batch, n, stream);
}

}  // namespace

size_t tropical_workspace_bytes(int64_t batch, int64_t n, int dt) {
  if (dt == RTC_I64) return narrow_bytes(batch, n) + pack_layout(batch, n).bytes;
  if (dt == RTC_I32) return pack_layout(batch, n).bytes;
  return 0;
}

namespace {

// see rtc_selftest_half_minmax: one thread per pattern x, 4096 partner pairs (y, z) each
__global__ __launch_bounds__(256) void selftest_half_minmax_kernel(uint32_t* __restrict__ mismatches) {
  const uint32_t x = blockIdx.x * 256 + threadIdx.x;
  if (x >= 0x7C00u) return;
  uint32_t bad = 0;
  for (uint32_t j = 0; j < 4096; ++j) {
    uint32_t y = (x * 2654435761u + j * 40503u) % 0x7C00u;
    uint32_t z = (x * 40503u + j * 2654435761u + 77u) % 0x7C00u;
    if (j == 0) { y = x; z = x; }
    if (j == 1) { y = 0; z = 0x7BFF; }
    if (j == 2) { y = x ? x - 1 : 0; z = x < 0x7BFF ? x + 1 : x; }
    const hf2 a = __builtin_bit_cast(hf2, x | (y << 16)), b = __builtin_bit_cast(hf2, y | (z << 16)),
              c = __builtin_bit_cast(hf2, z | (x << 16));
    const uint32_t mn = __builtin_bit_cast(uint32_t, __builtin_elementwise_minimum(__builtin_elementwise_minimum(a, b), c));
    const uint32_t mx = __builtin_bit_cast(uint32_t, __builtin_elementwise_maximum(__builtin_elementwise_maximum(a, b), c));
    const uint32_t lo = min(min(x, y), z), hi = max(max(x, y), z);
    bad += (mn != (lo | (lo << 16))) + (mx != (hi | (hi << 16)));
  }
  if (bad != 0) atomicAdd(mismatches, bad);
}

}  // namespace

int launch_selftest_half_minmax(uint32_t* mismatches, hipStream_t stream) {
  RTC_LAUNCH(selftest_half_minmax_kernel, dim3(0x7C00 / 256), dim3(256), 0, stream, mismatches);
  return hip_ok();
}

int launch_structure_probe(int op, const void* f, const void* g, int32_t* codes, int32_t* periods, int64_t batch,
                           int64_t n, int64_t stride_f, int64_t stride_g, int dt, hipStream_t stream) {
  static_assert(kSelSearch == RTC_STRUCTURE_BISECT && kSelEnds == RTC_STRUCTURE_ENDS &&
                    kSelBracket == RTC_STRUCTURE_BRACKET && kSelBracketSwapped == RTC_STRUCTURE_BRACKET_SWAPPED &&
                    kSelPeriodic == RTC_STRUCTURE_PERIODIC && kSelPeriodicSwapped == RTC_STRUCTURE_PERIODIC_SWAPPED,
                "selector codes are public");
  const int code_op = op == RTC_OP_CONV ? 0 : op == RTC_OP_DECONV ? 1 : op == RTC_OP_MAXCONV ? 2 : 3;
  if (periods != nullptr) {       // period_kernel writes the rows it accepts only
    const int blocks = (int)((batch + 255) / 256 < 65535 ? (batch + 255) / 256 : 65535);
    RTC_LAUNCH(fill_kernel<int32_t>, dim3(blocks), dim3(256), 0, stream, periods, batch, (int32_t)0);
  }
  if (dt == RTC_I32) {
    RTC_LAUNCH(probe_kernel<int32_t>, dim3((uint32_t)batch), dim3(1024), 0, stream,
                       static_cast<const int32_t*>(f), stride_f, static_cast<const int32_t*>(g), stride_g, (int)n,
                       code_op, (int32_t*)nullptr, (int32_t*)nullptr, codes, (int32_t*)nullptr);
    launch_period<int32_t>(static_cast<const int32_t*>(f), stride_f, static_cast<const int32_t*>(g), stride_g, codes,
                           periods, nullptr, batch, n, code_op, stream);
  } else if (dt == RTC_I64) {
    RTC_LAUNCH(probe_kernel<int64_t>, dim3((uint32_t)batch), dim3(1024), 0, stream,
                       static_cast<const int64_t*>(f), stride_f, static_cast<const int64_t*>(g), stride_g, (int)n,
                       code_op, (int32_t*)nullptr, (int32_t*)nullptr, codes, (int32_t*)nullptr);
    launch_period<int64_t>(static_cast<const int64_t*>(f), stride_f, static_cast<const int64_t*>(g), stride_g, codes,
                           periods, nullptr, batch, n, code_op, stream);
  } else {
    const int blocks = (int)((batch + 255) / 256 < 65535 ? (batch + 255) / 256 : 65535);
    RTC_LAUNCH(fill_kernel<int32_t>, dim3(blocks), dim3(256), 0, stream, codes, batch,
                       (int32_t)RTC_STRUCTURE_GENERAL);
  }
  return hip_ok();
}

int launch_tropical(int op, const void* f, const void* g, void* out, int64_t batch, int64_t n,
                    int64_t stride_f, int64_t stride_g, int dt, const void* cap, void* ws,
                    size_t ws_bytes, int32_t* dev_flags, hipStream_t stream, unsigned long long* census) {
  if (dt == RTC_I64 && (ws == nullptr || ws_bytes < tropical_workspace_bytes(batch, n, dt)))
    return RTC_ERR_WORKSPACE;
#define RTC_BY_OP(CALL)                                  \
  switch (op) {                                          \
    case RTC_OP_CONV: { constexpr int OP = 0; return CALL; }     \
    case RTC_OP_DECONV: { constexpr int OP = 1; return CALL; }   \
    case RTC_OP_MAXCONV: { constexpr int OP = 2; return CALL; }  \
    case RTC_OP_MINDECONV: { constexpr int OP = 3; return CALL; }\
    default: return RTC_ERR_MODE;                        \
  }
  switch (dt) {
    case RTC_I32:
      RTC_BY_OP((run_typed<int32_t, OP>(f, g, out, batch, n, stride_f, stride_g, cap, ws, ws_bytes, dev_flags, stream, census)))
    case RTC_F64:
      RTC_BY_OP((run_typed<double, OP>(f, g, out, batch, n, stride_f, stride_g, cap, ws, ws_bytes, dev_flags, stream, census)))
    case RTC_I64:
      RTC_BY_OP((run_i64<OP>(f, g, out, batch, n, stride_f, stride_g, cap, ws, dev_flags, stream, census)))
    default:
      return RTC_ERR_DTYPE;
  }
#undef RTC_BY_OP
}

}  // namespace rtc
