/* librtc -- (min,+) curve algebra of real-time calculus on AMD MI355X (gfx950).
 *
 * Curves are the sampled nondecreasing functions over Delta = 0..n-1 that the paper's
 * notation preamble names: arrival curves alpha^u / alpha^l, service curves beta^u /
 * beta^l, workload curves gamma^u / gamma^l and their pseudo-inverses (the curve macros
 * of the preamble).  The paper only supplies the symbols; each entry point below states
 * the textbook definition it evaluates.
 *
 * Conventions common to every call
 *   - All data pointers are DEVICE pointers (HBM).  The caller owns every buffer; the
 *     library never allocates, frees or retains device memory.
 *   - A batch is `batch` independent rows; a row is `n` contiguous samples.  Where a
 *     stride is given it is in ELEMENTS and is either 0 (one curve shared by all rows)
 *     or >= n.  Outputs are always dense [batch][n].
 *   - `hip_stream` is a hipStream_t passed as void*.  Every call only enqueues work on
 *     that stream and returns; there is no internal synchronisation.
 *   - Outputs must not alias inputs or the workspace.
 *   - Return value: RTC_OK, or a negative rtc_status.  Every status but RTC_ERR_HIP is decided on
 *     the host before the first kernel of the call is enqueued -- argument checks, and a dry run
 *     of the call's whole launch sequence, which turns a launch the runtime would not accept
 *     (more than 2^32 - 1 threads in one grid) into RTC_ERR_SHAPE: on such a status nothing was
 *     launched and no output byte changed.  RTC_ERR_HIP means that the runtime refused a launch
 *     while enqueueing; kernels of the same call enqueued before it still run.
 *     Data-dependent conditions are not errors: they set bits in the optional caller-provided
 *     device word `dev_flags` (never cleared by the library).
 *   - Host threads: calls from different host threads on different streams are independent
 *     (the library keeps no per-call state outside the caller's buffers).  The planner knobs
 *     (rtc_set_*) are process-wide values that every call reads once per launch decision; set
 *     them while no call is in progress.  rtc_profile_* serialises on a lock of its own and
 *     describes the calls of all threads together.
 *   - Integer arithmetic must not overflow: the caller guarantees that every candidate
 *     f[s]+g[t-s] (convolution) or f[t+u]-g[u] (deconvolution) fits the element type.
 *     With `dev_flags` non-NULL the library checks max+max / min-min style bounds of
 *     the two rows and sets RTC_FLAG_OVERFLOW when they do not prove it.
 *   - fp64 inputs must be finite and must not contain -0.0; results are then bit-exact
 *     (each candidate is a single rounded add or subtract, selection is exact).
 */
#ifndef RTC_H
#define RTC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { RTC_I32 = 0, RTC_I64 = 1, RTC_F64 = 2 } rtc_dtype;
typedef enum { RTC_INV_LOWER = 0, RTC_INV_UPPER = 1 } rtc_inv_mode;
typedef enum {
  RTC_OP_CONV = 0, RTC_OP_DECONV = 1, RTC_OP_GPC = 2, RTC_OP_MAXCONV = 3, RTC_OP_MINDECONV = 4,
  RTC_OP_CLOSURE = 5, RTC_OP_CHAIN = 6
} rtc_op;

typedef enum {
  RTC_OK = 0,
  RTC_ERR_NULL = -1,      /* a required pointer is NULL */
  RTC_ERR_SHAPE = -2,     /* batch < 1, n < 1, n > RTC_MAX_N, or some launch of the call would exceed the grid limit */
  RTC_ERR_DTYPE = -3,     /* unknown rtc_dtype */
  RTC_ERR_ALIGN = -4,     /* a pointer is not aligned to its element size */
  RTC_ERR_STRIDE = -5,    /* a stride is neither 0 nor >= n */
  RTC_ERR_WORKSPACE = -6, /* workspace missing or smaller than rtc_workspace_bytes() */
  RTC_ERR_HIP = -7,       /* the HIP runtime reported an error while enqueueing */
  RTC_ERR_MODE = -8       /* unknown rtc_inv_mode / rtc_op */
} rtc_status;

#define RTC_MAX_N (1 << 24)

#define RTC_FLAG_OVERFLOW 1  /* integer range precondition not provable from the rows' min/max */
#define RTC_FLAG_DOMAIN 2    /* rtc_compose: an index was outside [0, n_outer-1] and was clamped */
#define RTC_FLAG_UNBOUNDED 4 /* rtc_max_hdev: some alpha[D] is never reached by beta within the horizon */
#define RTC_FLAG_NOT_MONOTONE 8 /* rtc_validate_monotone: some row decreases somewhere */

/* Min-plus convolution, out[b][t] = min_{0<=s<=t} f[b][s] + g[b][t-s], t = 0..n-1.
 * Truncated horizon: samples beyond n-1 do not exist, the output has n samples.
 * f, g: [batch] rows with element strides stride_f / stride_g.  out: [batch][n].
 * ws / ws_bytes: device scratch, rtc_workspace_bytes(RTC_OP_CONV, ...) bytes.
 *   RTC_F64 needs none.  RTC_I64 requires it: the rows are probed and, when the value range
 *   (max - min) of each of the two rows is below 2^30, re-based to their minima, convolved in
 *   32-bit arithmetic on narrowed copies -- exact, because every candidate then fits -- and
 *   widened and shifted back on store; other rows take the 64-bit kernel.
 *   For RTC_I32 it is optional: with a workspace of the full size the library also uses its
 *   packed 16-bit kernel on every (tile, chunk of 1024 steps) whose detrended value ranges fit
 *   16 bits (same exact results, up to 2.6x faster where they fit 15); with ws == NULL or a
 *   smaller size only the 32-bit kernel runs.  The packed kernel applies to int64 rows narrowed as above, too.
 * Exact: there is one correct bit pattern per output (values only, no argmin). */
int rtc_minplus_conv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                     int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes,
                     int32_t* dev_flags, void* hip_stream);

/* Max-plus deconvolution on the finite horizon,
 * out[b][t] = max_{0<=u<=n-1-t} f[b][t+u] - g[b][u]: only pairs whose two samples exist.
 * (This under-approximates the infinite-horizon supremum near the end of the horizon.)
 * Arguments as for rtc_minplus_conv; results may be negative. */
int rtc_maxplus_deconv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                       int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes,
                       int32_t* dev_flags, void* hip_stream);

/* The two dual products (max-plus algebra), same arguments, workspace rules and exactness:
 *   rtc_maxplus_conv     out[b][t] = max_{0<=s<=t}     f[b][s]   + g[b][t-s]
 *   rtc_minplus_deconv   out[b][t] = min_{0<=u<=n-1-t} f[b][t+u] - g[b][u]
 * They are what the upper-service / lower-arrival side of a greedy processing component is
 * written with ((beta^u - alpha^l) max-plus-deconvolved by 0, and so on); with g = 0 they
 * reduce to a running maximum and a suffix minimum. */
int rtc_maxplus_conv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                     int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes,
                     int32_t* dev_flags, void* hip_stream);
int rtc_minplus_deconv(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                       int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes,
                       int32_t* dev_flags, void* hip_stream);

/* Pseudo-inverse of a nondecreasing sampled curve (e.g. gamma^{u-1}), per query x[b][j]:
 *   RTC_INV_LOWER: min{k in [0,n) : f[b][k] >= x}, or n when there is none; a plateau
 *                  returns its first index; f[inv(x)] >= x holds whenever inv(x) < n.
 *   RTC_INV_UPPER: max{k in [0,n) : f[b][k] <= x}, or -1 when there is none; a plateau
 *                  returns its last index; f[inv(x)] <= x holds whenever inv(x) >= 0.
 * f: [batch][n] (must be nondecreasing, unchecked), x: [batch][m] of the same dtype,
 * out_idx: int32 [batch][m]. */
int rtc_pseudo_inverse(const void* f, int64_t n, const void* x, int64_t m, int32_t* out_idx,
                       int64_t batch, rtc_inv_mode mode, rtc_dtype dt, void* hip_stream);

/* Composition of a workload curve with an event-count curve,
 * out[b][D] = outer[b][ clamp(inner[b][D], 0, n_outer-1) ]  (e.g. gamma^u o alpha-bar^u).
 * outer: [batch][n_outer] of dtype dt, inner: int32 [batch][n], out: [batch][n] of dtype dt.
 * A clamped index sets RTC_FLAG_DOMAIN in dev_flags (optional). */
int rtc_compose(const void* outer, int64_t n_outer, const int32_t* inner, int64_t n, void* out,
                int64_t batch, rtc_dtype dt, int32_t* dev_flags, void* hip_stream);

/* One greedy processing component, per row.  Upper-arrival / lower-service side (always):
 *   alpha_u_out = min( (alpha_u (x) beta_u) (/) beta_l , beta_u )
 *   beta_l_out[D] = max(0, max_{l<=D} beta_l[l] - alpha_u[l])
 * and, when gamma_u is given, the event-domain images of beta_l_out,
 *   events_lower / events_upper = lower / upper pseudo-inverse of gamma_u at beta_l_out.
 * Lower-arrival / upper-service side (when alpha_l is given; alpha_l_out and beta_u_out are
 * then required):
 *   alpha_l_out = min( (alpha_l (/) beta_u) (x) beta_l , beta_l )
 *   beta_u_out[D] = max(0, min_{l>=D} beta_u[l] - alpha_l[l])
 * and, when gamma_l is given, events_u_lower / events_u_upper = lower / upper pseudo-inverse
 * of gamma_l at beta_u_out.  (x) is the min-plus convolution, (/) the max-plus deconvolution
 * on the finite horizon, as defined above.
 * All curve pointers are dense [batch][n] of dtype dt (gamma_u: [batch][n_gamma], gamma_l:
 * [batch][n_gamma_l]).  Optional members may be NULL; zero-initialise the struct.
 * ws needs rtc_workspace_bytes(RTC_OP_GPC, ...). */
typedef struct rtc_gpc_args {
  const void* alpha_u;
  const void* beta_u;
  const void* beta_l;
  void* alpha_u_out;
  void* beta_l_out;
  const void* gamma_u;    /* optional */
  int64_t n_gamma;
  int32_t* events_lower;  /* optional, int32 [batch][n], needs gamma_u */
  int32_t* events_upper;  /* optional, int32 [batch][n], needs gamma_u */
  int64_t batch;
  int64_t n;
  rtc_dtype dt;
  void* ws;
  size_t ws_bytes;
  int32_t* dev_flags;     /* optional */
  const void* alpha_l;    /* optional: enables the lower-arrival / upper-service side */
  void* alpha_l_out;
  void* beta_u_out;
  const void* gamma_l;    /* optional */
  int64_t n_gamma_l;
  int32_t* events_u_lower; /* optional, int32 [batch][n], needs gamma_l */
  int32_t* events_u_upper; /* optional, int32 [batch][n], needs gamma_l */
} rtc_gpc_args;

int rtc_gpc_step(const rtc_gpc_args* a, void* hip_stream);

/* Sub-additive closure on the finite horizon, per row:
 *   out = min(delta_0, f, f (x) f, f (x) f (x) f, ...),  delta_0[0] = 0 and +infinity elsewhere,
 * i.e. out[0] = 0 and out[t] = the cheapest way to split t into positive parts priced by f.
 * Needs f[0] >= 0 (a row with f[0] < 0 has no finite closure: RTC_FLAG_DOMAIN is raised and the
 * row is treated as if f[0] were 0).  Computed by ceil(log2(n-1)) squarings g <- g (x) g starting
 * from g = f with g[0] = 0.  rtc_superadditive_closure is the max-plus dual
 * (max instead of min, rtc_maxplus_conv, needs f[0] <= 0).
 * RTC_F64: a k-fold sum depends on the order of its additions, so the powers are formed as the
 * definition writes them, one factor at a time from the left (h <- h (x) g, n - 2 products: cubic
 * in n, meant for short rows); since g[0] = 0 every power lies at or below the one before it, and
 * the last one is the closure.  Bit for bit the minimum over the powers so formed.
 * f, out: dense [batch][n]; ws needs rtc_workspace_bytes(RTC_OP_CLOSURE, ...). */
int rtc_subadditive_closure(const void* f, void* out, int64_t batch, int64_t n, rtc_dtype dt, void* ws,
                            size_t ws_bytes, int32_t* dev_flags, void* hip_stream);
int rtc_superadditive_closure(const void* f, void* out, int64_t batch, int64_t n, rtc_dtype dt, void* ws,
                              size_t ws_bytes, int32_t* dev_flags, void* hip_stream);

/* Concatenation of `count` curves per row (e.g. the service curves along a path, whose min-plus
 * convolution is the service the path offers end to end):
 *   out = curves[0] (x) curves[1] (x) ... (x) curves[count-1]
 * evaluated left to right (for RTC_F64 this fixes the rounding of every sum).
 * curves: dense [count][batch][n]; out: [batch][n]; 1 <= count <= 65536;
 * ws needs rtc_workspace_bytes(RTC_OP_CHAIN, ...). */
int rtc_conv_chain(const void* curves, int64_t count, void* out, int64_t batch, int64_t n, rtc_dtype dt,
                   void* ws, size_t ws_bytes, int32_t* dev_flags, void* hip_stream);

/* Delay bound: maximal horizontal deviation per row,
 *   out[b] = max_D max(0, min{k : beta[b][k] >= alpha[b][D]} - D);
 * an alpha[D] that beta never reaches inside the horizon contributes n - D and sets
 * RTC_FLAG_UNBOUNDED.  alpha, beta: [batch][n] nondecreasing; out: int32 [batch]. */
int rtc_max_hdev(const void* alpha, const void* beta, int32_t* out, int64_t batch, int64_t n,
                 rtc_dtype dt, int32_t* dev_flags, void* hip_stream);

/* Backlog bound: maximal vertical deviation per row, out[b] = max_D alpha[b][D] - beta[b][D]
 * (equal to (alpha (/) beta)[0]).  out: [batch] of dtype dt. */
int rtc_max_vdev(const void* alpha, const void* beta, void* out, int64_t batch, int64_t n,
                 rtc_dtype dt, void* hip_stream);

/* Both bounds from one pass over alpha and beta: out_h as rtc_max_hdev, out_v as rtc_max_vdev
 * (same definitions, flags and results; alpha is read once instead of twice). */
int rtc_max_deviations(const void* alpha, const void* beta, int32_t* out_h, void* out_v, int64_t batch, int64_t n,
                       rtc_dtype dt, int32_t* dev_flags, void* hip_stream);

/* Debug aid: the pseudo-inverse, the composition's inner curve, the deviations and the component
 * step take nondecreasing rows and do not check it.  This does: RTC_FLAG_NOT_MONOTONE is raised in
 * dev_flags (required) when some f[b][i+1] < f[b][i], and first_bad[b] (optional; device, [batch]
 * int32) receives the smallest such i, or -1 for a nondecreasing row.  f: [batch][n], row stride
 * `stride` elements (0 = one row for every b). */
int rtc_validate_monotone(const void* f, int64_t batch, int64_t n, int64_t stride, rtc_dtype dt,
                          int32_t* first_bad, int32_t* dev_flags, void* hip_stream);

/* Which kernel family the four products give a row pair (integer dtypes; fp64 rows are always
 * RTC_STRUCTURE_GENERAL).  With c(j) the candidates of one output (f[j] + g[t-j] for the
 * convolutions, f[t+j] - g[j] for the deconvolutions), a pair of convex / concave rows makes c a
 * convex or concave sequence, and the reduction needs no full scan:
 *   RTC_STRUCTURE_ENDS    min over a concave / max over a convex sequence: one of its two ends
 *   RTC_STRUCTURE_BISECT  min over a convex / max over a concave sequence: bisection on the sign
 *                         of c(j+1) - c(j)
 * (convolutions: f and g both convex, or both concave; deconvolutions: f convex and g concave,
 * or f concave and g convex; linear rows count as both).  With only one operand of the right
 * shape -- g (RTC_STRUCTURE_BRACKET) or f (RTC_STRUCTURE_BRACKET_SWAPPED) convex under the
 * min-plus convolution, concave under the max-plus one; f concave under the max-plus
 * deconvolution, convex under the min-plus one; the other operand arbitrary, e.g. any arrival
 * curve against a rate-latency service curve -- the optimal j still moves monotonically with
 * t: every 4096th output is scanned in full, every 64th between the optima of those, and the
 * outputs in between only between their neighbours' optima, about n^2/8192 + 128 n candidates
 * instead of n^2/2.
 * Pairs without such convexity are looked at for periodicity: a row w is periodic from index 1
 * on when w[i+p] = w[i] + c for all 1 <= i <= n-1-p (event streams with jitter, TDMA service;
 * index 0 is left out because such curves are 0 there), with a period p <= min(1024, n/16).
 * RTC_STRUCTURE_PERIODIC: g is (its smallest such period is used); RTC_STRUCTURE_PERIODIC_SWAPPED
 * (convolutions only): f is, and g is not or has a longer period that exceeds the length up to
 * which periods are multiplied anyway (between 32 and 256, about sqrt(1.2e6 / batch)).  Grouping the candidates by residue class of j turns the product into
 * one scan along each class of the other operand plus a window of p candidates per output,
 * n p candidates instead of n^2/2.  Not taken when the other row's range plus w's would leave
 * the type.  The search tests each period at 128 consecutive and a few spread positions first
 * and fully verifies at most four survivors per row, so a contrived row can escape it (and takes
 * the general kernels); a row it accepts is periodic.
 * The products detect all this on the device and compute such pairs with the same result bit
 * for bit, when a workspace is given, the problem is above the rtc_set_packed_min_work
 * threshold and rtc_set_structure_paths is on.
 * rtc_product_structure reports the classification: codes[b] for row pair b, op = RTC_OP_CONV,
 * _DECONV, _MAXCONV or _MINDECONV.  codes: device, [batch] int32. */
enum {
  RTC_STRUCTURE_GENERAL = 1, RTC_STRUCTURE_BISECT = 2, RTC_STRUCTURE_ENDS = 3, RTC_STRUCTURE_BRACKET = 4,
  RTC_STRUCTURE_BRACKET_SWAPPED = 5, RTC_STRUCTURE_PERIODIC = 6, RTC_STRUCTURE_PERIODIC_SWAPPED = 7
};
int rtc_product_structure(int op, const void* f, const void* g, int32_t* codes, int64_t batch, int64_t n,
                          int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* hip_stream);

/* rtc_product_structure, and in periods[b] (optional; device, [batch] int32) the window length
 * the periodic path uses for row pair b: a multiple of the period found, 0 for a pair that is
 * not RTC_STRUCTURE_PERIODIC(_SWAPPED).  Such a pair costs about n (periods[b] + 1) candidates
 * plus one scan of n steps. */
int rtc_product_periods(int op, const void* f, const void* g, int32_t* codes, int32_t* periods, int64_t batch,
                        int64_t n, int64_t stride_f, int64_t stride_g, rtc_dtype dt, void* hip_stream);

/* Measurement aid: how the iteration space of a product splits over the arithmetic flavours of
 * its kernels.  Takes the arguments of the product `op` (RTC_OP_CONV, _DECONV, _MAXCONV,
 * _MINDECONV) without `out`, classifies and prepares the rows in the workspace exactly as the
 * product would, and instead of computing it ADDS to the device array counts[RTC_CENSUS_COUNTS]
 * (the caller zeroes it) the number of units each flavour would take; a unit is one sub-chunk of
 * 128 steps of one tile of 2048 outputs (the diagonal's half-empty units count in full):
 *   counts[0]  15-bit packed flavour on the chunk's base     (0.5 VALU instructions per pair-op:
 *   counts[1]  15-bit packed flavour on sub-chunk bases       one 64-bit add + one packed min3 per four)
 *   counts[2]  16-bit saturating packed flavour               (1 per pair-op)
 *   counts[3]  32-bit work items                              (1.5 per pair-op)
 *   counts[4]  rows that other kernels do (64-bit, fp64, structure-exploiting paths)
 * so that a benchmark can price a launch against the instruction-issue ceiling of the mix it
 * actually ran. */
#define RTC_CENSUS_COUNTS 5
int rtc_product_census(int op, const void* f, const void* g, int64_t batch, int64_t n, int64_t stride_f,
                       int64_t stride_g, rtc_dtype dt, void* ws, size_t ws_bytes, uint64_t* counts,
                       void* hip_stream);

/* Planner knob: the packed 16-bit path of the int32 / narrowed-int64 products, and with it the
 * detection of convex, concave and periodic rows, is used when a workspace is present and
 * batch * n^2 >= this value (default RTC_DEFAULT_PACKED_MIN_WORK = 2^33, the measured break-even
 * on MI355X: below it the probes and preparation kernels cost more than the faster kernel
 * gains, and the 32-bit kernel alone is quicker).  0 uses it for every size.  Results do not
 * depend on it.  Process-wide. */
#define RTC_DEFAULT_PACKED_MIN_WORK 8589934592
int rtc_set_packed_min_work(double batch_times_n_squared);

/* Planner knob: rows of at most this many samples give the packed work items tiles of 1024
 * outputs instead of 2048 (fewer candidates wasted on the half-empty diagonal of a tile, more
 * loop overhead per candidate; default 4096, measured).  0 never does, a value >= RTC_MAX_N always does.  Results do not
 * depend on it.  Process-wide.  RTC_ERR_SHAPE for a negative value. */
int rtc_set_packed_small_n(int64_t n);

/* Planner knob: a product that the general kernel would cut into fewer work items than this
 * (default RTC_DEFAULT_SMALL_PROBLEM_ITEMS = 8192, eight wavefronts per SIMD of the chip, measured:
 * one pair of 4096 samples gives 10, one of 65536 gives 2080) runs with tiles of 256 outputs and
 * chunks of 256 steps instead of 1024 x 1024, which costs more instructions per candidate and
 * finishes sooner because more CUs take part and more wavefronts hide each other's waits.  0 never
 * does.  Results do not depend on it.  Process-wide.  RTC_ERR_SHAPE for a negative
 * value. */
#define RTC_DEFAULT_SMALL_PROBLEM_ITEMS 8192
int rtc_set_small_problem_items(int64_t items);

/* Planner knob for int64 row pairs whose values span 2^30 or more (too wide to be narrowed to
 * 32 bits by subtracting the row minima).  mode 2 (default): a pair that stays within 2^30 of a
 * line -- both rows minus i times the pair's common slope, half the sum of their mean slopes --
 * is narrowed with the slope removed and takes the 32-bit and packed kernels at their full rate
 * (cumulative curves in nanoseconds or cycles are of this kind); otherwise a pair that, minus the
 * same slope, varies slowly -- for every chunk of 1024 steps and window of 2048 samples,
 * range(chunk of one row) + range(window of the other) <= 2^31 - 2 -- runs in 32-bit arithmetic
 * on values re-based per chunk, about 2.5 times as fast as the 64-bit kernel; of the rest, pairs
 * whose values all lie within +-2^51 run in fp64 arithmetic, which is exact on such integers
 * (about 1.8 times as fast), and only the others in the 64-bit integer kernel.  mode 1: without
 * any slope removed; mode 0: the 64-bit integer kernel for every pair that spans 2^30 or more.  Results do not depend on it.  Process-wide.  RTC_ERR_MODE for other values. */
int rtc_set_rebase_wide(int mode);

/* Planner knob: 0 sends every row pair of the integer products through the general kernels,
 * whatever its convexity or periodicity (rtc_product_structure still reports what it finds);
 * non-zero (default) lets the structure-exploiting paths take the rows they recognise.  Results
 * do not depend on it.  Process-wide. */
int rtc_set_structure_paths(int enabled);

/* rtc_minplus_conv for callers that cannot allocate device memory: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * status codes as rtc_minplus_conv, without ws / ws_bytes: the workspace is a device array of
 * RTC_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs on holds it until the
 * process ends), and the call allocates and frees nothing.  A shape whose
 * rtc_workspace_bytes(RTC_OP_CONV, batch, n, dt) exceeds RTC_STATIC_SCRATCH_BYTES returns
 * RTC_ERR_WORKSPACE and launches nothing (int32: batch * n up to about 1.1 million samples,
 * int64: about 0.9 million; fp64 needs no workspace and is never refused for it).
 * All calls on one GPU share that array: calls that overlap in time on one GPU (different streams,
 * or different host threads) race and give undefined results; calls ordered on one stream are safe.
 * Nothing in the array has to be cleared between calls. */
#define RTC_STATIC_SCRATCH_BYTES (32 << 20)
int rtc_minplus_conv_static(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                            int64_t stride_f, int64_t stride_g, rtc_dtype dt, int32_t* dev_flags,
                            void* hip_stream);

/* Bytes of device workspace an operator needs for the given shape (0 on invalid input). */
size_t rtc_workspace_bytes(int op, int64_t batch, int64_t n, rtc_dtype dt);

/* Static description of a status code. */
const char* rtc_strerror(int status);

/* Properties of the current HIP device that the VALU roofline is derived from:
 * compute-unit count, nominal engine clock in kHz, LDS bytes per workgroup.
 * Any pointer may be NULL.  Host pointers. */
int rtc_device_info(int* cu_count, int* clock_khz, int* lds_bytes);

/* Device self-test of the arithmetic identity that the 15-bit flavour of the packed product
 * kernels rests on: for 16-bit patterns below 0x7C00 the packed three-operand half-float minimum /
 * maximum equals the integer minimum / maximum of the patterns (denormal patterns included).
 * Checks every pattern x in [0, 0x7C00) against 4096 partner pairs each (equal values, the range
 * ends, neighbours and a hash of the rest) and ADDS the number of mismatches to the device word
 * *mismatches (the caller zeroes it).  0 is the only acceptable outcome. */
int rtc_selftest_half_minmax(uint32_t* mismatches, void* hip_stream);

/* Measurement aid (not part of the curve algebra).  While enabled, every product kernel that
 * rtc_minplus_conv / rtc_maxplus_deconv / rtc_gpc_step launch is bracketed by a HIP event pair
 * on the call's stream (up to 1024 kernels; helper kernels such as probes and fills are not
 * recorded).  rtc_profile_enable(1) clears the record and starts, rtc_profile_enable(0) stops;
 * rtc_profile_enable(2) also records the launches that sit behind a per-row selector and may find
 * no row of their kind (the 64-bit, re-based and fp64-on-integers kernels of an int64 product),
 * which level 1 leaves out because every recorded launch costs about 10 us of idle stream.
 * rtc_profile_read waits for the recorded kernels and writes up to max_entries (kind, duration
 * in milliseconds) pairs to the HOST arrays kinds / ms; it returns the number written or a
 * negative status.  kind = RTC_PROFILE_KIND(dtype of the arithmetic, packed 16-bit kernel?,
 * product), product = 0 min-plus convolution, 1 max-plus deconvolution, 2 max-plus convolution,
 * 3 min-plus deconvolution.  One record for the whole process, serialised by a lock. */
#define RTC_PROFILE_KIND(dtype, packed, product) ((dtype) * 8 + (packed) * 4 + (product))
#define RTC_PROFILE_KIND_TAIL 64   /* the scan (+ event-domain inverses) kernel of rtc_gpc_step */
int rtc_profile_enable(int on);
int rtc_profile_read(int max_entries, int* kinds, float* ms);

#ifdef __cplusplus
}
#endif
#endif /* RTC_H */
