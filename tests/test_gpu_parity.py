"""Parity of the HIP path (through the C-ABI binding) against the CPU oracle.

Bit-exact for every dtype: integer results have one correct bit pattern, and for fp64
each candidate is a single rounded add/subtract and the selection is exact, so the
tolerance is 0 (np.array_equal on the raw values).
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle
from paper_1912_04050_amd import workloads as wl

pytestmark = pytest.mark.gpu

NP2T = {np.dtype(np.int32): torch.int32, np.dtype(np.int64): torch.int64, np.dtype(np.float64): torch.float64}
DTYPES = [np.int32, np.int64, np.float64]


@pytest.fixture(scope="module", params=["default-planner", "packed-wide-tiles", "packed-small-tiles"])
def rtc(request):
    """Every test runs three times: with the default planner (small problems take the generic
    kernel alone, with its small tiles), and with the packed 16-bit path forced on for every size
    that brings a workspace, once with its tiles of 2048 outputs and once with those of 1024
    (both with the generic kernel's large tiles for every size)."""
    from paper_1912_04050_amd import rtc as mod
    default_small_n = 4096
    if request.param != "default-planner":
        mod.rtc_set_packed_min_work(0.0)
        mod.rtc_set_packed_small_n(0 if request.param == "packed-wide-tiles" else 1 << 24)
        mod.rtc_set_small_problem_items(0)      # the generic kernel keeps its large tiles whatever the size
    yield mod
    mod.rtc_set_packed_min_work(mod.RTC_DEFAULT_PACKED_MIN_WORK)
    mod.rtc_set_packed_small_n(default_small_n)
    mod.rtc_set_small_problem_items(mod.RTC_DEFAULT_SMALL_PROBLEM_ITEMS)


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def check_products(rtc, f, g, tag):
    say(tag, "conv/deconv", f.dtype, f.shape, g.shape)
    got_c = host(rtc.rtc_minplus_conv(dev(f), dev(g)))
    got_d = host(rtc.rtc_maxplus_deconv(dev(f), dev(g)))
    assert np.array_equal(got_c, oracle.minplus_conv(f, g)), tag
    assert np.array_equal(got_d, oracle.maxplus_deconv(f, g)), tag


# sizes: below one block, around the 16-step block, around the 1024-output tile, several tiles
SIZES = [1, 2, 15, 16, 17, 31, 33, 64, 100, 1023, 1024, 1025, 1040, 2049, 3000, 4133]


@pytest.mark.parametrize("dtype", DTYPES)
def test_products_ragged_sizes(rtc, dtype):
    for n in SIZES:
        f = wl.random_monotone(7, 2 * n, 2, n, dtype)
        g = wl.random_monotone(7, 2 * n + 1, 2, n, dtype)
        check_products(rtc, f, g, f"ragged n={n}")


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_products_arbitrary_signed_values(rtc, dtype):
    rng = np.random.default_rng(5)
    for n in (1, 17, 700, 2500):
        f = rng.integers(-10**6, 10**6, (3, n)).astype(dtype)
        g = rng.integers(-10**6, 10**6, (3, n)).astype(dtype)
        check_products(rtc, f, g, f"signed n={n}")


def test_products_float_not_monotone(rtc):
    rng = np.random.default_rng(6)
    for n in (5, 1200):
        f = rng.normal(size=(2, n)) * 100 + 1000
        g = rng.normal(size=(2, n)) * 100 + 1000
        check_products(rtc, f, g, f"float wild n={n}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_products_broadcast_rows(rtc, dtype):
    n = 1500
    f = wl.random_monotone(8, 1, 4, n, dtype)
    g = wl.random_monotone(8, 2, 1, n, dtype)
    say("broadcast g", dtype)
    assert np.array_equal(host(rtc.rtc_minplus_conv(dev(f), dev(g))), oracle.minplus_conv(f, g))
    assert np.array_equal(host(rtc.rtc_maxplus_deconv(dev(f), dev(g))), oracle.maxplus_deconv(f, g))
    say("broadcast f", dtype)
    assert np.array_equal(host(rtc.rtc_minplus_conv(dev(g), dev(f))), oracle.minplus_conv(g, f))
    assert np.array_equal(host(rtc.rtc_maxplus_deconv(dev(g), dev(f))), oracle.maxplus_deconv(g, f))


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_structured_products_broadcast_rows(rtc, dtype):
    """One curve against a batch (row stride 0) where the pairs take the structure-exploiting
    kernels: a periodic, a convex and a concave curve broadcast as g and as f."""
    n = 4200
    rng = np.random.default_rng(51)
    many = np.stack([wl.random_monotone(52, k, 1, n, np.int64)[0] for k in range(60)]
                    + [wl.rate_latency(n, 3, 40), wl.token_bucket(n, 50, 2, np.int64, at_zero=False),
                       wl.tdma_lower(n, 4, 19), wl.periodic_jitter_upper(n, 25, 7)]).astype(dtype)
    for name, one in (("periodic", wl.tdma_lower(n, 9, 33)), ("convex", wl.rate_latency(n, 5, 700)),
                      ("concave", wl.token_bucket(n, 300, 4, np.int64, at_zero=False))):
        one = one.astype(dtype)[None, :]
        say("broadcast", name, "as g", dtype)
        check_products(rtc, many, one, f"broadcast {name} g")
        check_duals(rtc, many, one, f"broadcast {name} g")
        say("broadcast", name, "as f", dtype)
        check_products(rtc, one, many, f"broadcast {name} f")
        check_duals(rtc, one, many, f"broadcast {name} f")


def _both_paths(rtc, f, g, tag):
    """int32 products with the workspace (packed 16-bit chunks where they qualify) and with a
    token workspace (32-bit kernel only): both must equal the oracle."""
    say(tag, f.dtype, f.shape)
    want_c, want_d = oracle.minplus_conv(f, g), oracle.maxplus_deconv(f, g)
    tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
    for ws in (None, tiny):
        assert np.array_equal(host(rtc.rtc_minplus_conv(dev(f), dev(g), ws=ws)), want_c), (tag, ws is None)
        assert np.array_equal(host(rtc.rtc_maxplus_deconv(dev(f), dev(g), ws=ws)), want_d), (tag, ws is None)


def test_packed_path_mixed_chunks(rtc):
    """Rows whose chunks partly qualify for the packed kernel and partly fall back."""
    rng = np.random.default_rng(21)
    n = 7000
    # slow rows (every chunk packs), steep rows (none packs), rows with jumps (some chunks pack)
    slow = np.cumsum(rng.integers(0, 5, (2, n)), axis=1)
    steep = np.cumsum(rng.integers(0, 3000, (2, n)), axis=1)
    jumpy = np.cumsum(rng.integers(0, 5, (2, n)), axis=1)
    jumpy[:, 1500:] += 200000
    jumpy[:, 4100:] += 90000
    wild = np.concatenate([rng.integers(-40000, 40000, (1, n)), rng.integers(-9000, 9000, (1, n))])
    for dt in (np.int32, np.int64):
        f = np.concatenate([slow, steep, jumpy, wild]).astype(dt)
        g = np.concatenate([slow[::-1], slow, jumpy[::-1], wild[::-1]]).astype(dt)
        if dt == np.int32:
            _both_paths(rtc, f, g, "packed mixed")
            _both_paths(rtc, g, f, "packed mixed swapped")
        else:
            check_products(rtc, f, g, "packed mixed int64")


def test_packed_path_unequal_slopes(rtc):
    """Operands whose average slopes differ: whole chunks of 1024 steps do not fit 16 bits after
    detrending, runs of 128 steps do (the sub-chunk re-basing), steeper ones do not at all."""
    rng = np.random.default_rng(24)
    n = 6000
    rows = []
    for slope_f, slope_g in ((5, 64), (64, 5), (1, 300), (300, 280), (0, 450), (700, 3)):
        f = np.cumsum(rng.integers(0, 2 * slope_f + 1, n))
        g = np.cumsum(rng.integers(0, 2 * slope_g + 1, n))
        rows.append((f, g))
    f = np.stack([r[0] for r in rows]).astype(np.int32)
    g = np.stack([r[1] for r in rows]).astype(np.int32)
    _both_paths(rtc, f, g, "packed unequal slopes")
    check_duals(rtc, f, g, "packed unequal slopes, duals")
    check_products(rtc, f.astype(np.int64), g.astype(np.int64), "packed unequal slopes int64")


def test_packed_path_value_limits(rtc):
    """Values at the edge of the packed path's eligibility (|v| < 2^29) and beyond it."""
    n = 3000
    base = np.cumsum(np.random.default_rng(22).integers(0, 7, (4, n)), axis=1)
    f = base.copy()
    g = base[::-1].copy()
    f[0] += 2**29 - 1 - f[0].max()      # just inside
    f[1] += 2**29                       # just outside: 32-bit kernel only
    g[2] -= 2**29                       # negative, inside
    g[3] = -g[3] - 5                    # falling rows: slope estimate clamps to 0
    _both_paths(rtc, f.astype(np.int32), g.astype(np.int32), "packed limits")


def _bounded_rows(rng, n, span, period, offset=None):
    """Rows without trend whose every aligned run of `period` samples takes both 0 and `span`
    (so that each run's range is exactly span); offset[j] is added to run j."""
    v = rng.integers(0, span + 1, n)
    for s0 in range(0, n, period):
        m = min(period, n - s0)
        if m >= 2:
            i, j = rng.choice(m, 2, replace=False)
            v[s0 + i], v[s0 + j] = 0, span
    if offset is not None:
        v = v + np.repeat(offset, period)[:n]
    v[-1] = v[0] - 1 if v[0] > 0 else v[0]   # first >= last: the slope estimate stays 0
    return v


def test_packed_path_budget_edges(rtc):
    """Operand ranges on both sides of the two packed budgets: window range + 2 x run range
    <= 31742 for the 15-bit flavour, window range + run range <= 65534 for the 16-bit one; whole
    chunks of 1024 steps and sub-chunks of 128 steps."""
    rng = np.random.default_rng(25)
    n = 4300
    cases = []
    for span_w, span_u in ((0, 15871), (31742, 0), (11742, 10000), (11743, 10000), (11741, 10000),
                           (1, 15871), (31743, 0), (20000, 45534), (20000, 45535), (65534, 0), (65535, 0),
                           (0, 65534), (0, 65535), (3, 3)):
        cases.append((_bounded_rows(rng, n, span_u, 128), _bounded_rows(rng, n, span_w, 256)))
    # staircases: sub-chunk ranges fit, chunk ranges do not; narrow and wide sub-chunks mixed
    nsub = (n + 127) // 128
    stair = (np.arange(nsub) % 8) * 9000
    cases.append((_bounded_rows(rng, n, 700, 128, stair), _bounded_rows(rng, n, 30000, 256)))
    cases.append((_bounded_rows(rng, n, 700, 128, stair), _bounded_rows(rng, n, 30400, 256)))
    spans = rng.choice([100, 5000, 15000, 40000], nsub)
    mixed = np.concatenate([_bounded_rows(rng, 128, int(sp), 128) for sp in spans])[:n]
    mixed[-1] = min(mixed[-1], mixed[0])
    cases.append((mixed + np.repeat(stair, 128)[:n], _bounded_rows(rng, n, 1500, 256)))
    cases.append((mixed, _bounded_rows(rng, n, 20000, 256)))
    f = np.stack([c[0] for c in cases]).astype(np.int32)
    g = np.stack([c[1] for c in cases]).astype(np.int32)
    _both_paths(rtc, f, g, "packed budget edges")
    check_duals(rtc, f, g, "packed budget edges, duals")
    _both_paths(rtc, g, f, "packed budget edges, swapped")
    check_duals(rtc, g, f, "packed budget edges, swapped duals")


def test_packed_path_ragged_sizes(rtc):
    for n in (1, 17, 255, 256, 257, 1023, 1024, 1025, 2047, 2048, 2049, 3071, 3073, 5121):
        f = wl.random_monotone(23, 2 * n, 2, n, np.int32, max_inc=40)
        g = wl.random_monotone(23, 2 * n + 1, 2, n, np.int32, max_inc=25)
        _both_paths(rtc, f, g, f"packed ragged n={n}")


def test_int64_wide_and_mixed_rows(rtc):
    """Rows beyond the 32-bit range take the 64-bit kernel; rows inside take the narrowed one."""
    n = 1300
    f = wl.random_monotone(9, 1, 4, n, np.int64)
    g = wl.random_monotone(9, 2, 4, n, np.int64)
    f[1] += 2**40
    g[2] -= 2**35
    f[3] = f[3] * 2**20
    check_products(rtc, f, g, "int64 mixed")
    top = np.iinfo(np.int64).max
    f = (np.arange(n) * 3 + (top // 2 - 3 * n)).astype(np.int64)[None, :]
    g = (np.arange(n) * 5 + (top // 2 - 5 * n)).astype(np.int64)[None, :]
    check_products(rtc, f, g, "int64 near limit")


def test_int64_offset_rows_are_rebased(rtc):
    """int64 rows far from zero but of small range run in 32-bit arithmetic after re-basing."""
    n = 2600
    f = wl.random_monotone(10, 1, 5, n, np.int64, max_inc=30)
    g = wl.random_monotone(10, 2, 5, n, np.int64, max_inc=30)
    f[0] += 2**40
    g[1] -= 2**45
    f[2] += 2**61
    g[2] -= 2**61
    f[3] = -f[3] + 2**50          # falling row
    g[4] += 2**30 - int(g[4].min()) - 5   # straddles the 2^30 boundary
    check_products(rtc, f, g, "int64 offsets")
    check_duals(rtc, f, g, "int64 offsets")
    au, bu = f[:2] - f[:2].min(axis=1, keepdims=True), g[:2] - g[:2].min(axis=1, keepdims=True) + 2**41
    bl = np.minimum(bu, bu - 7)
    say("int64 offsets gpc")
    ao, blo = rtc.rtc_gpc_step(dev(au), dev(bu), dev(bl))
    want_a, want_b = oracle.gpc_step(au, bu, bl)
    assert np.array_equal(host(ao), want_a) and np.array_equal(host(blo), want_b)


def test_int32_near_limit(rtc):
    n = 1100
    top = np.iinfo(np.int32).max
    f = (np.arange(n) * 3 + (top // 2 - 3 * n)).astype(np.int32)
    g = (np.arange(n) * 5 + (top // 2 - 5 * n)).astype(np.int32)
    check_products(rtc, f[None, :], g[None, :], "int32 near limit")


@pytest.mark.parametrize("dtype", DTYPES)
def test_closed_form_on_gpu(rtc, dtype):
    n, b, r, R, T = 3000, 17, 2, 3, 250
    t = np.arange(n)
    alpha = wl.token_bucket(n, b, r, dtype)
    beta = wl.rate_latency(n, R, T, dtype)
    say("closed form", dtype)
    c = host(rtc.rtc_minplus_conv(dev(alpha), dev(beta)))[0]
    d = host(rtc.rtc_maxplus_deconv(dev(alpha), dev(beta)))[0]
    assert np.array_equal(c, (b + r * np.maximum(0, t - T)).astype(dtype))
    head = t <= n - 1 - T
    assert np.array_equal(d[head], (b + r * (t + T)).astype(dtype)[head])
    assert host(rtc.rtc_max_vdev(dev(alpha), dev(beta)))[0] == b + r * T
    assert host(rtc.rtc_max_hdev(dev(alpha), dev(beta)))[0] == T + -(-b // R)


def test_overflow_flag(rtc):
    n = 600
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    f = np.arange(n, dtype=np.int32)[None, :]
    say("overflow flag clean")
    rtc.rtc_minplus_conv(dev(f), dev(f), dev_flags=flags)
    assert int(host(flags)[0]) == 0
    big = (f + (2**31 - 1 - n)).astype(np.int32)
    say("overflow flag raised")
    rtc.rtc_minplus_conv(dev(big), dev(big), dev_flags=flags)
    assert int(host(flags)[0]) & rtc.RTC_FLAG_OVERFLOW


@pytest.mark.parametrize("dtype", DTYPES)
def test_pseudo_inverse(rtc, dtype):
    for n, m in ((1, 5), (7, 40), (1000, 3000), (20000, 5000)):
        f = wl.random_monotone(11, n, 3, n, dtype, max_inc=3)
        if np.dtype(dtype) == np.float64:
            x = np.sort(np.random.default_rng(n).random((3, m)) * (f[:, -1:] + 4) - 2, axis=1)
            x[:, : min(m, n)] = f[:, : min(m, n)]  # exact hits exercise the ties
        else:
            x = np.random.default_rng(n).integers(-2, int(f.max()) + 3, (3, m)).astype(dtype)
        for mode in (0, 1):
            say("pinv", dtype, n, m, mode)
            got = host(rtc.rtc_pseudo_inverse(dev(f), dev(x), mode))
            assert np.array_equal(got, oracle.pseudo_inverse(f, x, mode))


@pytest.mark.parametrize("dtype", DTYPES)
def test_pseudo_inverse_stretch_lengths(rtc, dtype):
    """The inverse stages the stretch of f between the answers of a block's smallest and largest
    query, pads it to one entry short of a power of two and searches it without bounds checks;
    a stretch as long as the window takes the plain search instead.  Blocks of 1024 queries whose
    stretch has exactly 0, 1, 2, 3 ... 2046, 2047, 2048, 2049 ... samples (f strictly increasing, the
    queries spread over [a, a + L]), in both modes, with ties, and with the largest value of the
    type as a query (it equals the padding)."""
    n, m = 9000, 1024
    rng = np.random.default_rng(19)
    top = np.inf if np.dtype(dtype) == np.float64 else np.iinfo(dtype).max
    for L in (0, 1, 2, 3, 4, 7, 8, 1022, 1023, 1024, 1025, 2045, 2046, 2047, 2048, 2049, 4000):
        f = (3 * np.arange(n, dtype=np.int64))[None, :].repeat(2, axis=0)
        f[1, 5000:] = f[1, 5000]                              # row 1 ends in a plateau
        a = int(rng.integers(1, n - L - 2))
        x = np.empty((2, m), np.int64)
        for b in range(2):
            q = rng.integers(3 * a, 3 * (a + L) + 1, m)       # values between and on the samples: ties in both modes
            q[0], q[-1] = 3 * a, 3 * (a + L)
            x[b] = np.sort(q) if b == 0 else q
        f, x = f.astype(dtype), x.astype(dtype)
        for mode in (0, 1):
            say("pinv stretch", dtype, L, mode)
            assert np.array_equal(host(rtc.rtc_pseudo_inverse(dev(f), dev(x), mode)), oracle.pseudo_inverse(f, x, mode))
        x[0, -1] = top                                         # beyond every sample; equal to the padding
        if np.dtype(dtype) != np.float64:
            f[0, -1] = top                                     # ... and to the row's last sample
        for mode in (0, 1):
            assert np.array_equal(host(rtc.rtc_pseudo_inverse(dev(f), dev(x), mode)), oracle.pseudo_inverse(f, x, mode))


@pytest.mark.parametrize("dtype", DTYPES)
def test_compose(rtc, dtype):
    rng = np.random.default_rng(12)
    for k, n in ((1, 9), (300, 1000), (5000, 70000)):
        outer = wl.random_monotone(12, k, 2, k, dtype)
        inner = rng.integers(0, k, (2, n)).astype(np.int32)
        flags = torch.zeros(1, dtype=torch.int32, device="cuda")
        say("compose", dtype, k, n)
        got = host(rtc.rtc_compose(dev(outer), dev(inner), dev_flags=flags))
        want, fl = oracle.compose(outer, inner)
        assert np.array_equal(got, want) and int(host(flags)[0]) == fl == 0
        inner[1, n // 2] = k + 3
        inner[0, 0] = -1
        got = host(rtc.rtc_compose(dev(outer), dev(inner), dev_flags=flags))
        want, fl = oracle.compose(outer, inner)
        assert np.array_equal(got, want) and int(host(flags)[0]) == fl == rtc.RTC_FLAG_DOMAIN


@pytest.mark.parametrize("dtype", DTYPES)
def test_gpc_step(rtc, dtype):
    for n in (1, 50, 1024, 4500, 9000):
        a = wl.random_monotone(13, 3 * n, 3, n, dtype, max_inc=6)
        bu = wl.random_monotone(13, 3 * n + 1, 3, n, dtype, max_inc=12, start_max=0)
        bl = np.minimum(bu, wl.random_monotone(13, 3 * n + 2, 3, n, dtype, max_inc=8, start_max=0))
        gam = wl.random_monotone(13, 3 * n + 3, 3, n + 5, dtype, max_inc=10, start_max=0)
        ev_lo = torch.empty((3, n), dtype=torch.int32, device="cuda")
        ev_up = torch.empty((3, n), dtype=torch.int32, device="cuda")
        say("gpc", dtype, n)
        ao, blo = rtc.rtc_gpc_step(dev(a), dev(bu), dev(bl), gamma_u=dev(gam), events_lower=ev_lo,
                                   events_upper=ev_up)
        want_a, want_b = oracle.gpc_step(a, bu, bl)
        assert np.array_equal(host(ao), want_a)
        assert np.array_equal(host(blo), want_b)
        assert np.array_equal(host(ev_lo), oracle.pseudo_inverse(gam, want_b, 0))
        assert np.array_equal(host(ev_up), oracle.pseudo_inverse(gam, want_b, 1))


@pytest.mark.parametrize("dtype", DTYPES)
def test_gpc_step_both_sides(rtc, dtype):
    for n in (1, 50, 1024, 4500):
        au = wl.random_monotone(15, 5 * n, 3, n, dtype, max_inc=6)
        al = np.minimum(au, wl.random_monotone(15, 5 * n + 1, 3, n, dtype, max_inc=4, start_max=0))
        bu = wl.random_monotone(15, 5 * n + 2, 3, n, dtype, max_inc=12, start_max=0)
        bl = np.minimum(bu, wl.random_monotone(15, 5 * n + 3, 3, n, dtype, max_inc=8, start_max=0))
        gl = wl.random_monotone(15, 5 * n + 4, 3, n + 3, dtype, max_inc=7, start_max=0)
        ev_lo = torch.empty((3, n), dtype=torch.int32, device="cuda")
        ev_up = torch.empty((3, n), dtype=torch.int32, device="cuda")
        say("gpc both sides", dtype, n)
        ao, blo, alo, buo = rtc.rtc_gpc_step(dev(au), dev(bu), dev(bl), alpha_l=dev(al), gamma_l=dev(gl),
                                             events_u_lower=ev_lo, events_u_upper=ev_up)
        want_a, want_b = oracle.gpc_step(au, bu, bl)
        want_al, want_bu = oracle.gpc_step_lower(al, bu, bl)
        assert np.array_equal(host(ao), want_a) and np.array_equal(host(blo), want_b)
        assert np.array_equal(host(alo), want_al)
        assert np.array_equal(host(buo), want_bu)
        assert np.array_equal(host(ev_lo), oracle.pseudo_inverse(gl, want_bu, 0))
        assert np.array_equal(host(ev_up), oracle.pseudo_inverse(gl, want_bu, 1))


@pytest.mark.parametrize("dtype", DTYPES)
def test_component_step_long_rows_few_pairs(rtc, dtype):
    """Few long rows: the remaining-service scans split a row over several workgroups (each reduces
    what lies before its segment itself); both sides of the component against the oracle, with the
    extremum of the difference placed early, late and at a segment boundary."""
    for batch, n, jumps in ((1, 16384, (8192,)), (3, 20001, (5, 19998, 12288)), (2, 70000, (12287, 69997))):
        alpha_u = wl.random_monotone(19, n, batch, n, dtype, max_inc=4)
        beta_l = wl.random_monotone(20, n + 1, batch, n, dtype, max_inc=4, start_max=0)
        beta_u = beta_l + wl.random_monotone(21, n + 2, batch, n, dtype, max_inc=2)
        alpha_l = alpha_u // 2 if np.dtype(dtype) != np.float64 else alpha_u / 2
        for row, at in zip(range(batch), jumps):
            beta_l[row, at:] += 1000           # a jump of beta - alpha at a chosen place
            beta_u[row, at:] += 1000
        say("component step, long rows", dtype, batch, n)
        got = rtc.rtc_gpc_step(dev(alpha_u), dev(beta_u), dev(beta_l), alpha_l=dev(np.ascontiguousarray(alpha_l)))
        want = (*oracle.gpc_step(alpha_u, beta_u, beta_l), *oracle.gpc_step_lower(np.ascontiguousarray(alpha_l), beta_u, beta_l))
        for name, g, w in zip(("alpha_u'", "beta_l'", "alpha_l'", "beta_u'"), got, want):
            assert np.array_equal(host(g), w), name


@pytest.mark.parametrize("dtype", DTYPES)
def test_component_step_many_rows_several_passes(rtc, dtype):
    """From 2048 rows on the scan takes one workgroup per row, pass after pass, with the carry and
    the prefetched pass of the loop, and its coarse table of gamma read by the workgroup itself
    (below that every pass is its own workgroup): both sides with the event-domain images, rows of
    2.2 passes, against the oracle."""
    batch, n = 2048, 2300
    au = wl.random_monotone(31, 1, batch, n, dtype, max_inc=6)
    al = np.minimum(au, wl.random_monotone(31, 2, batch, n, dtype, max_inc=4, start_max=0))
    bu = wl.random_monotone(31, 3, batch, n, dtype, max_inc=12, start_max=0)
    bl = np.minimum(bu, wl.random_monotone(31, 4, batch, n, dtype, max_inc=8, start_max=0))
    gu = wl.random_monotone(31, 5, batch, n + 7, dtype, max_inc=9, start_max=0)
    gl = wl.random_monotone(31, 6, batch, n + 3, dtype, max_inc=7, start_max=0)
    ev = [torch.empty((batch, n), dtype=torch.int32, device="cuda") for _ in range(4)]
    say("component step, many rows", dtype, batch, n)
    ao, blo, alo, buo = rtc.rtc_gpc_step(dev(au), dev(bu), dev(bl), gamma_u=dev(gu), events_lower=ev[0], events_upper=ev[1],
                                         alpha_l=dev(al), gamma_l=dev(gl), events_u_lower=ev[2], events_u_upper=ev[3])
    want_a, want_b = oracle.gpc_step(au, bu, bl)
    want_al, want_bu = oracle.gpc_step_lower(al, bu, bl)
    assert np.array_equal(host(ao), want_a) and np.array_equal(host(blo), want_b)
    assert np.array_equal(host(alo), want_al) and np.array_equal(host(buo), want_bu)
    assert np.array_equal(host(ev[0]), oracle.pseudo_inverse(gu, want_b, 0))
    assert np.array_equal(host(ev[1]), oracle.pseudo_inverse(gu, want_b, 1))
    assert np.array_equal(host(ev[2]), oracle.pseudo_inverse(gl, want_bu, 0))
    assert np.array_equal(host(ev[3]), oracle.pseudo_inverse(gl, want_bu, 1))


@pytest.mark.parametrize("dtype", DTYPES)
def test_deviations(rtc, dtype):
    for n in (1, 77, 5000):
        alpha = wl.random_monotone(14, n, 4, n, dtype, max_inc=5)
        beta = wl.random_monotone(14, n + 1, 4, n, dtype, max_inc=9, start_max=0)
        beta[3] = beta[3] // 3 if np.dtype(dtype) != np.float64 else beta[3] / 3  # row 3: unbounded
        flags = torch.zeros(1, dtype=torch.int32, device="cuda")
        say("deviations", dtype, n)
        h = host(rtc.rtc_max_hdev(dev(alpha), dev(beta), dev_flags=flags))
        v = host(rtc.rtc_max_vdev(dev(alpha), dev(beta)))
        want_h, fl = oracle.max_hdev(alpha, beta)
        assert np.array_equal(h, want_h) and int(host(flags)[0]) == fl
        assert np.array_equal(v, oracle.max_vdev(alpha, beta))
        # both bounds from one pass
        flags2 = torch.zeros(1, dtype=torch.int32, device="cuda")
        h2, v2 = rtc.rtc_max_deviations(dev(alpha), dev(beta), dev_flags=flags2)
        assert np.array_equal(host(h2), want_h) and int(host(flags2)[0]) == fl
        assert np.array_equal(host(v2), oracle.max_vdev(alpha, beta))


@pytest.mark.parametrize("dtype", DTYPES)
def test_deviations_long_rows_and_many_rows(rtc, dtype):
    """Rows of more than 32 blocks of 1024 samples: a workgroup of the horizontal deviation then
    takes several blocks in turn (one atomic per workgroup, at most 32 per row).  Thousands of rows:
    a workgroup of the vertical deviation takes its whole row in several trips."""
    batch, n = 2, 70001
    alpha = wl.random_monotone(33, 1, batch, n, dtype, max_inc=5)
    beta = wl.random_monotone(33, 2, batch, n, dtype, max_inc=9, start_max=0)
    beta[1, 20000:] = beta[1, 20000]          # row 1: the service stops growing, the delay is unbounded
    say("deviations, long rows", dtype, batch, n)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    h, v = rtc.rtc_max_deviations(dev(alpha), dev(beta), dev_flags=flags)
    want_h, fl = oracle.max_hdev(alpha, beta)
    assert np.array_equal(host(h), want_h) and int(host(flags)[0]) == fl
    assert np.array_equal(host(v), oracle.max_vdev(alpha, beta))
    assert np.array_equal(host(rtc.rtc_max_hdev(dev(alpha), dev(beta))), want_h)
    batch, n = 2500, 5000
    alpha = wl.random_monotone(33, 3, batch, n, dtype, max_inc=5)
    beta = wl.random_monotone(33, 4, batch, n, dtype, max_inc=9, start_max=0)
    say("vertical deviation, many rows", dtype, batch, n)
    assert np.array_equal(host(rtc.rtc_max_vdev(dev(alpha), dev(beta))), oracle.max_vdev(alpha, beta))


@pytest.mark.parametrize("dtype", DTYPES)
def test_horizontal_deviation_uneven_service(rtc, dtype):
    """With 64 rows or more of more than 32 blocks of 1024 samples, a workgroup of the horizontal
    deviation goes from one block of alpha to the next and starts the next stretch of beta where
    the last one ended, with a length guessed from the last one.  Service curves whose density
    changes abruptly (plateaus, slow climbs, steep stretches: stretches of a few hundred to more
    than ten thousand samples per block, so that the guess is too short, or the stretch too long
    for the window) and an arrival curve that steps back for a while (outside what the bound is
    used for, but the definition still has a value: a block with smaller queries than the one
    before it) must all come out as the plain search per sample gives them."""
    rng = np.random.default_rng(71)
    distinct, n = 6, 66000
    inc = np.zeros((distinct, n), np.int64)
    for b in range(distinct):
        at = 0
        while at < n:
            kind, run = int(rng.integers(0, 4)), int(rng.integers(200, 6000))
            inc[b, at:at + run] = 0 if kind == 0 else rng.integers(0, (1, 3, 40, 400)[kind], min(run, n - at))
            at += run
    beta = np.cumsum(inc, axis=1)
    beta[:, 0] = 0
    alpha = np.cumsum(rng.integers(0, 100, (distinct, n)), axis=1)
    alpha[0] = np.minimum(alpha[0], beta[0, -1])                 # row 0 stays bounded
    alpha[2, 9000:9500] -= alpha[2, 9000] // 2                   # row 2 steps back for a while
    alpha[3] = beta[3]                                           # row 3: no delay at all
    alpha[4] = np.minimum(alpha[4] // 3, beta[4, -1])            # row 4: arrivals far below the service
    alpha, beta = alpha.astype(dtype), beta.astype(dtype)
    want_h, fl = oracle.max_hdev(alpha, beta)
    want_v = oracle.max_vdev(alpha, beta)
    reps = 11                                                    # 66 rows: 32 workgroups per row, three blocks each
    alpha, beta = np.tile(alpha, (reps, 1)), np.tile(beta, (reps, 1))
    say("horizontal deviation, uneven service", dtype, alpha.shape)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert np.array_equal(host(rtc.rtc_max_hdev(dev(alpha), dev(beta), dev_flags=flags)), np.tile(want_h, reps))
    assert int(host(flags)[0]) == fl
    h, v = rtc.rtc_max_deviations(dev(alpha), dev(beta))
    assert np.array_equal(host(h), np.tile(want_h, reps)) and np.array_equal(host(v), np.tile(want_v, reps))


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_fused_cap_when_every_candidate_is_the_largest_value_of_the_type(rtc, dtype):
    """alpha'^l = min((alpha^l (/) beta^u) (x) beta^l, beta^l) on rows for which every candidate of
    the convolution equals the largest value of the type (a legitimate, overflow-free input): the
    result is the cap beta^l, whatever the number of work items the product is cut into."""
    top = int(np.iinfo(dtype).max)
    for n in (40, 3000, 9000):
        alpha_l = np.full((2, n), top - 5, dtype)
        beta_u = np.zeros((2, n), dtype)
        beta_l = np.full((2, n), 5, dtype)
        beta_l[1] = 3                      # candidates of row 1: top - 2, the cap still decides
        alpha_u = np.zeros((2, n), dtype)
        say("cap against type maximum", dtype, n)
        au, bl, al, bu = rtc.rtc_gpc_step(dev(alpha_u), dev(beta_u), dev(beta_l), alpha_l=dev(alpha_l))
        want_al, want_bu = oracle.gpc_step_lower(alpha_l, beta_u, beta_l)
        assert np.array_equal(want_al, beta_l)
        assert np.array_equal(host(al), want_al) and np.array_equal(host(bu), want_bu)


@pytest.mark.parametrize("dtype", DTYPES)
def test_gpc_tail_long_rows_and_scattered_events(rtc, dtype):
    """The fused tail of the component step (scan + both event-domain images in one kernel): rows
    long enough for several workgroups per row and several passes each, a workload curve gamma of
    another length than the rows, steep and flat stretches so that the answers of one pass span
    more of gamma than the staged window holds (the per-thread search then takes over), queries
    below gamma[0] and above its end, plateaus in gamma; both sides of the component."""
    rng = np.random.default_rng(77)
    for batch, n, ng in ((2, 70001, 50000), (3, 9000, 20000), (5, 300, 64)):
        alpha = wl.random_monotone(21, n, batch, n, dtype, max_inc=3)
        beta_u = wl.random_monotone(21, n + 1, batch, n, dtype, max_inc=40, start_max=0)
        beta_l = (beta_u // 2 if np.dtype(dtype) != np.float64 else beta_u / 2).astype(dtype)
        beta_l[0, n // 3 :] += 3000                       # a jump: the answers of that pass scatter
        alpha_l = (alpha // 3 if np.dtype(dtype) != np.float64 else alpha / 3).astype(dtype)
        inc = rng.integers(0, 7, (batch, ng))             # plateaus (zeros) included
        inc[:, 0] = 5                                      # some queries (0) lie below gamma[0]
        gamma = np.cumsum(inc, axis=1).astype(dtype)
        gamma_l = (gamma // 2 if np.dtype(dtype) != np.float64 else gamma / 2).astype(dtype)
        say("gpc tail", dtype, batch, n, ng)
        ev = [torch.empty((batch, n), dtype=torch.int32, device="cuda") for _ in range(4)]
        au, bl, al, bu = rtc.rtc_gpc_step(dev(alpha), dev(beta_u), dev(beta_l), gamma_u=dev(gamma), events_lower=ev[0],
                                          events_upper=ev[1], alpha_l=dev(alpha_l), gamma_l=dev(gamma_l),
                                          events_u_lower=ev[2], events_u_upper=ev[3])
        want_au, want_bl = oracle.gpc_step(alpha, beta_u, beta_l)
        want_al, want_bu = oracle.gpc_step_lower(alpha_l, beta_u, beta_l)
        assert np.array_equal(host(bl), want_bl) and np.array_equal(host(bu), want_bu)
        assert np.array_equal(host(au), want_au) and np.array_equal(host(al), want_al)
        assert np.array_equal(host(ev[0]), oracle.pseudo_inverse(gamma, want_bl, 0))
        assert np.array_equal(host(ev[1]), oracle.pseudo_inverse(gamma, want_bl, 1))
        assert np.array_equal(host(ev[2]), oracle.pseudo_inverse(gamma_l, want_bu, 0))
        assert np.array_equal(host(ev[3]), oracle.pseudo_inverse(gamma_l, want_bu, 1))
        # one inverse only
        only = torch.empty((batch, n), dtype=torch.int32, device="cuda")
        rtc.rtc_gpc_step(dev(alpha), dev(beta_u), dev(beta_l), gamma_u=dev(gamma), events_upper=only)
        assert np.array_equal(host(only), oracle.pseudo_inverse(gamma, want_bl, 1))


@pytest.mark.parametrize("dtype", DTYPES)
def test_validate_monotone(rtc, dtype):
    """The debug check of the precondition that the inverse, the composition and the deviations do not
    check: expectation straight from the definition (first index whose successor is smaller)."""
    rng = np.random.default_rng(99)
    for n in (1, 2, 255, 256, 257, 5000):
        f = wl.random_monotone(15, n, 9, n, dtype, max_inc=5)
        want = np.full(9, -1, dtype=np.int32)
        if n >= 2:
            for row in (1, 4, 8):                      # plant one to three decreases in three rows
                at = np.sort(rng.integers(0, n - 1, size=1 + row % 3))
                for i in at[::-1]:
                    f[row, i + 1 :] -= 7 + f[row, i + 1] - f[row, i]   # a drop by 7 at i, the rest shifted alike
                want[row] = at[0]
            f[8, n - 1] = f[8, n - 2] - 1              # and one at the very end of a row
            want[8] = min(want[8], n - 2)
        for i in range(9):
            d = np.nonzero(f[i, 1:] < f[i, :-1])[0]
            assert want[i] == (d[0] if d.size else -1)
        say("validate_monotone", dtype, n)
        first_bad, flags = rtc.rtc_validate_monotone(dev(f))
        assert np.array_equal(host(first_bad), want)
        assert int(host(flags)[0]) == (8 if n >= 2 else 0)
        first_bad, flags = rtc.rtc_validate_monotone(dev(f[0]))    # one clean row
        assert host(first_bad)[0] == -1 and int(host(flags)[0]) == 0
        first_bad, flags = rtc.rtc_validate_monotone(dev(f)[::2])  # strided rows 0 2 4 6 8
        assert np.array_equal(host(first_bad), want[::2])


@pytest.mark.parametrize("dtype", DTYPES)
def test_burst_delay_curves_shift(rtc, dtype):
    """Products with delta_T (0 up to T, a value above every sum beyond) delay or advance the other,
    nondecreasing operand by T: a closed form that needs no oracle, over several tiles and a ragged
    tail, the jump also beyond 32 bits for int64 rows."""
    n = 5000
    f = wl.random_monotone(17, n, 4, n, dtype, max_inc=6)
    t = np.arange(n)
    for T, big in ((0, 1 << 20), (1, 1 << 20), (777, 1 << 20), (4999, 1 << 20), (1500, 1 << 40)):
        if big > 1 << 30 and np.dtype(dtype) == np.int32:
            continue
        delta = np.broadcast_to(np.where(t <= T, 0, big).astype(dtype), f.shape).copy()
        say("burst delay", dtype, T, big)
        delayed, advanced = f[:, np.maximum(t - T, 0)], f[:, np.minimum(t + T, n - 1)]
        assert np.array_equal(host(rtc.rtc_minplus_conv(dev(f), dev(delta))), delayed)
        assert np.array_equal(host(rtc.rtc_minplus_conv(dev(delta), dev(f))), delayed)
        assert np.array_equal(host(rtc.rtc_maxplus_deconv(dev(f), dev(delta))), advanced)
        assert np.array_equal(host(rtc.rtc_maxplus_conv(dev(-f), dev(-delta))), -delayed)
        assert np.array_equal(host(rtc.rtc_minplus_deconv(dev(-f), dev(-delta))), -advanced)
        assert np.array_equal(oracle.minplus_conv(f, delta), delayed)


def test_host_validation_on_device_pointers(rtc):
    f = torch.zeros((2, 64), dtype=torch.int32, device="cuda")
    with pytest.raises(rtc.RtcError) as e:
        rtc.rtc_minplus_conv(f.to(torch.int64), f.to(torch.int64), ws=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -6


# ---------------------------------------------------------------------------
# dual products: max-plus convolution, min-plus deconvolution
# ---------------------------------------------------------------------------

def check_duals(rtc, f, g, tag, ws=None):
    say(tag, "maxconv/mindeconv", f.dtype, f.shape)
    assert np.array_equal(host(rtc.rtc_maxplus_conv(dev(f), dev(g), ws=ws)), oracle.maxplus_conv(f, g)), tag
    assert np.array_equal(host(rtc.rtc_minplus_deconv(dev(f), dev(g), ws=ws)), oracle.minplus_deconv(f, g)), tag


@pytest.mark.parametrize("dtype", DTYPES)
def test_dual_products_ragged_sizes(rtc, dtype):
    for n in (1, 2, 16, 17, 100, 1023, 1025, 2049, 3300):
        f = wl.random_monotone(31, 2 * n, 2, n, dtype)
        g = wl.random_monotone(31, 2 * n + 1, 2, n, dtype)
        check_duals(rtc, f, g, f"dual ragged n={n}")


def test_dual_products_signed_and_mixed_chunks(rtc):
    rng = np.random.default_rng(32)
    n = 6500
    slow = np.cumsum(rng.integers(0, 5, (2, n)), axis=1)
    jumpy = np.cumsum(rng.integers(0, 5, (2, n)), axis=1)
    jumpy[:, 2100:] += 150000
    wild = np.concatenate([rng.integers(-40000, 40000, (1, n)), rng.integers(-9000, 9000, (1, n))])
    f = np.concatenate([slow, jumpy, wild])
    g = np.concatenate([slow[::-1], jumpy[::-1], wild[::-1]])
    tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
    check_duals(rtc, f.astype(np.int32), g.astype(np.int32), "dual mixed int32")
    check_duals(rtc, f.astype(np.int32), g.astype(np.int32), "dual mixed int32, 32-bit kernel only", ws=tiny)
    check_duals(rtc, f.astype(np.int64), g.astype(np.int64), "dual mixed int64")
    f64 = f.astype(np.int64)
    f64[1] += 2**41
    check_duals(rtc, f64, g.astype(np.int64), "dual int64 wide row")


def _shaped_rows(rng, n, kind):
    """One row of a given shape: its second differences are >= 0 (convex), <= 0 (concave), 0
    (linear), of both signs (general), or of one sign except at a single sample (spoiled)."""
    inc = rng.integers(-40, 400, max(n - 1, 1))
    if kind in ("convex", "convex-spoiled-first", "convex-spoiled-last"):
        inc = np.sort(inc)
    elif kind in ("concave", "concave-spoiled-mid"):
        inc = np.sort(inc)[::-1]
    elif kind == "linear":
        inc = np.full(max(n - 1, 1), int(rng.integers(-5, 60)))
    elif kind == "token-bucket":
        inc = np.concatenate([[int(rng.integers(50, 900))], np.full(max(n - 2, 0), int(rng.integers(1, 30)))])[:max(n - 1, 1)]
    elif kind == "rate-latency":
        lat = int(rng.integers(0, max(n, 2)))
        inc = np.where(np.arange(max(n - 1, 1)) < lat, 0, int(rng.integers(1, 50)))
    elif kind == "staircase":      # long flat runs: many candidates tie
        inc = np.where(rng.integers(0, 40, max(n - 1, 1)) == 0, rng.integers(1, 4, max(n - 1, 1)) * 100, 0)
    v = np.concatenate([[int(rng.integers(-100, 100))], inc])[:n].cumsum()
    if n >= 4:
        if kind == "convex-spoiled-first":
            v[1] += 1 + (v[2] - 2 * v[1] + v[0]) // 2 + 1      # second difference at 1 turns negative
        if kind == "convex-spoiled-last":
            v[n - 1] -= (v[n - 1] - 2 * v[n - 2] + v[n - 3]) + 1
        if kind == "concave-spoiled-mid":
            v[n // 2] -= 1 - (v[n // 2 + 1] - 2 * v[n // 2] + v[n // 2 - 1]) // 2 + 1
    return v


SHAPES = ["convex", "concave", "linear", "token-bucket", "rate-latency", "general", "staircase", "convex-spoiled-first",
          "convex-spoiled-last", "concave-spoiled-mid"]


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_rows_of_exploitable_convexity(rtc, dtype):
    """Every pairing of row shapes in one batch: pairs whose candidates form a convex or concave
    sequence take the structured kernel (ends of the range, or bisection), pairs with one operand
    of the right shape its anchors-and-brackets branch, all others and the rows spoiled at one
    sample the general kernels; all four products must equal the oracle."""
    rng = np.random.default_rng(41)
    for n in (1, 2, 3, 4, 5, 257, 2500):
        fs, gs = [], []
        for kf in SHAPES:
            for kg in SHAPES:
                fs.append(_shaped_rows(rng, n, kf))
                gs.append(_shaped_rows(rng, n, kg))
        f, g = np.stack(fs).astype(dtype), np.stack(gs).astype(dtype)
        check_products(rtc, f, g, f"shaped n={n}")
        check_duals(rtc, f, g, f"shaped duals n={n}")
        if dtype == np.int64:
            scale = np.where(np.arange(len(fs)) % 3 == 0, 1 << 33, 1)[:, None]   # every third pair beyond 32 bits
            check_products(rtc, f * scale, g * scale, f"shaped wide n={n}")
            check_duals(rtc, f * scale, g * scale, f"shaped wide duals n={n}")


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_one_operand_of_exploitable_convexity_long_rows(rtc, dtype):
    """Arbitrary curves against convex / concave ones at a length of many anchor blocks with a
    ragged last block: plateaus and bursts make candidates tie, the rate-latency curves' long zero
    prefix makes brackets as wide as the row, and a length of 256 k + 1 makes the last two anchors
    coincide."""
    rng = np.random.default_rng(45)
    for n in (20001, 14849, 512):
        arb = np.stack([wl.random_monotone(46, 1, 1, n, np.int64)[0], _shaped_rows(rng, n, "staircase"),
                        _shaped_rows(rng, n, "general"), np.zeros(n, np.int64), _shaped_rows(rng, n, "staircase")])
        cvx = np.stack([wl.rate_latency(n, 7, n // 3), wl.rate_latency(n, 1, n - 2), _shaped_rows(rng, n, "convex"),
                        wl.rate_latency(n, 3, 0), np.maximum(0, np.arange(n) - 50) ** 2 // 64])
        ccv = np.stack([wl.token_bucket(n, 900, 5, np.int64, at_zero=False), wl.token_bucket(n, 0, 0, np.int64),
                        _shaped_rows(rng, n, "concave"), wl.token_bucket(n, 5, 1, np.int64), np.sqrt(np.arange(n) * 4096.0).astype(np.int64)])
        for tag, f, g in (("arbitrary, convex", arb, cvx), ("convex, arbitrary", cvx, arb), ("arbitrary, concave", arb, ccv),
                          ("concave, arbitrary", ccv, arb)):
            # every row against two partners (10 pairs: enough work for the planner to take these paths at each n)
            f, g = np.concatenate([f, np.roll(f, 1, axis=0)]).astype(dtype), np.concatenate([g, g]).astype(dtype)
            for name, op in (("conv", rtc.RTC_OP_CONV), ("deconv", rtc.RTC_OP_DECONV), ("maxconv", rtc.RTC_OP_MAXCONV),
                             ("mindeconv", rtc.RTC_OP_MINDECONV)):
                want = np.array([_structure_by_definition(f[b], g[b], name, batch=len(f)) for b in range(len(f))])
                assert np.array_equal(host(rtc.rtc_product_structure(op, dev(f), dev(g))), want), (tag, name, n)
            check_products(rtc, f, g, f"one-sided {tag} n={n}")
            check_duals(rtc, f, g, f"one-sided duals {tag} n={n}")
            if dtype == np.int64:
                check_products(rtc, f * (1 << 34), g * (1 << 34), f"one-sided wide {tag} n={n}")


def _periodic_row(rng, n, p, first=None, spoil=None):
    """w[0] = 0, w[1] = first, increments from index 1 on repeat a random pattern of length p
    (so w[i+p] = w[i] + const for i >= 1); `spoil` moves one sample by 1."""
    pat = rng.integers(0, 9, p)
    pat[rng.integers(0, p)] += 1 + int(rng.integers(0, 30))                 # not constant: no shorter period by accident
    inc = np.tile(pat, n // p + 2)[:max(n - 2, 0)]
    w = np.concatenate([[0, int(rng.integers(0, 60)) if first is None else first], np.zeros(max(n - 2, 0), np.int64)])[:n]
    w[2:] = w[1] + np.cumsum(inc)
    if spoil is not None:
        w[spoil] += 1
    return w


def _period_target(batch):
    target = 32
    while target < 256 and (target + 1) ** 2 * batch <= 1200000:
        target += 1
    return target


def _period_by_definition(w, n):
    """Smallest p <= min(1024, n // 16) with w[i+p] - w[i] constant over 1 <= i <= n-1-p, else 0."""
    w = np.asarray(w).astype(object) if np.abs(np.asarray(w, dtype=np.float64)).max() > 2.0 ** 61 else np.asarray(w, dtype=np.int64)
    for p in range(1, min(1024, n // 16) + 1):
        d = w[1 + p:] - w[1:n - p]
        if (d == d[0]).all():
            return p
    return 0


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_periodic_operands(rtc, dtype):
    """Curves that are periodic from index 1 on (event streams with jitter, TDMA service) against
    arbitrary ones and against each other: the periodic path's classification is pinned against
    the definition, and all four products against the oracle, next to rows whose period is too
    long, spoiled at one sample, or that another structured path takes first."""
    rng = np.random.default_rng(47)
    ops = (("conv", rtc.RTC_OP_CONV), ("deconv", rtc.RTC_OP_DECONV), ("maxconv", rtc.RTC_OP_MAXCONV),
           ("mindeconv", rtc.RTC_OP_MINDECONV))
    for n in (4113, 2100, 700, 64, 40):
        arb = lambda k: wl.random_monotone(48, k, 1, n, np.int64)[0]
        fs, gs = [], []
        for k, p in enumerate([1, 2, 3, 7, 10, 31, 64, 100, 128, 129, 200, 257]):
            per = _periodic_row(rng, n, min(p, n - 2))
            fs += [arb(3 * k), per, per]
            gs += [per, arb(3 * k + 1), _periodic_row(rng, n, max(1, min(p // 2 + 3, n - 2)))]
        fs += [arb(100), arb(101), arb(102), _shaped_rows(rng, n, "staircase"), wl.periodic_jitter_upper(n, 37, 20),
               wl.tdma_lower(n, 5, 17), wl.periodic_jitter_upper(n, 90, 0), _periodic_row(rng, n, 12, first=0)]
        gs += [_periodic_row(rng, n, 9, spoil=n - 1), _periodic_row(rng, n, 9, spoil=n // 2), _periodic_row(rng, n, 9, spoil=1),
               _periodic_row(rng, n, 6), wl.tdma_lower(n, 11, 40), wl.tdma_upper(n, 3, 9, 4), wl.rate_latency(n, 3, 50),
               wl.token_bucket(n, 30, 2, np.int64, at_zero=False)]
        f, g = np.stack(fs).astype(dtype), np.stack(gs).astype(dtype)
        for name, op in ops:
            got = host(rtc.rtc_product_structure(op, dev(f), dev(g)))
            codes, periods = rtc.rtc_product_periods(op, dev(f), dev(g))
            codes, periods = host(codes), host(periods)
            assert np.array_equal(codes, got)
            target, pmax = _period_target(len(fs)), min(1024, n // 16)
            for b in range(len(fs)):
                want = _structure_by_definition(f[b], g[b], name, batch=len(fs))
                assert got[b] == want, (name, n, b, got[b], want)
                if want in (6, 7):     # the window length: the period found, multiplied up to the target if shorter
                    p = _period_by_definition(g[b] if want == 6 else f[b], n)
                    use = p if p >= target else p * -(-target // p) if p * -(-target // p) <= pmax else p * (pmax // p)
                    assert periods[b] == use, (name, n, b, periods[b], p, use)
                else:
                    assert periods[b] == 0
        check_products(rtc, f, g, f"periodic n={n}")
        check_duals(rtc, f, g, f"periodic duals n={n}")
        if dtype == np.int64:
            check_products(rtc, f * (1 << 35), g * (1 << 33), f"periodic wide n={n}")
            check_duals(rtc, f * (1 << 35), g * (1 << 33), f"periodic wide duals n={n}")


def test_wide_int64_rows_rebased_per_chunk(rtc):
    """int64 rows that span far more than 32 bits: pairs close to a common line are narrowed with
    the slope removed, pairs that vary slowly take 32-bit arithmetic re-based per chunk, pairs
    with a jump beyond the budget, or steep ones, take the fp64 kernel if all their values are within
    +-2^51 and the 64-bit integer kernel otherwise.  All kinds next to
    each other in one batch, all four products, under the three settings of the knob."""
    rng = np.random.default_rng(53)
    for n in (1025, 5000, 20011):
        def slow(offset):               # monotone, increments up to 4e5: about 1.2e9 over a chunk plus a window
            return offset + np.cumsum(rng.integers(0, 400000, n))
        def walk(offset):               # not monotone
            return offset + np.cumsum(rng.integers(-300000, 300000, n))
        jump = slow(0)
        jump[n // 2:] += 1 << 40        # one step beyond any 32-bit budget: this pair is not re-based
        steep = np.cumsum(rng.integers(0, 1 << 24, n))
        edge = np.zeros(n, np.int64)    # ranges that just fit, and (next row) just do not
        edge[512:] = (1 << 30) - 1
        over = edge.copy()
        over[512:] += 2
        ramp = np.arange(n, dtype=np.int64)
        def line(rate):                 # steep line plus small increments
            return rate * ramp + np.cumsum(rng.integers(0, 90, n))
        # steep lines of different slopes: wide even with their common slope removed, yet every
        # chunk and window then fits (slopes 7e5 apart); 3e6 apart they do not
        f = np.stack([slow(1 << 45), walk(-(1 << 50)), jump, slow(0), steep, edge, over, slow(7),
                      line(1000000), line(1700000), line(1000000), -line(500000), jump + (1 << 55), jump - (1 << 51)]).astype(np.int64)
        g = np.stack([slow(-(1 << 44)), slow(1 << 33), slow(5), walk(1 << 41), slow(0), edge, over, walk(0),
                      line(1700000), line(1000000), line(4000000), line(200000), slow(0), slow(3)]).astype(np.int64)
        # (the pairs with `jump`: a step of 2^40 keeps them off the re-based path; within +-2^51 they
        # take the fp64 kernel, the pair lifted to 2^55 and the one reaching below -2^51 the 64-bit one)
        for mode in (2, 1, 0):
            rtc.rtc_set_rebase_wide(mode)
            try:
                check_products(rtc, f, g, f"wide rows n={n} mode={mode}")
                check_duals(rtc, f, g, f"wide rows duals n={n} mode={mode}")
            finally:
                rtc.rtc_set_rebase_wide(2)


def test_wide_int64_rows_broadcast_and_inside_the_component_step(rtc):
    """Steep int64 curves (slope 10^6 per step: far beyond 32 bits, close to a line) as a broadcast
    operand, through the greedy-processing-component step (whose deconvolution stores through the
    min with beta^u) and through a closure, under the three settings of the wide-row knob."""
    rng = np.random.default_rng(57)
    n = 3000
    ramp = np.arange(n, dtype=np.int64)
    def curve(rate, jitter):
        v = rate * ramp + np.cumsum(rng.integers(0, jitter, n))
        v[0] = 0
        return v
    alpha = np.stack([curve(1000000, 900), curve(999000, 50), curve(1000500, 4000)])
    beta_l = np.stack([curve(1000200, 300), curve(1001000, 10), curve(1000500, 2000)])
    beta_u = beta_l + np.stack([curve(3, 40), curve(0, 9), curve(10, 100)])
    one = curve(1000100, 700)[None, :]
    for mode in (2, 1, 0):
        rtc.rtc_set_rebase_wide(mode)
        try:
            check_products(rtc, alpha, one, f"wide broadcast g mode={mode}")
            check_duals(rtc, one, beta_l, f"wide broadcast f mode={mode}")
            say("gpc on steep int64 curves, mode", mode)
            au, bl = rtc.rtc_gpc_step(dev(alpha), dev(beta_u), dev(beta_l))
            want_au, want_bl = oracle.gpc_step(alpha, beta_u, beta_l)
            assert np.array_equal(host(au), want_au) and np.array_equal(host(bl), want_bl)
            say("closure of steep int64 curves, mode", mode)
            rows = alpha[:, :700]
            assert np.array_equal(host(rtc.rtc_subadditive_closure(dev(rows))), oracle.closure(rows)[0])
        finally:
            rtc.rtc_set_rebase_wide(2)


def test_structure_paths_knob(rtc):
    """The same rows through the structure-exploiting kernels and, with the knob off, through the
    general ones: the classification does not change, and both results equal the oracle."""
    rng = np.random.default_rng(49)
    n = 4200
    f = np.stack([wl.random_monotone(50, 0, 1, n, np.int64)[0], _periodic_row(rng, n, 23), wl.token_bucket(n, 90, 3, np.int64, at_zero=False),
                  wl.rate_latency(n, 4, 300), wl.random_monotone(50, 1, 1, n, np.int64)[0]] * 16)
    g = np.stack([wl.tdma_lower(n, 7, 31), wl.random_monotone(50, 2, 1, n, np.int64)[0], wl.token_bucket(n, 20, 1, np.int64, at_zero=False),
                  wl.rate_latency(n, 2, 10), wl.rate_latency(n, 5, 1000)] * 16)
    for dtype in (np.int32, np.int64):
        fd, gd = f.astype(dtype), g.astype(dtype)
        codes = host(rtc.rtc_product_structure(rtc.RTC_OP_CONV, dev(fd), dev(gd)))
        assert list(codes[:5]) == [6, 7, 3, 2, 4]
        try:
            rtc.rtc_set_structure_paths(False)
            assert np.array_equal(host(rtc.rtc_product_structure(rtc.RTC_OP_CONV, dev(fd), dev(gd))), codes)
            check_products(rtc, fd, gd, "general kernels on structured rows")
            check_duals(rtc, fd, gd, "general kernels on structured rows")
        finally:
            rtc.rtc_set_structure_paths(True)
        check_products(rtc, fd, gd, "structured kernels")
        check_duals(rtc, fd, gd, "structured kernels")


def _structure_by_definition(f, g, op, exact_differences=True, batch=1):
    """The documented rule: convexity first, then periodicity."""
    code = _convexity_by_definition(f, g, op) if exact_differences else 1
    n = len(f)
    if code != 1 or n // 16 < 1:
        return code
    pg = _period_by_definition(g, n)
    target = _period_target(batch)            # shorter periods are multiplied up to it: f is not looked at then
    pf = _period_by_definition(f, n) if op in ("conv", "maxconv") and not (0 < pg <= target) else 0
    return 6 if pg and (not pf or pg <= pf) else 7 if pf else 1


def _convexity_by_definition(f, g, op):
    """From second differences in exact Python integers."""
    def shape(v):
        d2 = [int(v[i + 1]) - 2 * int(v[i]) + int(v[i - 1]) for i in range(1, len(v) - 1)]
        return all(x >= 0 for x in d2), all(x <= 0 for x in d2)
    (fcvx, fccv), (gcvx, gccv) = shape(f), shape(g)
    deconv, is_max = op in ("deconv", "mindeconv"), op in ("deconv", "maxconv")
    cvx = (fcvx and gccv) if deconv else (fcvx and gcvx)
    ccv = (fccv and gcvx) if deconv else (fccv and gccv)
    if (cvx if is_max else ccv):
        return 3
    if (ccv if is_max else cvx):
        return 2
    # one operand of the right shape: f for the deconvolutions, g (4) or else f (5) for the convolutions
    want_f, want_g = (fccv, gccv) if is_max else (fcvx, gcvx)
    if deconv:
        return 4 if want_f else 1
    if want_g:
        return 4
    return 5 if want_f else 1


@pytest.mark.parametrize("dtype", [np.int32, np.int64, np.float64])
def test_product_structure_classification(rtc, dtype):
    rng = np.random.default_rng(44)
    ops = {"conv": rtc.RTC_OP_CONV, "deconv": rtc.RTC_OP_DECONV, "maxconv": rtc.RTC_OP_MAXCONV,
           "mindeconv": rtc.RTC_OP_MINDECONV}
    for n in (1, 2, 3, 4, 300, 2100):
        fs, gs = [], []
        for kf in SHAPES:
            for kg in SHAPES:
                fs.append(_shaped_rows(rng, n, kf))
                gs.append(_shaped_rows(rng, n, kg))
        f, g = np.stack(fs).astype(dtype), np.stack(gs).astype(dtype)
        if dtype == np.int64 and n >= 3:
            f[0] = _shaped_rows(rng, n, "convex") * (1 << 40)
            f[1, :] = 0
            f[1, -1] = 1 << 62                      # convex, but its range leaves the exact domain of the test
            g[1] = np.arange(n)
        for name, op in ops.items():
            got = host(rtc.rtc_product_structure(op, dev(f), dev(g)))
            if dtype == np.float64:
                assert np.all(got == 1), name
                continue
            want = np.array([_structure_by_definition(f[b], g[b], name, batch=len(fs)) for b in range(len(fs))])
            if dtype == np.int64 and n >= 3:    # second differences of that row are not exact on the device: not used
                want[1] = _structure_by_definition(f[1], g[1], name, exact_differences=False, batch=len(fs))
            assert np.array_equal(got, want), (name, n, np.nonzero(got != want))


def test_structured_rows_inside_gpc_and_closure(rtc):
    """Token-bucket arrivals through rate-latency service (the textbook closed-form case) next to
    general rows, through the component step, the closure and a chain."""
    n = 1800
    rng = np.random.default_rng(42)
    alpha = np.stack([wl.token_bucket(n, 300, 7, np.int64, at_zero=False), wl.random_monotone(43, 1, 1, n, np.int64)[0],
                      wl.token_bucket(n, 40, 2, np.int64, at_zero=False)]).astype(np.int32)
    beta_l = np.stack([wl.rate_latency(n, 9, 120), wl.rate_latency(n, 11, 15), wl.random_monotone(43, 2, 1, n, np.int64)[0]]).astype(np.int32)
    beta_u = beta_l + np.stack([wl.token_bucket(n, 500, 3, np.int64), wl.token_bucket(n, 10, 1, np.int64),
                                wl.token_bucket(n, 0, 0, np.int64)]).astype(np.int32)
    say("gpc on structured rows")
    au, bl = rtc.rtc_gpc_step(dev(alpha), dev(beta_u), dev(beta_l))
    want_au, want_bl = oracle.gpc_step(alpha, beta_u, beta_l)
    assert np.array_equal(host(au), want_au) and np.array_equal(host(bl), want_bl)
    say("closure of concave / convex rows")
    rows = np.stack([alpha[0, :600], beta_l[0, :600], alpha[1, :600]])
    assert np.array_equal(host(rtc.rtc_subadditive_closure(dev(rows))), oracle.closure(rows)[0])
    assert np.array_equal(host(rtc.rtc_superadditive_closure(dev(rows))), oracle.closure(rows, True)[0])
    say("chain of rate-latency curves")
    curves = np.stack([np.stack([wl.rate_latency(n, int(rng.integers(2, 20)), int(rng.integers(0, 300))) for _ in range(3)])
                       for _ in range(5)]).astype(np.int32)
    assert np.array_equal(host(rtc.rtc_conv_chain(dev(curves))), oracle.conv_chain(curves))


def test_dual_products_zero_curve_scans(rtc):
    """With g = 0 the duals are the running maximum and the suffix minimum."""
    rng = np.random.default_rng(33)
    for dtype in DTYPES:
        f = (rng.integers(-500, 500, (3, 2500))).astype(dtype)
        zero = np.zeros((1, 2500), dtype)
        say("dual zero curve", dtype)
        assert np.array_equal(host(rtc.rtc_maxplus_conv(dev(f), dev(zero))), np.maximum.accumulate(f, axis=1))
        assert np.array_equal(host(rtc.rtc_minplus_deconv(dev(f), dev(zero))),
                              np.minimum.accumulate(f[:, ::-1], axis=1)[:, ::-1])


def test_many_tiny_rows(rtc):
    """Large batch of short curves (more rows than tiles per row)."""
    for n in (1, 3, 70):
        f = wl.random_monotone(34, n, 6000, n, np.int32)
        g = wl.random_monotone(34, n + 1, 6000, n, np.int32)
        check_products(rtc, f, g, f"many tiny rows n={n}")
        check_duals(rtc, f, g, f"many tiny rows n={n}")


# ---------------------------------------------------------------------------
# closures and concatenation
# ---------------------------------------------------------------------------

def test_closures_fp64_by_definition(rtc):
    """Floating point: the powers one factor at a time from the left, as the oracle forms them
    (a squaring schedule would round other sums); tolerance 0."""
    rng = np.random.default_rng(43)
    for n in (1, 2, 3, 4, 17, 130, 300):
        f = np.abs(wl.random_monotone(43, n, 3, n, np.float64, max_inc=9)) + rng.random((3, n))
        f[1] = rng.permutation(f[1])                       # not monotone
        f[2, 0] = -3.5                                     # wrong sign at 0: flagged, read as 0
        flags = torch.zeros(1, dtype=torch.int32, device="cuda")
        say("closure fp64", n)
        got = host(rtc.rtc_subadditive_closure(dev(f), dev_flags=flags))
        want, fl = oracle.closure(f)
        assert np.array_equal(got, want) and int(host(flags)[0]) == fl == rtc.RTC_FLAG_DOMAIN
        flags.zero_()
        got = host(rtc.rtc_superadditive_closure(dev(-f), dev_flags=flags))
        want, fl = oracle.closure(-f, super_additive=True)
        assert np.array_equal(got, want) and int(host(flags)[0]) == fl


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_closures(rtc, dtype):
    rng = np.random.default_rng(41)
    for n in (1, 2, 3, 17, 130, 1500):
        f = np.abs(wl.random_monotone(41, n, 3, n, dtype, max_inc=9))
        f[1] = rng.permutation(f[1])                       # not monotone
        f[2, 0] = -3                                       # wrong sign at 0: flagged, read as 0
        flags = torch.zeros(1, dtype=torch.int32, device="cuda")
        say("closure", dtype, n)
        got = host(rtc.rtc_subadditive_closure(dev(f), dev_flags=flags))
        want, fl = oracle.closure(f)
        assert np.array_equal(got, want) and int(host(flags)[0]) == fl == rtc.RTC_FLAG_DOMAIN
        flags.zero_()
        got = host(rtc.rtc_superadditive_closure(dev(-f), dev_flags=flags))
        want, fl = oracle.closure(-f, super_additive=True)
        assert np.array_equal(got, want) and int(host(flags)[0]) == fl


@pytest.mark.parametrize("dtype", DTYPES)
def test_conv_chain(rtc, dtype):
    for count, n in ((1, 40), (2, 700), (5, 1300)):
        curves = np.stack([wl.random_monotone(42, 10 * count + k, 3, n, dtype, max_inc=4 + k) for k in range(count)])
        say("chain", dtype, count, n)
        got = host(rtc.rtc_conv_chain(dev(curves)))
        assert np.array_equal(got, oracle.conv_chain(curves))
    n = 2000
    params = [(5, 10), (3, 25), (4, 0), (7, 40)]
    curves = np.stack([wl.rate_latency(n, R, T, dtype)[None, :] for R, T in params])
    assert np.array_equal(host(rtc.rtc_conv_chain(dev(curves)))[0], wl.rate_latency(n, 3, 75, dtype))


def test_half_float_minmax_is_integer_minmax_on_this_device(rtc):
    """The 15-bit packed flavour relies on it; the kernel checks every pattern below 0x7C00."""
    assert rtc.rtc_selftest_half_minmax() == 0


# ---------------------------------------------------------------------------
# measurement aids of the boundary
# ---------------------------------------------------------------------------
def test_device_info_and_kernel_timing_record(rtc):
    """rtc_device_info reports the device the roofline is derived from; the timing record holds one
    entry per product kernel launched while it is enabled, of the documented kinds, and none after
    it is stopped."""
    info = rtc.rtc_device_info()
    props = torch.cuda.get_device_properties(0)
    assert info["cu_count"] == props.multi_processor_count and info["clock_khz"] > 100000
    assert info["lds_bytes"] >= 64 * 1024
    f = dev(wl.random_monotone(18, 3000, 3, 3000, np.int32, max_inc=5))
    say("timing record")
    try:
        rtc.rtc_profile_enable(True)
        rtc.rtc_minplus_conv(f, f)
        rtc.rtc_maxplus_deconv(f, f)
        got = rtc.rtc_profile_read()
    finally:
        rtc.rtc_profile_enable(False)
    kinds = {k for k, _ in got}
    conv_kinds = {rtc.RTC_PROFILE_KIND(0, p, 0) for p in (0, 1)}
    deconv_kinds = {rtc.RTC_PROFILE_KIND(0, p, 1) for p in (0, 1)}
    assert kinds & conv_kinds and kinds & deconv_kinds and kinds <= conv_kinds | deconv_kinds
    assert all(0.0 < ms < 1000.0 for _, ms in got)
    rtc.rtc_minplus_conv(f, f)
    rtc.rtc_profile_enable(True)          # restarting clears the record; nothing launched since
    try:
        assert rtc.rtc_profile_read() == []
    finally:
        rtc.rtc_profile_enable(False)
