"""Randomised parity: shapes, dtypes, value styles and operators drawn from a seeded generator,
HIP path against the CPU oracle, bit-exact.  Complements the hand-picked cases: a few hundred
combinations nobody chose by hand, under both planner settings of the packed path."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", params=["default-planner", "packed-forced"])
def rtc(request):
    from paper_1912_04050_amd import rtc as mod
    if request.param == "packed-forced":
        mod.rtc_set_packed_min_work(0.0)
        mod.rtc_set_small_problem_items(0)      # and the generic kernel's large tiles for every size
    yield mod
    mod.rtc_set_packed_min_work(mod.RTC_DEFAULT_PACKED_MIN_WORK)
    mod.rtc_set_small_problem_items(mod.RTC_DEFAULT_SMALL_PROBLEM_ITEMS)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def draw_rows(rng, batch, n, dtype):
    """A batch of rows in one of several styles (chosen per row)."""
    rows = []
    for _ in range(batch):
        style = rng.integers(0, 8)
        if style == 6:      # periodic from index 1 on (event stream with jitter, TDMA-like service)
            p = int(rng.integers(1, max(2, min(300, n // 8 + 1))))
            pat = rng.integers(0, 6, p) * (rng.random(p) < 0.4)
            v = np.concatenate([[0, int(rng.integers(0, 40))], np.tile(pat, n // p + 2)])[:n]
            v[1:] = np.cumsum(v[1:])
        elif style == 7:    # plateaus and rare steps
            v = np.cumsum(np.where(rng.random(n) < 0.01, rng.integers(1, 50, n), 0))
        elif style == 0:    # slow staircase
            v = np.cumsum(rng.integers(0, 4, n))
        elif style == 1:    # bursts
            v = np.cumsum(np.where(rng.random(n) < 0.02, rng.integers(100, 5000, n), rng.integers(0, 3, n)))
        elif style == 2:    # steep
            v = np.cumsum(rng.integers(0, 4000, n))
        elif style == 3:    # not monotone, both signs
            v = rng.integers(-30000, 30000, n)
        elif style == 4:    # convex or concave
            inc = np.sort(rng.integers(-50, 300, max(n - 1, 1)))
            v = np.concatenate([[int(rng.integers(-5, 5))], inc if rng.random() < 0.5 else inc[::-1]])[:n].cumsum()
        else:               # constant / plateau
            v = np.full(n, int(rng.integers(-9, 9)))
        if np.issubdtype(dtype, np.floating):
            v = v * 0.37 + rng.random(n) * (style not in (5, 6, 7))
        rows.append(v)
    return np.stack(rows).astype(dtype)


@pytest.mark.parametrize("case", range(96))
def test_random_products(rtc, case):
    rng = np.random.default_rng(1000 + case)
    dtype = [np.int32, np.int64, np.float64][case % 3]
    n = int(rng.choice([1, 2, 3, 17, 100, 1023, 1024, 1025, 2048, 2500, 4097, 6000]))
    batch = int(rng.integers(1, 5))
    f, g = draw_rows(rng, batch, n, dtype), draw_rows(rng, batch, n, dtype)
    if dtype == np.int64:
        kind = (case // 3) % 4
        ramp = np.arange(n, dtype=np.int64)
        if kind == 1:           # beyond the 32-bit kernels in every respect
            f, g = f * (1 << 34), g * (1 << 34)
        elif kind == 2:         # steep lines: narrow once the pair's common slope is removed
            f, g = f + int(rng.integers(900000, 1100000)) * ramp, g + int(rng.integers(900000, 1100000)) * ramp
        elif kind == 3:         # far from zero and slowly varying: re-based per chunk
            f = f + np.cumsum(rng.integers(0, 300000, (batch, n)), axis=1) + (1 << 44)
            g = g + np.cumsum(rng.integers(0, 300000, (batch, n)), axis=1) - (1 << 45)
    print("[case]", case, dtype.__name__, batch, n, flush=True)
    sys.stdout.flush()
    fd, gd = dev(f), dev(g)
    assert np.array_equal(host(rtc.rtc_minplus_conv(fd, gd)), oracle.minplus_conv(f, g))
    assert np.array_equal(host(rtc.rtc_maxplus_deconv(fd, gd)), oracle.maxplus_deconv(f, g))
    assert np.array_equal(host(rtc.rtc_maxplus_conv(fd, gd)), oracle.maxplus_conv(f, g))
    assert np.array_equal(host(rtc.rtc_minplus_deconv(fd, gd)), oracle.minplus_deconv(f, g))


@pytest.mark.parametrize("case", range(24))
def test_random_curve_operators(rtc, case):
    rng = np.random.default_rng(2000 + case)
    dtype = [np.int32, np.int64, np.float64][case % 3]
    n = int(rng.choice([1, 5, 64, 1000, 3001]))
    batch = int(rng.integers(1, 4))
    mono = lambda: np.cumsum(rng.integers(0, 9, (batch, n)), axis=1).astype(dtype)
    print("[case]", case, dtype.__name__, batch, n, flush=True)
    f = mono()
    x = rng.integers(-2, int(f.max()) + 3, (batch, int(rng.integers(1, 700)))).astype(dtype)
    for mode in (0, 1):
        assert np.array_equal(host(rtc.rtc_pseudo_inverse(dev(f), dev(x), mode)), oracle.pseudo_inverse(f, x, mode))
    inner = rng.integers(-3, n + 3, (batch, int(rng.integers(1, 900)))).astype(np.int32)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    want, want_flags = oracle.compose(f, inner)
    assert np.array_equal(host(rtc.rtc_compose(dev(f), dev(inner), dev_flags=flags)), want)
    assert int(host(flags)[0]) == want_flags
    alpha, beta_l = mono(), mono()
    beta_u = beta_l + np.cumsum(rng.integers(0, 3, (batch, n)), axis=1).astype(dtype)
    au, bl = rtc.rtc_gpc_step(dev(alpha), dev(beta_u), dev(beta_l))
    want_au, want_bl = oracle.gpc_step(alpha, beta_u, beta_l)
    assert np.array_equal(host(au), want_au) and np.array_equal(host(bl), want_bl)
    assert np.array_equal(host(rtc.rtc_max_vdev(dev(alpha), dev(beta_l))), oracle.max_vdev(alpha, beta_l))
    flags.zero_()
    want_h, want_hf = oracle.max_hdev(alpha, beta_l)
    assert np.array_equal(host(rtc.rtc_max_hdev(dev(alpha), dev(beta_l), dev_flags=flags)), want_h)
    assert int(host(flags)[0]) == want_hf
