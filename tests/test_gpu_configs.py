"""The five benchmark configurations end to end: HIP path against the CPU oracle, bit-exact.

Reduced sizes run three seeds with every output compared.  Full sizes run in the launch
configuration the benchmark uses and every output of every configuration is compared with the
oracle (configuration 4: all 256 chains x 16 components, the GPU run once over the whole batch,
the oracle in eight slices of 32 chains so that each test reports within half a minute);
only configuration 5's pseudo-inverse, whose linear-scan oracle is quadratic, is compared on
sampled queries plus the two-sided inequality that fixes every answer.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle
from paper_1912_04050_amd import workloads as wl

pytestmark = pytest.mark.gpu
SEEDS = [wl.DEFAULT_SEED, 1, 77]


@pytest.fixture(scope="module")
def rtc():
    from paper_1912_04050_amd import rtc as mod
    return mod


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def products_equal(rtc, f, g):
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    c = host(rtc.rtc_minplus_conv(dev(f), dev(g), dev_flags=flags))
    d = host(rtc.rtc_maxplus_deconv(dev(f), dev(g), dev_flags=flags))
    assert int(host(flags)[0]) == 0
    assert np.array_equal(c, oracle.minplus_conv(f, g))
    assert np.array_equal(d, oracle.maxplus_deconv(f, g))
    return c, d


@pytest.mark.parametrize("seed", SEEDS)
def test_config1(rtc, seed):
    say("config1 full", seed)
    c = wl.config1(seed)
    products_equal(rtc, c["f"], c["g"])


def run_config2(rtc, seed, batch, n):
    c = wl.config2(seed, batch, n)
    a, b = c["alpha_u"], c["beta_l"]
    _, d = products_equal(rtc, a, b)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    h = host(rtc.rtc_max_hdev(dev(a), dev(b), dev_flags=flags))
    v = host(rtc.rtc_max_vdev(dev(a), dev(b)))
    want_h, fl = oracle.max_hdev(a, b)
    assert np.array_equal(h, want_h) and int(host(flags)[0]) == fl
    assert np.array_equal(v, oracle.max_vdev(a, b))
    assert np.array_equal(v, d[:, 0])  # backlog bound = (alpha (/) beta)[0]


@pytest.mark.parametrize("seed", SEEDS)
def test_config2_reduced(rtc, seed):
    say("config2 reduced", seed)
    run_config2(rtc, seed, 48, 1500)


def test_config2_full(rtc):
    say("config2 full")
    run_config2(rtc, wl.DEFAULT_SEED, 1024, 4096)


@pytest.mark.parametrize("seed", SEEDS)
def test_config3_reduced(rtc, seed):
    say("config3 reduced", seed)
    c = wl.config3(seed, 5, 5000)
    products_equal(rtc, c["f"], c["g"])


def test_config3_full_int64_storage(rtc):
    say("config3 full, int64")
    c = wl.config3(wl.DEFAULT_SEED, 64, 65536)
    products_equal(rtc, c["f"], c["g"])


def test_config3_full_native_int32(rtc):
    say("config3 full, int32 rows, all 64 rows in full")
    c = wl.config3(wl.DEFAULT_SEED, 64, 65536, np.int32)
    products_equal(rtc, c["f"], c["g"])


def run_chain_gpu(rtc, c, chains, components):
    """All components of all chains on the GPU; returns per-component host copies."""
    n = c["alpha_bar_u"].shape[1]
    gam = dev(c["gamma_u"][:chains])
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    a = rtc.rtc_compose(gam, dev(c["alpha_bar_u"][:chains]), dev_flags=flags)
    a0 = host(a)
    outs = []
    for i in range(components):
        ev_lo = torch.empty((chains, n), dtype=torch.int32, device="cuda")
        ev_up = torch.empty((chains, n), dtype=torch.int32, device="cuda")
        au, bl = rtc.rtc_gpc_step(a, dev(c["beta_u"][i, :chains]), dev(c["beta_l"][i, :chains]), gamma_u=gam,
                                  events_lower=ev_lo, events_upper=ev_up, dev_flags=flags)
        outs.append((host(au), host(bl), host(ev_lo), host(ev_up)))
        a = au
    assert int(host(flags)[0]) == 0  # no overflow, composition stayed inside gamma's domain
    return a0, outs


def check_chain_oracle(c, rows, a0, outs):
    want_a, fl = oracle.compose(c["gamma_u"][rows], c["alpha_bar_u"][rows])
    assert fl == 0 and np.array_equal(a0[rows], want_a)
    a = want_a
    for i, (au, bl, lo, up) in enumerate(outs):
        want_au, want_bl = oracle.gpc_step(a, c["beta_u"][i][rows], c["beta_l"][i][rows])
        assert np.array_equal(au[rows], want_au), i
        assert np.array_equal(bl[rows], want_bl), i
        assert np.array_equal(lo[rows], oracle.pseudo_inverse(c["gamma_u"][rows], want_bl, 0)), i
        assert np.array_equal(up[rows], oracle.pseudo_inverse(c["gamma_u"][rows], want_bl, 1)), i
        a = want_au


@pytest.mark.parametrize("seed", SEEDS)
def test_config4_reduced(rtc, seed):
    say("config4 reduced", seed)
    c = wl.config4(seed, chains=6, components=4, n=2500)
    a0, outs = run_chain_gpu(rtc, c, 6, 4)
    check_chain_oracle(c, np.arange(6), a0, outs)


@pytest.fixture(scope="module")
def config4_full(rtc):
    """Configuration 4 at full size, run once on the GPU over the whole batch of 256 chains (the
    launch configuration the benchmark times); the tests below compare slices of it."""
    chains, comps = 256, 16
    c = wl.config4(wl.DEFAULT_SEED, chains, comps, 16384)
    a0, outs = run_chain_gpu(rtc, c, chains, comps)
    return c, a0, outs


@pytest.mark.parametrize("part", range(8))
def test_config4_full(config4_full, part):
    """Every output of every component of chains 32*part .. 32*part+31 against the oracle:
    alpha'^u, beta'^l and both event-domain images (the eight parts cover all 256 x 16)."""
    c, a0, outs = config4_full
    rows = np.arange(32 * part, 32 * part + 32)
    say("config4 full: oracle on chains", rows[0], "..", rows[-1])
    check_chain_oracle(c, rows, a0, outs)


def test_config4_full_invariants(config4_full):
    c, a0, outs = config4_full
    gam = c["gamma_u"]
    for i, (au, bl, lo, up) in enumerate(outs):
        assert np.all(au <= c["beta_u"][i]) and np.all(np.diff(au, axis=1) >= 0), i
        assert np.all(bl >= 0) and np.all(np.diff(bl, axis=1) >= 0) and np.all(bl <= c["beta_l"][i]), i
        inside = lo < gam.shape[1]
        r = np.nonzero(inside)
        assert np.all(gam[r[0], lo[r]] >= bl[r])                      # gamma(gamma^-1(x)) >= x
        assert np.all(np.take_along_axis(gam, np.maximum(up, 0), 1)[up >= 0] <= bl[up >= 0])
        assert np.all(up >= lo - 1)


def run_chain_bounds(rtc, c, chains, components):
    """Delay and backlog bounds of a whole chain: the service curves of its components are
    concatenated (beta_1 (x) beta_2 (x) ...), then the arrival curve's horizontal and vertical
    deviation from the concatenation, all on the GPU, against the oracle doing the same."""
    gam, ab = c["gamma_u"][:chains], c["alpha_bar_u"][:chains]
    curves = np.ascontiguousarray(c["beta_l"][:components, :chains])
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    a = rtc.rtc_compose(dev(gam), dev(ab), dev_flags=flags)
    path = rtc.rtc_conv_chain(dev(curves), dev_flags=flags)
    hflags = torch.zeros(1, dtype=torch.int32, device="cuda")
    h = host(rtc.rtc_max_hdev(a, path, dev_flags=hflags))
    v = host(rtc.rtc_max_vdev(a, path))
    assert int(host(flags)[0]) == 0
    want_a, _ = oracle.compose(gam, ab)
    want_path = oracle.conv_chain(curves)
    assert np.array_equal(host(path), want_path)
    want_h, fl = oracle.max_hdev(want_a, want_path)
    assert np.array_equal(h, want_h) and int(host(hflags)[0]) == fl
    assert np.array_equal(v, oracle.max_vdev(want_a, want_path))
    # "pay bursts only once": the bound through the concatenation is at most the sum of the
    # per-component bounds of the same arrival curve
    per_node = sum(oracle.max_hdev(want_a, curves[i])[0].astype(np.int64) for i in range(components))
    assert np.all(h <= per_node)


@pytest.mark.parametrize("seed", SEEDS)
def test_chain_bounds_reduced(rtc, seed):
    say("chain delay / backlog bounds, reduced", seed)
    run_chain_bounds(rtc, wl.config4(seed, chains=6, components=4, n=2500), 6, 4)


def test_chain_bounds_config4_shape(rtc):
    say("chain delay / backlog bounds, 24 chains x 16 components, N=16384")
    run_chain_bounds(rtc, wl.config4(wl.DEFAULT_SEED, 24, 16, 16384), 24, 16)


def test_product_census(rtc):
    """rtc_product_census: the units it reports add up to the iteration space, rows of the headline
    kind run in the 15-bit flavour, and a product without the packed path counts as 32-bit items."""
    n, batch = 6000, 3
    c = wl.config3(5, batch, n)
    units = batch * sum((min((t + 1) * 2048, n) + 127) // 128 for t in range((n + 2047) // 2048))
    for f, g in ((c["f"], c["g"]), (c["f"].astype(np.int32), c["g"].astype(np.int32))):
        rtc.rtc_set_packed_min_work(0.0)
        try:
            counts = host(rtc.rtc_product_census(rtc.RTC_OP_CONV, dev(f), dev(g)))
        finally:
            rtc.rtc_set_packed_min_work(rtc.RTC_DEFAULT_PACKED_MIN_WORK)
        assert counts.sum() == units and counts[0] + counts[1] > 0.9 * units and counts[4] == 0
    rtc.rtc_set_packed_min_work(1e30)
    try:
        counts = host(rtc.rtc_product_census(rtc.RTC_OP_DECONV, dev(c["f"].astype(np.int32)), dev(c["g"].astype(np.int32))))
        assert counts.tolist() == [0, 0, 0, units, 0]
        counts = host(rtc.rtc_product_census(rtc.RTC_OP_CONV, dev(c["f"].astype(np.float64)), dev(c["g"].astype(np.float64))))
        assert counts.tolist() == [0, 0, 0, 0, units]
    finally:
        rtc.rtc_set_packed_min_work(rtc.RTC_DEFAULT_PACKED_MIN_WORK)


def test_a_refused_call_changes_no_output(rtc):
    """A component step over 2^24 rows of two samples: its two products would fit, the scan after them
    (workgroups of 256 threads) would need 2^32 threads in one grid.  The call is refused with RTC_ERR_SHAPE before its first
    kernel: both outputs still hold what they held.  One row fewer runs, and equals the oracle."""
    batch, n = 1 << 24, 2
    rng = np.random.default_rng(8)
    alpha = np.cumsum(rng.integers(0, 5, (batch, n)), axis=1).astype(np.int32)
    beta_u = np.cumsum(rng.integers(0, 9, (batch, n)), axis=1).astype(np.int32)
    beta_l = (beta_u // 2).astype(np.int32)
    au = torch.full((batch, n), -77, dtype=torch.int32, device="cuda")
    bl = torch.full((batch, n), -78, dtype=torch.int32, device="cuda")
    say("refused component step", batch, n)
    with pytest.raises(rtc.RtcError) as e:
        rtc.rtc_gpc_step(dev(alpha), dev(beta_u), dev(beta_l), alpha_u_out=au, beta_l_out=bl)
    assert e.value.status == -2
    torch.cuda.synchronize()
    assert int((au != -77).sum().item()) == 0 and int((bl != -78).sum().item()) == 0
    m = batch - 1
    got_au, got_bl = rtc.rtc_gpc_step(dev(alpha[:m]), dev(beta_u[:m]), dev(beta_l[:m]))
    got_au, got_bl = host(got_au), host(got_bl)
    for rows in (slice(0, 3000), slice(m - 3000, m)):       # (the oracle takes a parallel region per row)
        want_au, want_bl = oracle.gpc_step(alpha[rows], beta_u[rows], beta_l[rows])
        assert np.array_equal(got_au[rows], want_au) and np.array_equal(got_bl[rows], want_bl)
    # every row: two samples have closed forms
    c0 = alpha[:m, 0] + beta_u[:m, 0]
    c1 = np.minimum(alpha[:m, 0] + beta_u[:m, 1], alpha[:m, 1] + beta_u[:m, 0])
    d0 = np.maximum(c0 - beta_l[:m, 0], c1 - beta_l[:m, 1])
    d1 = c1 - beta_l[:m, 0]
    assert np.array_equal(got_au, np.minimum(np.stack([d0, d1], 1), beta_u[:m]))


def run_config5(rtc, seed, n):
    c = wl.config5(seed, n)
    f, g, x = c["f"], c["g"], c["x"]
    products_equal(rtc, f, g)
    for mode in (0, 1):
        got = host(rtc.rtc_pseudo_inverse(dev(f), dev(x), mode))
        # the oracle's linear scan is O(n^2) here; searchsorted pins it in the CPU tests,
        # so compare sampled queries with the oracle and all of them with the invariants
        idx = np.unique(np.concatenate([[0, 1, n - 1], np.random.default_rng(seed).integers(0, n, 2000)]))
        assert np.array_equal(got[:, idx], oracle.pseudo_inverse(f, x[:, idx], mode))
        k = got[0]
        if mode == 0:
            ok = k < n
            assert np.all(f[0, k[ok]] >= x[0, ok]) and np.all(f[0, np.maximum(k[ok] - 1, 0)][k[ok] > 0] < x[0, ok][k[ok] > 0])
            assert np.all(x[0, ~ok] > f[0, -1])
        else:
            ok = k >= 0
            assert np.all(f[0, k[ok]] <= x[0, ok])
            nxt = ok & (k < n - 1)
            assert np.all(f[0, k[nxt] + 1] > x[0, nxt])


@pytest.mark.parametrize("seed", SEEDS)
def test_config5_reduced(rtc, seed):
    say("config5 reduced", seed)
    run_config5(rtc, seed, 6000)


def test_config5_full(rtc):
    say("config5 full: fp64, N=262144")
    run_config5(rtc, wl.DEFAULT_SEED, 262144)


def test_maximum_curve_length(rtc):
    """n = RTC_MAX_N = 2^24 samples: the HBM-bound operators in full, the products on sampled
    outputs (one product is 1.4e14 pair-ops: a few seconds on the GPU, out of reach for the
    oracle except output by output)."""
    n = 1 << 24
    rng = np.random.default_rng(5)
    f = np.cumsum(rng.integers(0, 4, n, dtype=np.int32), dtype=np.int64).astype(np.int32)[None, :]
    g = np.cumsum(rng.integers(0, 6, n, dtype=np.int32), dtype=np.int64).astype(np.int32)[None, :]
    fd, gd = dev(f), dev(g)
    say("max n: vdev, compose, pinv")
    assert np.array_equal(host(rtc.rtc_max_vdev(fd, gd)), oracle.max_vdev(f, g))
    inner = rng.integers(0, n, (1, 100000)).astype(np.int32)
    assert np.array_equal(host(rtc.rtc_compose(fd, dev(inner))), oracle.compose(f, inner)[0])
    x = rng.integers(-1, int(f[0, -1]) + 2, (1, 3000)).astype(np.int32)
    for mode in (0, 1):
        assert np.array_equal(host(rtc.rtc_pseudo_inverse(fd, dev(x), mode)), oracle.pseudo_inverse(f, x, mode))
    idx = np.unique(np.concatenate([[0, 1, 2047, 2048, n // 2, n - 2049, n - 2, n - 1], rng.integers(0, n, 40)]))
    say("max n: convolution")
    got = host(rtc.rtc_minplus_conv(fd, gd))
    assert np.array_equal(got[0, idx], oracle.product_at(f[0], g[0], idx, False))
    assert np.all(np.diff(got[0]) >= 0) and got[0, 0] == f[0, 0] + g[0, 0]
    say("max n: deconvolution")
    got = host(rtc.rtc_maxplus_deconv(gd, fd))
    assert np.array_equal(got[0, idx], oracle.product_at(g[0], f[0], idx, True))
    assert got[0, -1] == g[0, -1] - f[0, 0]
