"""Checks of the seeded input generators (CPU only)."""
import numpy as np

from paper_1912_04050_amd import workloads as wl


def test_stream_reproducible_and_keyed():
    a = wl.stream(1, 2, 3, 100)
    assert np.array_equal(a, wl.stream(1, 2, 3, 100))
    assert np.array_equal(a[:10], wl.stream(1, 2, 3, 10))
    assert not np.array_equal(a, wl.stream(1, 2, 4, 100))
    assert not np.array_equal(a, wl.stream(2, 2, 3, 100))
    u = wl.uniform_int(wl.stream(5, 0, 0, 20000), 3, 11)
    assert u.min() == 3 and u.max() == 11
    d = wl.uniform_double(wl.stream(5, 0, 1, 20000))
    assert 0.0 <= d.min() and d.max() < 1.0 and abs(d.mean() - 0.5) < 0.02


def _tdma_window_service(s, c, n):
    """Service delivered in any window of length D by 'slot s every c ticks', min/max over offsets."""
    on = np.array([1 if (k % c) < s else 0 for k in range(n + c)])
    pre = np.concatenate([[0], np.cumsum(on)])
    lo = np.empty(n, np.int64)
    hi = np.empty(n, np.int64)
    for d in range(n):
        w = [pre[o + d] - pre[o] for o in range(c)]
        lo[d], hi[d] = min(w), max(w)
    return lo, hi


def test_tdma_curves_match_sliding_window():
    rng = np.random.default_rng(3)
    for _ in range(40):
        s = int(rng.integers(1, 30))
        c = int(rng.integers(s, 4 * s + 1))
        n = 300
        lo, hi = _tdma_window_service(s, c, n)
        assert np.array_equal(wl.tdma_lower(n, s, c), lo), (s, c)
        assert np.array_equal(wl.tdma_upper(n, s, c), hi), (s, c)


def test_workload_curves():
    dem = wl.uniform_int(wl.stream(7, 4, 16, 500), 100, 1000)
    gu, gl = wl.workload_curves(dem)
    assert gu[0] == 0 and gl[0] == 0 and len(gu) == 501
    assert np.all(gu >= gl) and gu[-1] == gl[-1] == dem.sum()
    assert np.all(np.diff(gu, 2) <= 0) and np.all(np.diff(gl, 2) >= 0)
    assert gu[3] == np.sort(dem)[-3:].sum() and gl[3] == np.sort(dem)[:3].sum()


def test_config_shapes_and_ranges():
    c1 = wl.config1(n=512)
    assert c1["f"].dtype == np.int32 and c1["f"].shape == (1, 512) and c1["f"][0, 0] == 0
    inc = np.diff(c1["f"][0])
    assert inc.min() >= 0 and inc.max() <= 8
    assert c1["g"][0, 100] == 0 and c1["g"][0, 101] == 3

    c2 = wl.config2(batch=16, n=512)
    assert np.all(np.diff(c2["alpha_u"], axis=1) >= 0) and np.all(np.diff(c2["beta_l"], axis=1) >= 0)
    assert np.all((c2["P"] >= 20) & (c2["P"] <= 200) & (c2["J"] >= 0) & (c2["J"] <= c2["P"]))
    assert np.all((c2["s"] >= 10) & (c2["s"] <= 50) & (c2["c"] >= c2["s"]) & (c2["c"] <= 4 * c2["s"]))
    assert np.all(c2["alpha_u"][:, 0] <= 1)

    c3 = wl.config3(batch=2, n=4096)
    assert c3["f"].dtype == np.int64 and np.all(c3["f"][:, 0] == 0)
    inc = np.diff(c3["g"], axis=1)
    assert np.all((inc <= 4) | ((inc >= 50) & (inc <= 500))) and inc.min() >= 0
    assert 0.25 < np.mean(inc >= 50) < 0.35
    assert not np.array_equal(c3["f"][0], c3["g"][0]) and not np.array_equal(c3["f"][0], c3["f"][1])

    c4 = wl.config4(chains=3, components=2, n=1024)
    assert c4["beta_u"].shape == (2, 3, 1024) and c4["gamma_u"].shape == (3, 1024)
    assert np.all(c4["beta_u"] >= c4["beta_l"]) and np.all(c4["gamma_u"] >= c4["gamma_l"])
    assert np.all(np.diff(c4["beta_l"], axis=2) >= 0)
    assert c4["alpha_bar_u"].max() < 1024  # composition never leaves gamma's domain

    c5 = wl.config5(n=4096)
    assert c5["f"].dtype == np.float64 and c5["f"][0, 0] == 0.0
    assert np.all(np.diff(c5["f"][0]) >= 0) and np.all(np.diff(c5["g"][0]) >= 0)
    assert np.all(np.isfinite(c5["f"])) and not np.any(np.signbit(c5["g"]))
    assert abs(np.diff(c5["f"][0]).mean() - 1.0) < 0.1
