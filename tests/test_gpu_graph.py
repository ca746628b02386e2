"""The library under HIP graph capture: it allocates nothing, never synchronises and clears
memory with kernels only, so a sequence of calls can be captured once and replayed.  Every replay
(with new data written into the captured buffers, and eager calls and synchronisations in
between) must equal the oracle bit for bit."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle
from paper_1912_04050_amd import workloads as wl

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def _rows(rng, n, dtype, variant):
    """Six row pairs that take different kernels: general, periodic, convex / concave, one-sided,
    and (int64) steep lines and far offsets; `variant` changes the data, not the kinds."""
    ramp = np.arange(n, dtype=np.int64)
    gen = lambda: np.cumsum(rng.integers(0, 9 + variant, n))
    f = [gen(), gen(), wl.token_bucket(n, 300 + variant, 4, np.int64, at_zero=False), gen(), gen(), gen()]
    g = [gen(), wl.tdma_lower(n, 7 + variant, 31), wl.token_bucket(n, 50, 2 + variant, np.int64, at_zero=False),
         wl.rate_latency(n, 3, 100 + 10 * variant), gen(), gen()]
    if dtype == np.int64:
        f[4], g[4] = f[4] + 1000003 * ramp, g[4] + 999983 * ramp
        f[5], g[5] = f[5] + (1 << 45), g[5] + np.cumsum(rng.integers(0, 300000, n))
    return np.stack(f).astype(dtype), np.stack(g).astype(dtype)


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_products_and_component_step_replay_in_a_graph(dtype):
    from paper_1912_04050_amd import rtc
    rtc.rtc_set_packed_min_work(0.0)          # every path that needs a workspace is taken at this size
    try:
        n, rng = 3000, np.random.default_rng(61)
        f_h, g_h = _rows(rng, n, dtype, 0)
        f, g = dev(f_h), dev(g_h)
        tdt = f.dtype
        conv, deconv = torch.empty_like(f), torch.empty_like(f)
        au, bl = torch.empty_like(f), torch.empty_like(f)
        beta_u = torch.empty_like(f)
        ws = torch.empty(rtc.rtc_workspace_bytes(rtc.RTC_OP_GPC, f.shape[0], n, tdt), dtype=torch.uint8, device="cuda")

        def calls():
            rtc.rtc_minplus_conv(f, g, out=conv, ws=ws)
            rtc.rtc_maxplus_deconv(f, g, out=deconv, ws=ws)
            rtc.rtc_gpc_step(f, beta_u, g, alpha_u_out=au, beta_l_out=bl, ws=ws)

        def check(tag, f_now, g_now):
            print("[case]", tag, np.dtype(dtype).name, flush=True)
            sys.stdout.flush()
            bu_now = g_now + 5
            assert np.array_equal(host(conv), oracle.minplus_conv(f_now, g_now)), tag
            assert np.array_equal(host(deconv), oracle.maxplus_deconv(f_now, g_now)), tag
            want_au, want_bl = oracle.gpc_step(f_now, bu_now, g_now)
            assert np.array_equal(host(au), want_au) and np.array_equal(host(bl), want_bl), tag

        beta_u.copy_(g + 5)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):          # warm-up outside the capture, as torch asks for
            calls()
        torch.cuda.current_stream().wait_stream(side)
        check("eager", f_h, g_h)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            calls()
        for variant in (1, 2, 3):
            f_new, g_new = _rows(rng, n, dtype, variant)
            f.copy_(dev(f_new)); g.copy_(dev(g_new)); beta_u.copy_(g + 5)
            for t in (conv, deconv, au, bl):
                t.zero_()
            graph.replay()
            check(f"replay {variant}", f_new, g_new)
            # the program's own eager work between replays
            assert np.array_equal(host(rtc.rtc_minplus_conv(f, g)), oracle.minplus_conv(f_new, g_new))
    finally:
        rtc.rtc_set_packed_min_work(rtc.RTC_DEFAULT_PACKED_MIN_WORK)
