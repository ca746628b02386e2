"""rtc_minplus_conv_static (the entry point that allocates nothing) against rtc_minplus_conv,
bit for bit, on two calls in a row, the second on a smaller input: both share the library's
static device workspace, so the second call runs on what the first one left there."""
import ctypes
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_1912_04050_amd import workloads as wl

pytestmark = pytest.mark.gpu

NP2CODE = {np.dtype(np.int32): 0, np.dtype(np.int64): 1, np.dtype(np.float64): 2}


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def both_ways(rtc, f, g, tag):
    """(result of the static entry point, result of rtc_minplus_conv), as host arrays; the static
    one is called through the C ABI directly, with raw pointers."""
    say(tag, f.dtype, f.shape)
    df, dg = dev(f), dev(g)
    batch, n = f.shape
    out = torch.full((batch, n), -7, dtype=df.dtype, device="cuda")
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    status = rtc._lib.rtc_minplus_conv_static(ctypes.c_void_p(df.data_ptr()), ctypes.c_void_p(dg.data_ptr()),
                                              ctypes.c_void_p(out.data_ptr()), batch, n, n, n, NP2CODE[f.dtype],
                                              ctypes.c_void_p(flags.data_ptr()), stream)
    assert status == 0, rtc.rtc_strerror(status)
    want = rtc.rtc_minplus_conv(df, dg)
    torch.cuda.synchronize()
    assert int(flags.item()) == 0
    return out.cpu().numpy(), want.cpu().numpy()


@pytest.mark.parametrize("dtype", [np.int64, np.int32])
def test_static_entry_point_matches_workspace_entry_point(dtype):
    from paper_1912_04050_amd import rtc
    # first call: a shape that uses the workspace (int64 rows always do: their narrowed copies live
    # there; 2 x 65536 int32 rows are above the work threshold of the packed path, whose arrays do)
    big = (6, 8192) if dtype == np.int64 else (2, 65536)
    small = (3, 2500) if dtype == np.int64 else (1, 5000)
    for k, (batch, n) in enumerate((big, small)):
        tdt = torch.int64 if dtype == np.int64 else torch.int32
        assert 0 < rtc.rtc_workspace_bytes(rtc.RTC_OP_CONV, batch, n, tdt) <= rtc.RTC_STATIC_SCRATCH_BYTES
        f = wl.random_monotone(91, 2 * k, batch, n, dtype)
        g = wl.random_monotone(91, 2 * k + 1, batch, n, dtype)
        got, want = both_ways(rtc, f, g, f"static call {k}")
        assert np.array_equal(got, want)


def test_static_entry_point_with_packed_path_forced():
    """Small shapes with the packed 16-bit path forced on, so that both calls go through every array
    of the workspace (prepared operands, block tables, selectors), the second on a smaller input."""
    from paper_1912_04050_amd import rtc
    rtc.rtc_set_packed_min_work(0.0)
    try:
        for k, (batch, n) in enumerate(((5, 6000), (2, 1777))):
            f = wl.random_monotone(92, 2 * k, batch, n, np.int32)
            g = wl.random_monotone(92, 2 * k + 1, batch, n, np.int32)
            got, want = both_ways(rtc, f, g, f"static packed call {k}")
            assert np.array_equal(got, want)
    finally:
        rtc.rtc_set_packed_min_work(rtc.RTC_DEFAULT_PACKED_MIN_WORK)


def test_static_entry_point_rejects_large_shapes():
    from paper_1912_04050_amd import rtc
    batch, n = 64, 65536
    assert rtc.rtc_workspace_bytes(rtc.RTC_OP_CONV, batch, n, torch.int64) > rtc.RTC_STATIC_SCRATCH_BYTES
    f = torch.zeros((batch, n), dtype=torch.int64, device="cuda")
    out = torch.full((batch, n), 5, dtype=torch.int64, device="cuda")
    with pytest.raises(rtc.RtcError) as e:
        rtc.rtc_minplus_conv_static(f, f, out)
    assert e.value.status == -6
    torch.cuda.synchronize()
    assert int(out.min().item()) == 5 and int(out.max().item()) == 5   # nothing was launched
    # fp64 needs no workspace: never refused for its size
    fd = torch.zeros((2, 70000), dtype=torch.float64, device="cuda")
    outd = torch.empty_like(fd)
    rtc.rtc_minplus_conv_static(fd, fd, outd)
    torch.cuda.synchronize()
    assert float(outd.abs().max().item()) == 0.0
