"""The C-ABI library loads, exports every declared entry point, and rejects bad arguments
on the host before anything is launched (no GPU needed: no call here reaches a kernel)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1912_04050_amd", "librtc.so")
HEADER = os.path.join(ROOT, "include", "rtc.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_1912_04050_amd import _build
        _build.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    names = set()
    for header in ("rtc.h", "bnn.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b((?:rtc|bnn)_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"rtc_minplus_conv", "rtc_maxplus_deconv", "rtc_pseudo_inverse", "rtc_compose",
            "rtc_gpc_step", "rtc_max_hdev", "rtc_max_vdev", "rtc_workspace_bytes",
            "rtc_strerror", "bnn_pack_channels", "bnn_weight_words", "bnn_pack_weights", "bnn_binary_conv2d",
            "bnn_strerror"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_workspace_sizes_and_messages(lib):
    lib.rtc_workspace_bytes.restype = ctypes.c_size_t
    lib.rtc_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
    assert lib.rtc_workspace_bytes(0, 4, 1000, 0) >= 2 * 4 * 1000 * 4   # packed-path arrays (optional)
    assert lib.rtc_workspace_bytes(0, 4, 1000, 2) == 0
    assert lib.rtc_workspace_bytes(1, 4, 1000, 1) >= 2 * 4 * 1000 * 4 + 16
    assert lib.rtc_workspace_bytes(2, 4, 1000, 0) >= 4 * 1000 * 4
    assert lib.rtc_workspace_bytes(0, 0, 1000, 0) == 0 and lib.rtc_workspace_bytes(0, 1, 1 << 25, 0) == 0
    lib.rtc_strerror.restype = ctypes.c_char_p
    seen = {lib.rtc_strerror(s) for s in range(0, -9, -1)}
    assert len(seen) == 9 and b"ok" in seen


def test_products_reject_bad_arguments(lib):
    sig = [ctypes.c_void_p] * 3 + [ctypes.c_int64] * 4 + [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                                         ctypes.c_void_p, ctypes.c_void_p]
    p = ctypes.c_void_p(0x1000)  # never dereferenced: every call below fails validation first
    for fn in (lib.rtc_minplus_conv, lib.rtc_maxplus_deconv):
        fn.argtypes = sig
        assert fn(None, p, p, 1, 8, 8, 8, 0, None, 0, None, None) == -1
        assert fn(p, p, p, 0, 8, 8, 8, 0, None, 0, None, None) == -2
        assert fn(p, p, p, 1, 0, 8, 8, 0, None, 0, None, None) == -2
        assert fn(p, p, p, 1, (1 << 24) + 1, 1 << 25, 1 << 25, 0, None, 0, None, None) == -2
        assert fn(p, p, p, 1, 8, 8, 8, 7, None, 0, None, None) == -3
        assert fn(ctypes.c_void_p(0x1002), p, p, 1, 8, 8, 8, 0, None, 0, None, None) == -4
        assert fn(p, p, p, 2, 8, 4, 8, 0, None, 0, None, None) == -5
        assert fn(p, p, p, 1, 8, 8, 8, 1, None, 0, None, None) == -6   # int64 needs a workspace
        assert fn(p, p, p, 1, 8, 8, 8, 1, p, 8, None, None) == -6


def test_other_entry_points_reject_bad_arguments(lib):
    p = ctypes.c_void_p(0x1000)
    lib.rtc_pseudo_inverse.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                       ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_void_p]
    assert lib.rtc_pseudo_inverse(None, 8, p, 8, p, 1, 0, 0, None) == -1
    assert lib.rtc_pseudo_inverse(p, 8, p, 8, p, 1, 2, 0, None) == -8
    assert lib.rtc_pseudo_inverse(p, 8, p, 0, p, 1, 0, 0, None) == -2
    lib.rtc_compose.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p,
                                ctypes.c_void_p]
    assert lib.rtc_compose(p, 0, p, 8, p, 1, 0, None, None) == -2
    assert lib.rtc_compose(p, 8, None, 8, p, 1, 0, None, None) == -1
    lib.rtc_max_hdev.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                 ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.rtc_max_hdev(p, p, None, 1, 8, 0, None, None) == -1
    lib.rtc_max_vdev.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                 ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]
    assert lib.rtc_max_vdev(p, p, p, 1, 8, 5, None) == -3
    lib.rtc_validate_monotone.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.rtc_validate_monotone(p, 1, 8, 8, 0, None, None, None) == -1    # the flag word is required
    assert lib.rtc_validate_monotone(p, 2, 8, 4, 0, None, p, None) == -5
    assert lib.rtc_validate_monotone(p, 2, 8, 8, 7, None, p, None) == -3
    assert lib.rtc_validate_monotone(p, 2, 0, 8, 0, None, p, None) == -2
    lib.rtc_gpc_step.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    assert lib.rtc_gpc_step(None, None) == -1
    lib.rtc_product_structure.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_int, ctypes.c_void_p]
    assert lib.rtc_product_structure(0, p, p, None, 1, 8, 8, 8, 0, None) == -1
    assert lib.rtc_product_structure(2, p, p, p, 1, 8, 8, 8, 0, None) == -8     # RTC_OP_GPC is no product
    assert lib.rtc_product_structure(0, p, p, p, 1, 8, 4, 8, 0, None) == -5
    assert lib.rtc_product_structure(0, p, p, p, 0, 8, 8, 8, 0, None) == -2
    assert lib.rtc_selftest_half_minmax(None, None) == -1
    lib.rtc_set_packed_small_n.argtypes = [ctypes.c_int64]
    assert lib.rtc_set_packed_small_n(-1) == -2
    assert lib.rtc_set_packed_small_n(4096) == 0
    lib.rtc_set_small_problem_items.argtypes = [ctypes.c_int64]
    assert lib.rtc_set_small_problem_items(-1) == -2
    assert lib.rtc_set_small_problem_items(8192) == 0
    assert lib.rtc_set_structure_paths(1) == 0
    lib.rtc_product_periods.argtypes = [ctypes.c_int] + [ctypes.c_void_p] * 4 + [ctypes.c_int64] * 4 + [ctypes.c_int, ctypes.c_void_p]
    assert lib.rtc_product_periods(0, p, p, None, p, 1, 8, 8, 8, 0, None) == -1      # codes are required
    assert lib.rtc_product_periods(2, p, p, p, p, 1, 8, 8, 8, 0, None) == -8         # RTC_OP_GPC is no product


def test_bnn_entry_points_reject_bad_arguments(lib):
    p = ctypes.c_void_p(0x1000)
    i64 = ctypes.c_int64
    lib.bnn_pack_channels.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, i64, i64, ctypes.c_void_p]
    assert lib.bnn_pack_channels(None, 0, p, 4, 32, None) == -1
    assert lib.bnn_pack_channels(p, 2, p, 4, 32, None) == -3
    assert lib.bnn_pack_channels(p, 0, p, 0, 32, None) == -2
    assert lib.bnn_pack_channels(ctypes.c_void_p(0x1002), 1, p, 4, 32, None) == -4
    lib.bnn_weight_words.argtypes = [i64] * 4
    lib.bnn_weight_words.restype = ctypes.c_size_t
    assert lib.bnn_weight_words(70, 3, 3, 40) == 9 * 2 * 128 + 9 * 128      # K padded to 128, two words per pixel
    assert lib.bnn_weight_words(0, 3, 3, 40) == 0
    # a matrix-core shape carries the filters once more as int8 (K 9 C bytes)
    assert lib.bnn_weight_words(64, 3, 3, 128) == 9 * 4 * 64 + 9 * 64 + 64 * 9 * 128 // 4
    assert lib.bnn_weight_words(64, 3, 3, 96) == 9 * 3 * 64 + 9 * 64
    # the planner's choice of the matrix-core kernel: shape rules, the size threshold, the knob
    lib.bnn_matrix_path_applies.argtypes = [i64] * 9
    assert lib.bnn_matrix_path_applies(256, 13, 13, 1024, 1024, 3, 3, 1, 1) == 1
    assert lib.bnn_matrix_path_applies(1, 13, 13, 1024, 1024, 3, 3, 1, 1) == 0        # too few pixels to fill the chip
    assert lib.bnn_matrix_path_applies(256, 13, 13, 1024, 1000, 3, 3, 1, 1) == 0      # K not a multiple of 64
    assert lib.bnn_matrix_path_applies(256, 13, 13, 64, 1024, 3, 3, 1, 1) == 0        # too few channels
    assert lib.bnn_matrix_path_applies(256, 13, 13, 1024, 1024, 3, 3, 2, 1) == 0      # stride 2
    assert lib.bnn_matrix_path_applies(64, 8, 300, 128, 64, 3, 3, 1, 1) == 0          # rows too long for the staged range
    assert lib.bnn_set_matrix_path(1) == 0
    assert lib.bnn_matrix_path_applies(1, 13, 13, 1024, 1024, 3, 3, 1, 1) == 1
    assert lib.bnn_set_matrix_path(-1) == 0
    assert lib.bnn_matrix_path_applies(256, 13, 13, 1024, 1024, 3, 3, 1, 1) == 0
    assert lib.bnn_set_matrix_path(2) < 0 and lib.bnn_set_matrix_path(5) < 0
    assert lib.bnn_set_matrix_path(3) == 0 and lib.bnn_set_matrix_path(4) == 0
    assert lib.bnn_set_matrix_path(0) == 0
    lib.bnn_pack_weights.argtypes = [ctypes.c_void_p, ctypes.c_void_p, i64, i64, i64, i64, ctypes.c_void_p]
    assert lib.bnn_pack_weights(p, None, 8, 3, 3, 32, None) == -1
    assert lib.bnn_pack_weights(p, p, 8, 3, 0, 32, None) == -2
    lib.bnn_binary_conv2d.argtypes = [ctypes.c_void_p] * 6 + [i64] * 9 + [ctypes.c_void_p]
    ok = (1, 8, 8, 32, 64, 3, 3, 1, 1)
    assert lib.bnn_binary_conv2d(p, p, None, None, None, None, *ok, None) == -1          # no output
    assert lib.bnn_binary_conv2d(p, p, None, None, None, p, *ok, None) == -1             # x4 without thresholds
    assert lib.bnn_binary_conv2d(p, p, p, p, p, p, 1, 8, 8, 32, 64, 3, 4, 1, 1, None) == -5    # S = 4
    assert lib.bnn_binary_conv2d(p, p, p, p, p, p, 1, 8, 8, 32, 64, 3, 3, 3, 1, None) == -5    # stride 3
    assert lib.bnn_binary_conv2d(p, p, p, p, p, p, 1, 2, 2, 32, 64, 5, 5, 1, 0, None) == -2    # empty output
    assert lib.bnn_binary_conv2d(p, p, p, p, p, p, 0, 8, 8, 32, 64, 3, 3, 1, 1, None) == -2
    lib.bnn_strerror.restype = ctypes.c_char_p
    assert b"width" in lib.bnn_strerror(-5)


def test_binding_constants_match_the_headers():
    """Every enumerator and flag of the two headers that the Python bindings also define has the
    header's value there (the bindings restate them; nothing generates one from the other)."""
    from paper_1912_04050_amd import bnn, rtc

    def constants(path):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        found = {m.group(1): int(m.group(2), 0) for m in re.finditer(r"#define\s+((?:RTC|BNN)_\w+)\s+(-?\w+)\s*$", text, re.M)
                 if re.fullmatch(r"-?(0x[0-9a-fA-F]+|\d+)", m.group(2))}
        for body in re.findall(r"enum\s*\w*\s*\{(.*?)\}", text, re.S):
            nxt = 0
            for item in body.split(","):
                item = item.strip()
                if not item:
                    continue
                name, _, val = item.partition("=")
                nxt = int(val.strip(), 0) if val.strip() else nxt
                found[name.strip()] = nxt
                nxt += 1
        return found

    checked = 0
    for mod, header in ((rtc, HEADER), (bnn, os.path.join(ROOT, "include", "bnn.h"))):
        for name, value in constants(header).items():
            if hasattr(mod, name):
                assert getattr(mod, name) == value, (name, getattr(mod, name), value)
                checked += 1
    assert checked >= 20


def test_a_launch_that_would_not_fit_is_refused_before_anything_is_enqueued(lib):
    """Every entry point walks its launch sequence in a dry run first.  A component step over
    2^24 rows of two samples: both products fit (workgroups of 64 threads), the scan that follows
    them would need 2^24 workgroups of 256 threads = 2^32 threads, which the runtime does not
    take.  The call returns RTC_ERR_SHAPE from the dry run, i.e. without a single HIP call (which
    is why this runs without a GPU, on pointers that are never dereferenced); the GPU suite
    repeats it on real buffers and checks that no output byte changed."""
    from paper_1912_04050_amd import rtc
    lib.rtc_gpc_step.argtypes = [ctypes.POINTER(rtc.rtc_gpc_args), ctypes.c_void_p]
    lib.rtc_workspace_bytes.restype = ctypes.c_size_t
    lib.rtc_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
    batch, n = 1 << 24, 2
    a = rtc.rtc_gpc_args()
    for k, name in enumerate(("alpha_u", "beta_u", "beta_l", "alpha_u_out", "beta_l_out", "ws")):
        setattr(a, name, 0x100000 * (k + 1))
    a.batch, a.n, a.dt = batch, n, 0
    a.ws_bytes = lib.rtc_workspace_bytes(2, batch, n, 0)
    assert a.ws_bytes > 0
    assert lib.rtc_gpc_step(ctypes.byref(a), None) == -2
    # the products alone fit at this size; one row more per 64-thread workgroup limit does not
    sig = [ctypes.c_void_p] * 3 + [ctypes.c_int64] * 4 + [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                                         ctypes.c_void_p, ctypes.c_void_p]
    lib.rtc_minplus_conv.argtypes = sig
    p = ctypes.c_void_p(0x100000)
    assert lib.rtc_minplus_conv(p, p, ctypes.c_void_p(0x200000), 1 << 26, 1, 1, 1, 0, None, 0, None, None) == -2
