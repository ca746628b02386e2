"""Pins for the CPU oracle of the binary convolution layer.  None of these touch the GPU.

The oracle is pinned to things other than itself: a library convolution on the same +1 / -1
tensors (exact in float64), the xor / popcount identity evaluated with numpy bit operations, the
whole truth table of the integrated layer, the unfused batch-norm chain, bit patterns packed by
hand, and pure-Python brute force on tiny cases.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import bnn
from paper_1912_04050_amd import bnn_workloads as bw

SEED = bw.DEFAULT_SEED


def torch_conv(x, w, stride, pad):
    """x [N][H][W][C], w [K][R][S][C] (any numeric) -> float64 [N][Ho][Wo][K] via the library routine."""
    xt = torch.from_numpy(np.ascontiguousarray(x, np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.ascontiguousarray(w, np.float64)).permute(0, 3, 1, 2)
    return torch.nn.functional.conv2d(xt, wt, stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()


@pytest.mark.parametrize("shape", [
    # N, H, W, C, K, R, S, stride, pad
    (2, 7, 9, 5, 4, 3, 3, 1, 1), (1, 8, 8, 32, 16, 3, 3, 1, 0), (1, 9, 6, 40, 7, 5, 3, 2, 2), (3, 4, 4, 64, 33, 1, 1, 1, 0),
    (1, 13, 13, 96, 10, 3, 3, 1, 1), (1, 6, 5, 3, 2, 3, 3, 2, 1), (1, 3, 3, 8, 8, 3, 3, 1, 1)])
def test_conv_equals_library_convolution(shape):
    N, H, W, C, K, R, S, stride, pad = shape
    x = bw.random_signs(SEED, 1, (N, H, W, C))
    w = bw.random_signs(SEED, 2, (K, R, S, C))
    got = bnn.conv2d(x, w, stride, pad)
    want = torch_conv(x, w, stride, pad)
    assert got.shape == want.shape
    assert np.array_equal(got, want.astype(np.int32))


def test_conv_brute_force_tiny():
    x = bw.random_signs(SEED, 3, (1, 4, 5, 3))
    w = bw.random_signs(SEED, 4, (2, 3, 3, 3))
    got = bnn.conv2d(x, w, 1, 1)
    for ho in range(4):
        for wo in range(5):
            for k in range(2):
                total = 0
                for r in range(3):
                    for s in range(3):
                        hi, wi = ho - 1 + r, wo - 1 + s
                        if 0 <= hi < 4 and 0 <= wi < 5:
                            total += sum(int(x[0, hi, wi, c]) * int(w[k, r, s, c]) for c in range(3))
                assert got[0, ho, wo, k] == total


def test_conv_extremes():
    """All-equal operands give +Len, opposite ones -Len, Len counting only the taps inside the image."""
    x = np.ones((1, 5, 5, 24), np.int8)
    w = np.ones((1, 3, 3, 24), np.int8)
    out = bnn.conv2d(x, w, 1, 1)[0, :, :, 0]
    taps = np.array([[(3 - (h == 0) - (h == 4)) * (3 - (v == 0) - (v == 4)) for v in range(5)] for h in range(5)])
    assert np.array_equal(out, 24 * taps)
    assert np.array_equal(bnn.conv2d(x, -w, 1, 1)[0, :, :, 0], -24 * taps)


@pytest.mark.parametrize("length", [1, 8, 31, 32, 33, 64, 100, 1000])
def test_xor_popcount_identity(length):
    a = bw.random_signs(SEED, 5, (length,))
    b = bw.random_signs(SEED, 6, (length,))
    pa, pb = bnn.pack(a), bnn.pack(b)
    plain = int(np.dot(a.astype(np.int64), b.astype(np.int64)))
    assert bnn.dot_packed(pa, pb, length) == plain
    # the same with numpy's own bit operations on the packed words
    differing = int(np.unpackbits((pa ^ pb).view(np.uint8)).sum())
    assert length - 2 * differing == plain


def test_conv_through_packed_words():
    """One interior output of the convolution = Len - 2 popcount(xor) over the packed taps."""
    x = bw.random_signs(SEED, 7, (1, 6, 6, 70))
    w = bw.random_signs(SEED, 8, (3, 3, 3, 70))
    out = bnn.conv2d(x, w, 1, 0)
    px, pw = bnn.pack(x), bnn.pack(w)
    for ho, wo, k in ((0, 0, 0), (2, 3, 1), (3, 3, 2)):
        differing = 0
        for r in range(3):
            for s in range(3):
                differing += int(np.unpackbits((px[0, ho + r, wo + s] ^ pw[k, r, s]).view(np.uint8)).sum())
        assert out[0, ho, wo, k] == 9 * 70 - 2 * differing


def test_pack_bit_order_by_hand():
    """Channel c sits in bit c mod 32 of word c div 32, least significant bit first; bits of the
    last word beyond C stay 0.  Pattern worked by hand: +1 at channels 0, 3, 32 and 39 of 40."""
    v = -np.ones(40, np.int8)
    v[[0, 3, 32, 39]] = 1
    assert bnn.pack(v).tolist() == [0b1001, (1 << 0) | (1 << 7)]
    assert bnn.pack(np.ones(33, np.int8)).tolist() == [0xFFFFFFFF, 1]
    assert bnn.pack(-np.ones(5, np.int8)).tolist() == [0]


def test_integrated_layer_truth_table():
    """The four cases against the boolean form (A xor B) or C with A = x1 < xi, B = gamma > 0,
    C = x1 = xi, over every combination of the three predicates."""
    x1 = np.array([[-3, -3, 0, 0, 5, 5]], np.int32).T.repeat(1, axis=1)           # rows = cases of x1
    for xi_v in (-3.0, 0.0, 5.0, -2.5, 0.25, 7.0):
        for g in (0.5, -2.0):
            xi = np.full(1, xi_v, np.float32)
            gamma = np.full(1, g, np.float32)
            got = bnn.binarize(x1, xi, gamma)[:, 0]
            A = x1[:, 0].astype(np.float32) < xi_v
            B = g > 0
            C = x1[:, 0].astype(np.float32) == xi_v
            assert np.array_equal(got.astype(bool), np.logical_or(np.logical_xor(A, B), C))
    with pytest.raises(ValueError):
        bnn.binarize(x1, np.zeros(1, np.float32), np.zeros(1, np.float32))


def test_threshold_form_equals_batchnorm_chain():
    """xi = mu - beta sigma / gamma - b turns bias + batch norm + sign into one comparison.
    Checked away from the rounding boundary (|x1 - xi| > 1e-3), which fp32 thresholds blur."""
    K, rows, length = 64, 500, 9 * 128
    b, mu, sigma, gamma, beta = bw.batchnorm_parameters(SEED, 9, K, length)
    rng = np.random.default_rng(3)
    x1 = rng.integers(-120, 121, (rows, K)).astype(np.int32)
    xi = mu - beta * sigma / gamma - b
    clear = np.abs(x1 - xi[None, :]) > 1e-3
    assert clear.mean() > 0.99
    fused = bnn.binarize(x1, xi.astype(np.float32), gamma.astype(np.float32))
    chain = bnn.batchnorm_sign(x1, b, mu, sigma, gamma, beta)
    assert np.array_equal(fused[clear], chain[clear])
    assert 0.2 < fused.mean() < 0.8   # both outcomes occur


def test_bitplane_layer_closed_form():
    """With bit-planes read as +1 / -1, sum_i 2^(i-1) <I_i . W> = 2 (x * w) - 255 (1 * w), the
    convolutions on the right being ordinary ones of the 8-bit input and of an all-ones image
    (zero padding in both)."""
    x = bw.random_bytes(SEED, 10, (2, 6, 7, 3))
    w = bw.random_signs(SEED, 11, (5, 3, 3, 3))
    got = bnn.bitplane_conv2d(x, w, 1, 1)
    want = 2 * torch_conv(x, w, 1, 1) - 255 * torch_conv(np.ones_like(x), w, 1, 1)
    assert np.array_equal(got, want.astype(np.int64))
    # and plane by plane through the binary convolution itself
    total = np.zeros_like(got)
    for i in range(8):
        plane = (((x >> i) & 1).astype(np.int8) * 2 - 1)
        total += (1 << i) * bnn.conv2d(plane, w, 1, 1)
    assert np.array_equal(got, total)


def test_generators_are_reproducible_and_balanced():
    a = bw.random_signs(SEED, 1, (1000,))
    assert np.array_equal(a, bw.random_signs(SEED, 1, (1000,)))
    assert not np.array_equal(a, bw.random_signs(SEED + 1, 1, (1000,)))
    assert abs(a.astype(np.int64).sum()) < 150
    xi, gamma = bw.thresholds(SEED, 2, 256, 9 * 64)
    assert np.all(gamma != 0) and (gamma > 0).any() and (gamma < 0).any()
    assert (xi == np.round(xi)).mean() > 0.3
