"""ctypes loader for the CPU oracle of the binary convolution layer (bnn_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The product package never imports this module.
All arguments are numpy arrays on the host; results are returned as new arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bnn_oracle.cpp")
_LIB = os.path.join(_HERE, "libbnnoracle.so")
_lib = None


def build(force: bool = True) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["g++", "-std=c++17", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-shared",
                        "-fPIC", "-o", _LIB, _SRC], check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_bnn_dot_packed.restype = ctypes.c_int64
    return _lib


def _p(a):
    return ctypes.c_void_p(a.ctypes.data)


def _i(v):
    return ctypes.c_int64(int(v))


def out_shape(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def conv2d(x, w, stride=1, pad=0):
    """x: int8 [N][H][W][C] of +1/-1, w: int8 [K][R][S][C] of +1/-1 -> int32 [N][Ho][Wo][K]."""
    x = np.ascontiguousarray(x, np.int8)
    w = np.ascontiguousarray(w, np.int8)
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    assert C == C2
    Ho, Wo = out_shape(H, W, R, S, stride, pad)
    out = np.empty((N, Ho, Wo, K), np.int32)
    rc = lib().oracle_bnn_conv2d(_p(x), _p(w), _p(out), _i(N), _i(H), _i(W), _i(C), _i(K), _i(R), _i(S), _i(stride), _i(pad))
    assert rc == 0, rc
    return out


def bitplane_conv2d(x, w, stride=1, pad=0):
    """x: uint8 [N][H][W][C], w: int8 [K][R][S][C] of +1/-1 -> int32 [N][Ho][Wo][K]."""
    x = np.ascontiguousarray(x, np.uint8)
    w = np.ascontiguousarray(w, np.int8)
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    assert C == C2
    Ho, Wo = out_shape(H, W, R, S, stride, pad)
    out = np.empty((N, Ho, Wo, K), np.int32)
    rc = lib().oracle_bnn_bitplane_conv2d(_p(x), _p(w), _p(out), _i(N), _i(H), _i(W), _i(C), _i(K), _i(R), _i(S), _i(stride),
                                          _i(pad))
    assert rc == 0, rc
    return out


def binarize(x1, xi, gamma):
    """Integrated batch-norm + sign: x1 int32 [...][K], xi / gamma float32 [K] -> uint8 0/1 of x1's shape."""
    x1 = np.ascontiguousarray(x1, np.int32)
    xi = np.ascontiguousarray(xi, np.float32)
    gamma = np.ascontiguousarray(gamma, np.float32)
    K = x1.shape[-1]
    assert xi.shape == (K,) and gamma.shape == (K,)
    out = np.empty(x1.shape, np.uint8)
    rc = lib().oracle_bnn_binarize(_p(x1), _p(xi), _p(gamma), _p(out), _i(x1.size // K), _i(K))
    if rc == -4:
        raise ValueError("gamma = 0 is outside the domain of the integrated layer")
    assert rc == 0, rc
    return out


def batchnorm_sign(x1, b, mu, sigma, gamma, beta):
    x1 = np.ascontiguousarray(x1, np.int32)
    K = x1.shape[-1]
    arrs = [np.ascontiguousarray(a, np.float64) for a in (b, mu, sigma, gamma, beta)]
    assert all(a.shape == (K,) for a in arrs)
    out = np.empty(x1.shape, np.uint8)
    rc = lib().oracle_bnn_batchnorm_sign(_p(x1), *[_p(a) for a in arrs], _p(out), _i(x1.size // K), _i(K))
    assert rc == 0, rc
    return out


def pack(bits):
    """[...][C] of +1 (set) / anything else (clear) -> uint32 [...][ceil(C/32)]."""
    bits = np.ascontiguousarray(bits, np.int8)
    C = bits.shape[-1]
    out = np.empty(bits.shape[:-1] + ((C + 31) // 32,), np.uint32)
    rc = lib().oracle_bnn_pack(_p(bits), _p(out), _i(bits.size // C), _i(C))
    assert rc == 0, rc
    return out


def dot_packed(a, b, length):
    a = np.ascontiguousarray(a, np.uint32)
    b = np.ascontiguousarray(b, np.uint32)
    return int(lib().oracle_bnn_dot_packed(_p(a), _p(b), _i(length)))
