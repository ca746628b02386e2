"""ctypes binding of the binary convolution entry points (include/bnn.h).

Marshalling only: torch tensors provide device memory and the current stream; every step of
the layer runs in the HIP kernels of librtc.so.  Fails loudly if the library is missing.
"""
from __future__ import annotations

import ctypes

import torch

from . import _build

_lib = ctypes.CDLL(_build.ensure_built())
_i64, _vp, _int = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int

BNN_VALUE_INT8, BNN_VALUE_FLOAT = 0, 1
BNN_PROFILE_KIND = 32   # kind of the convolution kernel in rtc.rtc_profile_read()

_lib.bnn_pack_channels.argtypes = [_vp, _int, _vp, _i64, _i64, _vp]
_lib.bnn_pack_channels.restype = _int
_lib.bnn_weight_words.argtypes = [_i64, _i64, _i64, _i64]
_lib.bnn_weight_words.restype = ctypes.c_size_t
_lib.bnn_pack_weights.argtypes = [_vp, _vp, _i64, _i64, _i64, _i64, _vp]
_lib.bnn_pack_weights.restype = _int
_lib.bnn_binary_conv2d.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp] + [_i64] * 9 + [_vp]
_lib.bnn_binary_conv2d.restype = _int
_lib.bnn_strerror.argtypes = [_int]
_lib.bnn_strerror.restype = ctypes.c_char_p


_lib.bnn_set_planner.argtypes = [_int, _int]
_lib.bnn_set_planner.restype = _int
_lib.bnn_set_matrix_path.argtypes = [_int]
_lib.bnn_set_matrix_path.restype = _int
_lib.bnn_matrix_path_applies.argtypes = [_i64] * 9
_lib.bnn_matrix_path_applies.restype = _int


class BnnError(RuntimeError):
    def __init__(self, status: int):
        super().__init__(f"libbnn status {status}: {_lib.bnn_strerror(status).decode()}")
        self.status = status


def _check(status: int):
    if status != 0:
        raise BnnError(status)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dense_cuda(t, name):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a dense device tensor")
    return t


def bnn_set_planner(tile_pixels: int = 0, filter_blocks: int = 0):
    _check(_lib.bnn_set_planner(tile_pixels, filter_blocks))


def bnn_set_matrix_path(mode: int = 0):
    _check(_lib.bnn_set_matrix_path(mode))


def bnn_matrix_path_applies(N, H, W, C, K, R=3, S=3, stride=1, pad=1) -> bool:
    return bool(_lib.bnn_matrix_path_applies(N, H, W, C, K, R, S, stride, pad))


def out_shape(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def bnn_pack_channels(x, out=None):
    """x: [..., C] int8 or float32 device tensor -> int32 [..., ceil(C/32)] (bit patterns of uint32 words)."""
    _dense_cuda(x, "x")
    if x.dtype not in (torch.int8, torch.float32):
        raise ValueError("x must be int8 or float32")
    C = x.shape[-1]
    rows = x.numel() // C
    if out is None:
        out = torch.empty(x.shape[:-1] + ((C + 31) // 32,), dtype=torch.int32, device=x.device)
    _check(_lib.bnn_pack_channels(_ptr(x), BNN_VALUE_INT8 if x.dtype == torch.int8 else BNN_VALUE_FLOAT, _ptr(out), rows,
                                  C, _stream()))
    return out


def bnn_weight_words(K, R, S, C) -> int:
    return int(_lib.bnn_weight_words(K, R, S, C))


def bnn_pack_weights(w, out=None):
    """w: [K][R][S][C] int8 of +1 / -1 -> the filter bank in the kernel's layout (int32 words)."""
    _dense_cuda(w, "w")
    if w.dtype != torch.int8 or w.dim() != 4:
        raise ValueError("w must be int8 [K][R][S][C]")
    K, R, S, C = w.shape
    if out is None:
        out = torch.empty(bnn_weight_words(K, R, S, C), dtype=torch.int32, device=w.device)
    _check(_lib.bnn_pack_weights(_ptr(w), _ptr(out), K, R, S, C, _stream()))
    return out


def bnn_binary_conv2d(x_words, w_packed, shape, xi=None, gamma=None, want_x1=False, want_x4=True, stride=1, pad=0,
                      out_x1=None, out_x4=None):
    """shape = (N, H, W, C, K, R, S).  Returns (x1 or None, packed x4 or None)."""
    N, H, W, C, K, R, S = shape
    _dense_cuda(x_words, "x_words")
    _dense_cuda(w_packed, "w_packed")
    if x_words.numel() != N * H * W * ((C + 31) // 32) or w_packed.numel() != bnn_weight_words(K, R, S, C):
        raise ValueError("operand sizes do not match the shape")
    Ho, Wo = out_shape(H, W, R, S, stride, pad)
    if want_x1 and out_x1 is None:
        out_x1 = torch.empty((N, Ho, Wo, K), dtype=torch.int32, device=x_words.device)
    if want_x4 and out_x4 is None:
        out_x4 = torch.empty((N, Ho, Wo, (K + 31) // 32), dtype=torch.int32, device=x_words.device)
    if out_x4 is not None:
        if xi is None or gamma is None or xi.numel() != K or gamma.numel() != K or xi.dtype != torch.float32 or \
                gamma.dtype != torch.float32:
            raise ValueError("xi and gamma must be float32 [K]")
    _check(_lib.bnn_binary_conv2d(_ptr(x_words), _ptr(w_packed), _ptr(xi), _ptr(gamma), _ptr(out_x1), _ptr(out_x4), N, H,
                                  W, C, K, R, S, stride, pad, _stream()))
    return out_x1, out_x4
