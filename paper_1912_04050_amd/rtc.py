"""Thin Python binding of librtc (include/rtc.h): argument marshalling only.

Every function has the name of the C entry point it calls, takes torch tensors that
already live in HBM, and enqueues on torch's current HIP stream.  No step of the
curve algebra runs in Python or in torch ops; torch only supplies device memory
and the stream.  Importing this module without a built librtc.so raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librtc.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_1912_04050_amd._build` "
        "(there is no CPU fallback)")

_lib = ctypes.CDLL(LIB_PATH)

RTC_I32, RTC_I64, RTC_F64 = 0, 1, 2
RTC_INV_LOWER, RTC_INV_UPPER = 0, 1
RTC_OP_CONV, RTC_OP_DECONV, RTC_OP_GPC, RTC_OP_MAXCONV, RTC_OP_MINDECONV = 0, 1, 2, 3, 4
RTC_OP_CLOSURE, RTC_OP_CHAIN = 5, 6
RTC_FLAG_OVERFLOW, RTC_FLAG_DOMAIN, RTC_FLAG_UNBOUNDED = 1, 2, 4

_DT = {torch.int32: RTC_I32, torch.int64: RTC_I64, torch.float64: RTC_F64}

_i64, _vp, _sz, _int = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int


class rtc_gpc_args(ctypes.Structure):
    _fields_ = [("alpha_u", _vp), ("beta_u", _vp), ("beta_l", _vp), ("alpha_u_out", _vp),
                ("beta_l_out", _vp), ("gamma_u", _vp), ("n_gamma", _i64), ("events_lower", _vp),
                ("events_upper", _vp), ("batch", _i64), ("n", _i64), ("dt", _int), ("ws", _vp),
                ("ws_bytes", _sz), ("dev_flags", _vp), ("alpha_l", _vp), ("alpha_l_out", _vp),
                ("beta_u_out", _vp), ("gamma_l", _vp), ("n_gamma_l", _i64), ("events_u_lower", _vp),
                ("events_u_upper", _vp)]


_product_sig = [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _int, _vp, _sz, _vp, _vp]
_lib.rtc_minplus_conv.argtypes = _product_sig
_lib.rtc_maxplus_deconv.argtypes = _product_sig
_lib.rtc_maxplus_conv.argtypes = _product_sig
_lib.rtc_minplus_deconv.argtypes = _product_sig
_lib.rtc_pseudo_inverse.argtypes = [_vp, _i64, _vp, _i64, _vp, _i64, _int, _int, _vp]
_lib.rtc_compose.argtypes = [_vp, _i64, _vp, _i64, _vp, _i64, _int, _vp, _vp]
_lib.rtc_gpc_step.argtypes = [ctypes.POINTER(rtc_gpc_args), _vp]
_lib.rtc_max_hdev.argtypes = [_vp, _vp, _vp, _i64, _i64, _int, _vp, _vp]
_lib.rtc_max_vdev.argtypes = [_vp, _vp, _vp, _i64, _i64, _int, _vp]
_lib.rtc_workspace_bytes.argtypes = [_int, _i64, _i64, _int]
_lib.rtc_workspace_bytes.restype = _sz
_lib.rtc_strerror.argtypes = [_int]
_lib.rtc_strerror.restype = ctypes.c_char_p
_lib.rtc_device_info.argtypes = [ctypes.POINTER(_int)] * 3
for _name in ("rtc_minplus_conv", "rtc_maxplus_deconv", "rtc_maxplus_conv", "rtc_minplus_deconv", "rtc_pseudo_inverse", "rtc_compose",
              "rtc_gpc_step", "rtc_max_hdev", "rtc_max_vdev", "rtc_device_info"):
    getattr(_lib, _name).restype = _int


class RtcError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"librtc status {status}: {_lib.rtc_strerror(status).decode()}")


def _check(status: int):
    if status != 0:
        raise RtcError(status)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _rows(t: torch.Tensor):
    """(tensor, rows, n, element stride) of a [n] or [rows][n] device tensor."""
    if not t.is_cuda:
        raise ValueError("librtc takes device tensors")
    if t.dim() == 1:
        t = t.unsqueeze(0)
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("curves must be [n] or [batch][n] with contiguous samples")
    return t, t.shape[0], t.shape[1], (t.stride(0) if t.shape[0] > 1 else 0)


def _row_stride(t, rows, batch, n):
    if batch == 1:
        return n
    return 0 if rows == 1 else t.stride(0)


def _dense(t: torch.Tensor):
    """A [n] or [batch][n] device tensor that must already be dense (no copies are made here)."""
    t, rows, n, _ = _rows(t)
    if not t.is_contiguous():
        raise ValueError("this argument must be a dense [batch][n] tensor")
    return t, rows, n


def rtc_workspace_bytes(op: int, batch: int, n: int, dtype: torch.dtype) -> int:
    return int(_lib.rtc_workspace_bytes(op, batch, n, _DT[dtype]))


def rtc_strerror(status: int) -> str:
    return _lib.rtc_strerror(status).decode()


def rtc_device_info():
    cu, khz, lds = _int(), _int(), _int()
    _check(_lib.rtc_device_info(ctypes.byref(cu), ctypes.byref(khz), ctypes.byref(lds)))
    return {"cu_count": cu.value, "clock_khz": khz.value, "lds_bytes": lds.value}


_lib.rtc_profile_enable.argtypes = [_int]
_lib.rtc_profile_enable.restype = _int
_lib.rtc_profile_read.argtypes = [_int, ctypes.POINTER(_int), ctypes.POINTER(ctypes.c_float)]
_lib.rtc_profile_read.restype = _int


def RTC_PROFILE_KIND(dtype_code: int, packed: int, product: int) -> int:
    return dtype_code * 8 + packed * 4 + product


_lib.rtc_set_packed_min_work.argtypes = [ctypes.c_double]
_lib.rtc_set_packed_min_work.restype = _int


RTC_DEFAULT_PACKED_MIN_WORK = 2 ** 33


def rtc_set_packed_min_work(batch_times_n_squared: float):
    _check(_lib.rtc_set_packed_min_work(float(batch_times_n_squared)))


_lib.rtc_selftest_half_minmax.argtypes = [_vp, _vp]
_lib.rtc_selftest_half_minmax.restype = _int


def rtc_selftest_half_minmax() -> int:
    """Mismatches of the packed half-float min3 / max3 against integer min / max (must be 0)."""
    word = torch.zeros(1, dtype=torch.int32, device="cuda")
    _check(_lib.rtc_selftest_half_minmax(_ptr(word), _stream()))
    torch.cuda.synchronize()
    return int(word.item())


_lib.rtc_product_structure.argtypes = [_int, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _int, _vp]
_lib.rtc_product_structure.restype = _int
_lib.rtc_product_periods.argtypes = [_int, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _int, _vp]
_lib.rtc_product_periods.restype = _int
RTC_STRUCTURE_GENERAL, RTC_STRUCTURE_BISECT, RTC_STRUCTURE_ENDS = 1, 2, 3
RTC_STRUCTURE_BRACKET, RTC_STRUCTURE_BRACKET_SWAPPED = 4, 5
RTC_STRUCTURE_PERIODIC, RTC_STRUCTURE_PERIODIC_SWAPPED = 6, 7


_lib.rtc_validate_monotone.argtypes = [_vp, _i64, _i64, _i64, _int, _vp, _vp, _vp]
_lib.rtc_validate_monotone.restype = _int
RTC_FLAG_NOT_MONOTONE = 8


def rtc_validate_monotone(f, dev_flags=None):
    """(first_bad, dev_flags): per row the first index i with f[i+1] < f[i] or -1; the flag word gets
    RTC_FLAG_NOT_MONOTONE when there is one."""
    f, batch, n, stride = _rows(f)
    if dev_flags is None:
        dev_flags = torch.zeros(1, dtype=torch.int32, device=f.device)
    first_bad = torch.empty(batch, dtype=torch.int32, device=f.device)
    _check(_lib.rtc_validate_monotone(_ptr(f), batch, n, stride, _DT[f.dtype], _ptr(first_bad), _ptr(dev_flags), _stream()))
    return first_bad, dev_flags


def rtc_product_periods(op: int, f, g):
    """(codes, periods) per row pair: rtc_product_structure plus the periodic path's window length."""
    f, bf, n, _ = _rows(f)
    g, bg, ng, _ = _rows(g)
    if ng != n or f.dtype != g.dtype or (bf != bg and 1 not in (bf, bg)):
        raise ValueError("operands must have the same length and dtype, batch equal or 1")
    batch = max(bf, bg)
    codes = torch.empty(batch, dtype=torch.int32, device=f.device)
    periods = torch.empty(batch, dtype=torch.int32, device=f.device)
    _check(_lib.rtc_product_periods(op, _ptr(f), _ptr(g), _ptr(codes), _ptr(periods), batch, n,
                                    _row_stride(f, bf, batch, n), _row_stride(g, bg, batch, n), _DT[f.dtype], _stream()))
    return codes, periods


def rtc_product_structure(op: int, f, g, out=None):
    """Per row pair: which kernel family the product `op` (RTC_OP_CONV, ...) gives it."""
    f, bf, n, _ = _rows(f)
    g, bg, ng, _ = _rows(g)
    if ng != n or f.dtype != g.dtype or (bf != bg and 1 not in (bf, bg)):
        raise ValueError("operands must have the same length and dtype, batch equal or 1")
    batch = max(bf, bg)
    if out is None:
        out = torch.empty(batch, dtype=torch.int32, device=f.device)
    _check(_lib.rtc_product_structure(op, _ptr(f), _ptr(g), _ptr(out), batch, n, _row_stride(f, bf, batch, n),
                                      _row_stride(g, bg, batch, n), _DT[f.dtype], _stream()))
    return out


_lib.rtc_product_census.argtypes = [_int, _vp, _vp, _i64, _i64, _i64, _i64, _int, _vp, _sz, _vp, _vp]
_lib.rtc_product_census.restype = _int
RTC_CENSUS_COUNTS = 5


def rtc_product_census(op: int, f, g, ws=None, counts=None):
    """counts[RTC_CENSUS_COUNTS] (int64, device): units of the product's iteration space per arithmetic
    flavour (15-bit on chunk base, 15-bit on sub-chunk bases, 16-bit saturating, 32-bit, other kernels)."""
    f, bf, n, _ = _rows(f)
    g, bg, ng, _ = _rows(g)
    if ng != n or f.dtype != g.dtype or (bf != bg and 1 not in (bf, bg)):
        raise ValueError("operands must have the same length and dtype, batch equal or 1")
    batch = max(bf, bg)
    if counts is None:
        counts = torch.zeros(RTC_CENSUS_COUNTS, dtype=torch.int64, device=f.device)
    ws, ws_bytes = _workspace(op, batch, n, f.dtype, f.device, ws)
    _check(_lib.rtc_product_census(op, _ptr(f), _ptr(g), batch, n, _row_stride(f, bf, batch, n),
                                   _row_stride(g, bg, batch, n), _DT[f.dtype], _ptr(ws), ws_bytes, _ptr(counts), _stream()))
    return counts


_lib.rtc_set_packed_small_n.argtypes = [_i64]
_lib.rtc_set_packed_small_n.restype = _int


def rtc_set_packed_small_n(n: int):
    _check(_lib.rtc_set_packed_small_n(int(n)))


_lib.rtc_set_small_problem_items.argtypes = [_i64]
_lib.rtc_set_small_problem_items.restype = _int


RTC_DEFAULT_SMALL_PROBLEM_ITEMS = 8192


def rtc_set_small_problem_items(items: int):
    _check(_lib.rtc_set_small_problem_items(int(items)))


_lib.rtc_set_rebase_wide.argtypes = [_int]
_lib.rtc_set_rebase_wide.restype = _int


def rtc_set_rebase_wide(mode: int):
    """0: wide int64 rows stay with the 64-bit kernel; 1: slowly varying ones are re-based per chunk;
    2 (default): before that, pairs close to a line are narrowed with their common slope removed."""
    _check(_lib.rtc_set_rebase_wide(int(mode)))


_lib.rtc_set_structure_paths.argtypes = [_int]
_lib.rtc_set_structure_paths.restype = _int


def rtc_set_structure_paths(enabled: bool):
    _check(_lib.rtc_set_structure_paths(1 if enabled else 0))


def rtc_profile_enable(on):
    """False / 0 stops; True / 1 records the product kernels; 2 also those behind a per-row selector."""
    _check(_lib.rtc_profile_enable(int(on)))


def rtc_profile_read(max_entries: int = 1024):
    """[(kind, milliseconds)] of the product kernels recorded since rtc_profile_enable(True)."""
    kinds = (_int * max_entries)()
    ms = (ctypes.c_float * max_entries)()
    got = _lib.rtc_profile_read(max_entries, kinds, ms)
    if got < 0:
        raise RtcError(got)
    return [(kinds[i], ms[i]) for i in range(got)]


def _workspace(op, batch, n, dtype, device, ws):
    need = rtc_workspace_bytes(op, batch, n, dtype)
    if ws is None and need > 0:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    return ws, (0 if ws is None else ws.numel() * ws.element_size())


def _product(fn, op, f, g, out, ws, dev_flags):
    f, bf, n, sf = _rows(f)
    g, bg, ng, sg = _rows(g)
    if ng != n or f.dtype != g.dtype or (bf != bg and 1 not in (bf, bg)):
        raise ValueError("operands must have the same length and dtype, batch equal or 1")
    batch = max(bf, bg)
    sf = _row_stride(f, bf, batch, n)
    sg = _row_stride(g, bg, batch, n)
    if out is None:
        out = torch.empty((batch, n), dtype=f.dtype, device=f.device)
    ws, ws_bytes = _workspace(op, batch, n, f.dtype, f.device, ws)
    _check(fn(_ptr(f), _ptr(g), _ptr(out), batch, n, sf, sg, _DT[f.dtype], _ptr(ws), ws_bytes,
              _ptr(dev_flags), _stream()))
    return out


def rtc_minplus_conv(f, g, out=None, ws=None, dev_flags=None):
    """out[b][t] = min_{0<=s<=t} f[b][s] + g[b][t-s]."""
    return _product(_lib.rtc_minplus_conv, RTC_OP_CONV, f, g, out, ws, dev_flags)


_lib.rtc_minplus_conv_static.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _int, _vp, _vp]
_lib.rtc_minplus_conv_static.restype = _int
RTC_STATIC_SCRATCH_BYTES = 32 << 20


def rtc_minplus_conv_static(f, g, out, dev_flags=None):
    """rtc_minplus_conv on the library's own static workspace; `out` is the caller's ([batch][n])."""
    f, bf, n, _ = _rows(f)
    g, bg, ng, _ = _rows(g)
    if ng != n or f.dtype != g.dtype or (bf != bg and 1 not in (bf, bg)):
        raise ValueError("operands must have the same length and dtype, batch equal or 1")
    batch = max(bf, bg)
    if out.dtype != f.dtype or out.numel() != batch * n or not out.is_contiguous():
        raise ValueError("out must be a dense [batch][n] tensor of the operands' dtype")
    _check(_lib.rtc_minplus_conv_static(_ptr(f), _ptr(g), _ptr(out), batch, n, _row_stride(f, bf, batch, n),
                                        _row_stride(g, bg, batch, n), _DT[f.dtype], _ptr(dev_flags), _stream()))
    return out


def rtc_maxplus_deconv(f, g, out=None, ws=None, dev_flags=None):
    """out[b][t] = max_{0<=u<=n-1-t} f[b][t+u] - g[b][u]."""
    return _product(_lib.rtc_maxplus_deconv, RTC_OP_DECONV, f, g, out, ws, dev_flags)


def rtc_maxplus_conv(f, g, out=None, ws=None, dev_flags=None):
    """out[b][t] = max_{0<=s<=t} f[b][s] + g[b][t-s]."""
    return _product(_lib.rtc_maxplus_conv, RTC_OP_MAXCONV, f, g, out, ws, dev_flags)


def rtc_minplus_deconv(f, g, out=None, ws=None, dev_flags=None):
    """out[b][t] = min_{0<=u<=n-1-t} f[b][t+u] - g[b][u]."""
    return _product(_lib.rtc_minplus_deconv, RTC_OP_MINDECONV, f, g, out, ws, dev_flags)


def rtc_pseudo_inverse(f, x, mode: int = RTC_INV_LOWER, out=None):
    f, batch, n = _dense(f)
    x, bx, m = _dense(x)
    if bx != batch or x.dtype != f.dtype:
        raise ValueError("x must have f's batch and dtype")
    if out is None:
        out = torch.empty((batch, m), dtype=torch.int32, device=f.device)
    _check(_lib.rtc_pseudo_inverse(_ptr(f), n, _ptr(x), m, _ptr(out), batch, mode, _DT[f.dtype], _stream()))
    return out


def rtc_compose(outer, inner, out=None, dev_flags=None):
    outer, batch, n_outer = _dense(outer)
    inner, bi, n = _dense(inner)
    if bi != batch or inner.dtype != torch.int32:
        raise ValueError("inner must be int32 with outer's batch")
    if out is None:
        out = torch.empty((batch, n), dtype=outer.dtype, device=outer.device)
    _check(_lib.rtc_compose(_ptr(outer), n_outer, _ptr(inner), n, _ptr(out), batch, _DT[outer.dtype],
                            _ptr(dev_flags), _stream()))
    return out


def rtc_gpc_step(alpha_u, beta_u, beta_l, alpha_u_out=None, beta_l_out=None, gamma_u=None,
                 events_lower=None, events_upper=None, ws=None, dev_flags=None, alpha_l=None,
                 alpha_l_out=None, beta_u_out=None, gamma_l=None, events_u_lower=None, events_u_upper=None):
    """One greedy processing component; returns (alpha'^u, beta'^l), or with alpha_l given
    (alpha'^u, beta'^l, alpha'^l, beta'^u)."""
    alpha_u, batch, n = _dense(alpha_u)
    beta_u = _dense(beta_u)[0]
    beta_l = _dense(beta_l)[0]
    if beta_u.shape != alpha_u.shape or beta_l.shape != alpha_u.shape:
        raise ValueError("alpha_u, beta_u, beta_l must have one shape")
    if alpha_u_out is None:
        alpha_u_out = torch.empty_like(alpha_u)
    if beta_l_out is None:
        beta_l_out = torch.empty_like(alpha_u)
    ws, ws_bytes = _workspace(RTC_OP_GPC, batch, n, alpha_u.dtype, alpha_u.device, ws)
    a = rtc_gpc_args()
    a.alpha_u, a.beta_u, a.beta_l = alpha_u.data_ptr(), beta_u.data_ptr(), beta_l.data_ptr()
    a.alpha_u_out, a.beta_l_out = alpha_u_out.data_ptr(), beta_l_out.data_ptr()
    if gamma_u is not None:
        gamma_u = _dense(gamma_u)[0]
        a.gamma_u, a.n_gamma = gamma_u.data_ptr(), gamma_u.shape[1]
    a.events_lower = None if events_lower is None else events_lower.data_ptr()
    a.events_upper = None if events_upper is None else events_upper.data_ptr()
    a.batch, a.n, a.dt = batch, n, _DT[alpha_u.dtype]
    a.ws, a.ws_bytes = (None if ws is None else ws.data_ptr()), ws_bytes
    a.dev_flags = None if dev_flags is None else dev_flags.data_ptr()
    if alpha_l is not None:
        alpha_l = _dense(alpha_l)[0]
        if alpha_l.shape != alpha_u.shape or alpha_l.dtype != alpha_u.dtype:
            raise ValueError("alpha_l must have alpha_u's shape and dtype")
        if alpha_l_out is None:
            alpha_l_out = torch.empty_like(alpha_u)
        if beta_u_out is None:
            beta_u_out = torch.empty_like(alpha_u)
        a.alpha_l, a.alpha_l_out, a.beta_u_out = alpha_l.data_ptr(), alpha_l_out.data_ptr(), beta_u_out.data_ptr()
        if gamma_l is not None:
            gamma_l = _dense(gamma_l)[0]
            a.gamma_l, a.n_gamma_l = gamma_l.data_ptr(), gamma_l.shape[1]
        a.events_u_lower = None if events_u_lower is None else events_u_lower.data_ptr()
        a.events_u_upper = None if events_u_upper is None else events_u_upper.data_ptr()
    _check(_lib.rtc_gpc_step(ctypes.byref(a), _stream()))
    if alpha_l is not None:
        return alpha_u_out, beta_l_out, alpha_l_out, beta_u_out
    return alpha_u_out, beta_l_out


_closure_sig = [_vp, _vp, _i64, _i64, _int, _vp, _sz, _vp, _vp]
_lib.rtc_subadditive_closure.argtypes = _closure_sig
_lib.rtc_superadditive_closure.argtypes = _closure_sig
_lib.rtc_conv_chain.argtypes = [_vp, _i64, _vp, _i64, _i64, _int, _vp, _sz, _vp, _vp]
for _name in ("rtc_subadditive_closure", "rtc_superadditive_closure", "rtc_conv_chain"):
    getattr(_lib, _name).restype = _int


def _closure(fn, f, out, ws, dev_flags):
    f, batch, n = _dense(f)
    if out is None:
        out = torch.empty_like(f)
    ws, ws_bytes = _workspace(RTC_OP_CLOSURE, batch, n, f.dtype, f.device, ws)
    _check(fn(_ptr(f), _ptr(out), batch, n, _DT[f.dtype], _ptr(ws), ws_bytes, _ptr(dev_flags), _stream()))
    return out


def rtc_subadditive_closure(f, out=None, ws=None, dev_flags=None):
    """min(delta_0, f, f (x) f, ...) per row."""
    return _closure(_lib.rtc_subadditive_closure, f, out, ws, dev_flags)


def rtc_superadditive_closure(f, out=None, ws=None, dev_flags=None):
    """max(delta_0, f, f max-plus-convolved with itself, ...) per row."""
    return _closure(_lib.rtc_superadditive_closure, f, out, ws, dev_flags)


def rtc_conv_chain(curves, out=None, ws=None, dev_flags=None):
    """curves: dense [count][batch][n]; returns their min-plus convolution per row, [batch][n]."""
    if not curves.is_cuda or curves.dim() != 3 or not curves.is_contiguous():
        raise ValueError("curves must be a dense [count][batch][n] device tensor")
    count, batch, n = curves.shape
    if out is None:
        out = torch.empty((batch, n), dtype=curves.dtype, device=curves.device)
    ws, ws_bytes = _workspace(RTC_OP_CHAIN, batch, n, curves.dtype, curves.device, ws)
    _check(_lib.rtc_conv_chain(_ptr(curves), count, _ptr(out), batch, n, _DT[curves.dtype], _ptr(ws), ws_bytes,
                               _ptr(dev_flags), _stream()))
    return out


def rtc_max_hdev(alpha, beta, out=None, dev_flags=None):
    alpha, batch, n = _dense(alpha)
    beta = _dense(beta)[0]
    if beta.shape != alpha.shape or beta.dtype != alpha.dtype:
        raise ValueError("alpha and beta must have one shape and dtype")
    if out is None:
        out = torch.empty(batch, dtype=torch.int32, device=alpha.device)
    _check(_lib.rtc_max_hdev(_ptr(alpha), _ptr(beta), _ptr(out), batch, n, _DT[alpha.dtype],
                             _ptr(dev_flags), _stream()))
    return out


_lib.rtc_max_deviations.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _int, _vp, _vp]
_lib.rtc_max_deviations.restype = _int
RTC_PROFILE_KIND_TAIL = 64


def rtc_max_deviations(alpha, beta, out_h=None, out_v=None, dev_flags=None):
    """(delay bound, backlog bound) per row from one pass: rtc_max_hdev and rtc_max_vdev together."""
    alpha, batch, n = _dense(alpha)
    beta = _dense(beta)[0]
    if beta.shape != alpha.shape or beta.dtype != alpha.dtype:
        raise ValueError("alpha and beta must have one shape and dtype")
    if out_h is None:
        out_h = torch.empty(batch, dtype=torch.int32, device=alpha.device)
    if out_v is None:
        out_v = torch.empty(batch, dtype=alpha.dtype, device=alpha.device)
    _check(_lib.rtc_max_deviations(_ptr(alpha), _ptr(beta), _ptr(out_h), _ptr(out_v), batch, n, _DT[alpha.dtype],
                                   _ptr(dev_flags), _stream()))
    return out_h, out_v


def rtc_max_vdev(alpha, beta, out=None):
    alpha, batch, n = _dense(alpha)
    beta = _dense(beta)[0]
    if beta.shape != alpha.shape or beta.dtype != alpha.dtype:
        raise ValueError("alpha and beta must have one shape and dtype")
    if out is None:
        out = torch.empty(batch, dtype=alpha.dtype, device=alpha.device)
    _check(_lib.rtc_max_vdev(_ptr(alpha), _ptr(beta), _ptr(out), batch, n, _DT[alpha.dtype], _stream()))
    return out
