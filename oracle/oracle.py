"""ctypes loader for the CPU oracle (rtc_oracle.cpp).

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
_SRC = os.path.join(_HERE, "rtc_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

_DT = {np.dtype(np.int32): 0, np.dtype(np.int64): 1, np.dtype(np.float64): 2}

_LIB_CHECKED = os.path.join(_HERE, "liboracle_checked.so")

_libs = {}
_checked = False

_FLAGS = ["g++", "-std=c++17", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC"]


def build(force: bool = True) -> str:
    """Compile the oracle with g++ (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run([*_FLAGS, "-o", _LIB, _SRC], check=True)
    return _LIB


def build_checked(force: bool = True) -> str:
    """The debug build: every integer addition / subtraction of two samples is checked for overflow
    and counted (overflow_count); same loops, same results on inputs that obey the precondition."""
    if force or not os.path.exists(_LIB_CHECKED) or os.path.getmtime(_LIB_CHECKED) < os.path.getmtime(_SRC):
        subprocess.run([*_FLAGS, "-DORACLE_CHECK_OVERFLOW", "-o", _LIB_CHECKED, _SRC], check=True)
    return _LIB_CHECKED


def use_checked_build(on: bool) -> None:
    """Route every call of this module through the overflow-checking debug build (tests only)."""
    global _checked
    _checked = bool(on)


def lib():
    key = "checked" if _checked else "plain"
    if key not in _libs:
        path = build_checked(force=False) if _checked else build(force=False)
        handle = ctypes.CDLL(path)
        handle.oracle_num_threads.restype = ctypes.c_int
        handle.oracle_overflow_count.restype = ctypes.c_longlong
        handle.oracle_overflow_count.argtypes = [ctypes.c_int]
        _libs[key] = handle
    return _libs[key]


def overflow_count(reset: bool = True) -> int:
    """Overflowing sample additions / subtractions since the last reset; -1 in the normal build."""
    return int(lib().oracle_overflow_count(1 if reset else 0))


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _p(a):
    return ctypes.c_void_p(a.ctypes.data)


def _rows(a):
    a = np.ascontiguousarray(a)
    if a.ndim == 1:
        a = a[None, :]
    assert a.ndim == 2
    return a


def _binary(name, f, g):
    f = _rows(f)
    g = _rows(g)
    assert f.dtype == g.dtype and f.shape[1] == g.shape[1]
    batch = max(f.shape[0], g.shape[0])
    n = f.shape[1]
    sf = n if f.shape[0] == batch else 0
    sg = n if g.shape[0] == batch else 0
    assert (f.shape[0] in (1, batch)) and (g.shape[0] in (1, batch))
    out = np.empty((batch, n), f.dtype)
    rc = getattr(lib(), name)(_p(f), _p(g), _p(out), ctypes.c_int64(batch), ctypes.c_int64(n),
                              ctypes.c_int64(sf), ctypes.c_int64(sg), ctypes.c_int(_DT[f.dtype]))
    assert rc == 0, rc
    return out


def minplus_conv(f, g):
    return _binary("oracle_minplus_conv", f, g)


def maxplus_deconv(f, g):
    return _binary("oracle_maxplus_deconv", f, g)


def maxplus_conv(f, g):
    return _binary("oracle_maxplus_conv", f, g)


def minplus_deconv(f, g):
    return _binary("oracle_minplus_deconv", f, g)


def product_at(f, g, t_idx, deconv: bool):
    """Selected outputs of f (x) g (deconv=False) or f (/) g (deconv=True) for one row pair."""
    f = np.ascontiguousarray(f).reshape(-1)
    g = np.ascontiguousarray(g).reshape(-1)
    assert f.dtype == g.dtype and f.shape == g.shape
    t_idx = np.ascontiguousarray(t_idx, dtype=np.int64)
    out = np.empty(t_idx.shape, f.dtype)
    rc = lib().oracle_product_at(_p(f), _p(g), ctypes.c_int64(f.size), _p(t_idx), ctypes.c_int64(t_idx.size),
                                 _p(out), ctypes.c_int(1 if deconv else 0), ctypes.c_int(_DT[f.dtype]))
    assert rc == 0, rc
    return out


def pseudo_inverse(f, x, mode: int = 0):
    f = _rows(f)
    x = _rows(np.asarray(x, dtype=f.dtype))
    assert f.shape[0] == x.shape[0]
    out = np.empty(x.shape, np.int32)
    rc = lib().oracle_pseudo_inverse(_p(f), ctypes.c_int64(f.shape[1]), _p(x), ctypes.c_int64(x.shape[1]),
                                     _p(out), ctypes.c_int64(f.shape[0]), ctypes.c_int(mode),
                                     ctypes.c_int(_DT[f.dtype]))
    assert rc == 0, rc
    return out


def compose(outer, inner):
    outer = _rows(outer)
    inner = _rows(np.asarray(inner, dtype=np.int32))
    assert outer.shape[0] == inner.shape[0]
    out = np.empty(inner.shape, outer.dtype)
    flags = np.zeros(1, np.int32)
    rc = lib().oracle_compose(_p(outer), ctypes.c_int64(outer.shape[1]), _p(inner),
                              ctypes.c_int64(inner.shape[1]), _p(out), ctypes.c_int64(outer.shape[0]),
                              ctypes.c_int(_DT[outer.dtype]), _p(flags))
    assert rc == 0, rc
    return out, int(flags[0])


def gpc_step(alpha_u, beta_u, beta_l):
    """Returns (alpha'^u, beta'^l) of one greedy processing component per row."""
    a = _rows(alpha_u)
    u = _rows(beta_u)
    l = _rows(beta_l)
    assert a.shape == u.shape == l.shape and a.dtype == u.dtype == l.dtype
    ao = np.empty_like(a)
    lo = np.empty_like(a)
    tmp = np.empty_like(a)
    rc = lib().oracle_gpc_step(_p(a), _p(u), _p(l), _p(ao), _p(lo), _p(tmp), ctypes.c_int64(a.shape[0]),
                               ctypes.c_int64(a.shape[1]), ctypes.c_int(_DT[a.dtype]))
    assert rc == 0, rc
    return ao, lo


def gpc_step_lower(alpha_l, beta_u, beta_l):
    """Returns (alpha'^l, beta'^u) of one greedy processing component per row."""
    a = _rows(alpha_l)
    u = _rows(beta_u)
    l = _rows(beta_l)
    assert a.shape == u.shape == l.shape and a.dtype == u.dtype == l.dtype
    ao = np.empty_like(a)
    uo = np.empty_like(a)
    tmp = np.empty_like(a)
    rc = lib().oracle_gpc_step_lower(_p(a), _p(u), _p(l), _p(ao), _p(uo), _p(tmp), ctypes.c_int64(a.shape[0]),
                                     ctypes.c_int64(a.shape[1]), ctypes.c_int(_DT[a.dtype]))
    assert rc == 0, rc
    return ao, uo


def closure(f, super_additive: bool = False):
    """Sub-additive (default) or super-additive closure per row; returns (closure, flags)."""
    f = _rows(f)
    out = np.empty_like(f)
    scratch = np.empty(3 * f.shape[1], f.dtype)
    flags = np.zeros(1, np.int32)
    rc = lib().oracle_closure(_p(f), _p(out), _p(scratch), ctypes.c_int64(f.shape[0]), ctypes.c_int64(f.shape[1]),
                              ctypes.c_int(1 if super_additive else 0), ctypes.c_int(_DT[f.dtype]), _p(flags))
    assert rc == 0, rc
    return out, int(flags[0])


def conv_chain(curves):
    """curves: [count][batch][n]; their min-plus convolution per row."""
    c = np.ascontiguousarray(curves)
    assert c.ndim == 3
    out = np.empty(c.shape[1:], c.dtype)
    scratch = np.empty(c.shape[2], c.dtype)
    rc = lib().oracle_conv_chain(_p(c), ctypes.c_int64(c.shape[0]), _p(out), _p(scratch), ctypes.c_int64(c.shape[1]),
                                 ctypes.c_int64(c.shape[2]), ctypes.c_int(_DT[c.dtype]))
    assert rc == 0, rc
    return out


def max_hdev(alpha, beta):
    a = _rows(alpha)
    b = _rows(beta)
    assert a.shape == b.shape and a.dtype == b.dtype
    out = np.empty(a.shape[0], np.int32)
    flags = np.zeros(1, np.int32)
    rc = lib().oracle_max_hdev(_p(a), _p(b), _p(out), ctypes.c_int64(a.shape[0]), ctypes.c_int64(a.shape[1]),
                               ctypes.c_int(_DT[a.dtype]), _p(flags))
    assert rc == 0, rc
    return out, int(flags[0])


def max_vdev(alpha, beta):
    a = _rows(alpha)
    b = _rows(beta)
    assert a.shape == b.shape and a.dtype == b.dtype
    out = np.empty(a.shape[0], a.dtype)
    rc = lib().oracle_max_vdev(_p(a), _p(b), _p(out), ctypes.c_int64(a.shape[0]), ctypes.c_int64(a.shape[1]),
                               ctypes.c_int(_DT[a.dtype]))
    assert rc == 0, rc
    return out
