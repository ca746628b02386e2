"""Seeded synthetic curve generators for the five benchmark configurations.

This module only *constructs inputs*: sampled nondecreasing curves over
Delta = 0..N-1 (arrival curves alpha, service curves beta, workload curves
gamma, in the notation of the paper's curve macros).  It holds none of the
(min,+) operators; both the CPU oracle's tests and the HIP path's tests feed
from it so that they see identical data.

Random numbers: a counter-based splitmix64 (state_i = key + (i+1)*GOLDEN, then
the standard 64-bit finaliser).  Integers are drawn as ``x % range`` (the
modulo bias of at most range/2^64 is accepted), uniform doubles as
``(x >> 11) * 2**-53`` and Exp(1) as ``-log(1-u)``.  Every stream is keyed by
(seed, config id, stream id) so that curves of one configuration are
independent of each other and reproducible one by one.
"""
from __future__ import annotations

import numpy as np

DEFAULT_SEED = 20191204

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def stream(seed: int, config_id: int, stream_id: int, count: int) -> np.ndarray:
    """``count`` 64-bit words of the splitmix64 stream keyed by the triple."""
    with np.errstate(over="ignore"):
        key = np.array([(seed ^ (config_id << 32) ^ (stream_id * 0x632BE59BD9B4E019)) & (2**64 - 1)],
                       dtype=np.uint64)
        key = _mix(key + _GOLDEN)
        ctr = np.arange(1, count + 1, dtype=np.uint64)
        return _mix(key + ctr * _GOLDEN)


def uniform_int(words: np.ndarray, lo, hi) -> np.ndarray:
    """Map 64-bit words to integers uniform on {lo..hi} (inclusive), int64."""
    lo = np.asarray(lo, dtype=np.int64)
    hi = np.asarray(hi, dtype=np.int64)
    span = (hi - lo + 1).astype(np.uint64)
    return (words % span).astype(np.int64) + lo


def uniform_double(words: np.ndarray) -> np.ndarray:
    return (words >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


# ----------------------------------------------------------------------------
# elementary curve shapes (inputs only)
# ----------------------------------------------------------------------------

def token_bucket(n: int, b: int, r: int, dtype=np.int64, at_zero: bool = True) -> np.ndarray:
    """alpha[D] = b + r*D; ``at_zero=False`` gives the left-continuous variant alpha[0]=0."""
    d = np.arange(n, dtype=np.int64)
    a = b + r * d
    if not at_zero:
        a[0] = 0
    return a.astype(dtype)


def rate_latency(n: int, R, T, dtype=np.int64) -> np.ndarray:
    """beta[D] = R * max(0, D - T)."""
    d = np.arange(n, dtype=np.int64)
    return (R * np.maximum(0, d - T)).astype(dtype)


def periodic_jitter_upper(n: int, P: int, J: int) -> np.ndarray:
    """alpha^u[D] = ceil((D + J) / P), event counts (int64)."""
    d = np.arange(n, dtype=np.int64)
    return (d + J + P - 1) // P


def tdma_lower(n: int, s: int, c: int, bw: int = 1) -> np.ndarray:
    """Lower service curve of a slot of length s in a cycle of length c."""
    d = np.arange(n, dtype=np.int64)
    fl = d // c
    ce = (d + c - 1) // c
    return bw * np.maximum(fl * s, d - ce * (c - s))


def tdma_upper(n: int, s: int, c: int, bw: int = 1) -> np.ndarray:
    """Upper service curve of a slot of length s in a cycle of length c."""
    d = np.arange(n, dtype=np.int64)
    fl = d // c
    ce = (d + c - 1) // c
    return bw * np.minimum(ce * s, d - fl * (c - s))


def workload_curves(demands: np.ndarray):
    """gamma^u[k] / gamma^l[k] = sum of the k largest / smallest demands, k = 0..M."""
    asc = np.sort(np.asarray(demands, dtype=np.int64))
    gl = np.concatenate([[0], np.cumsum(asc)])
    gu = np.concatenate([[0], np.cumsum(asc[::-1])])
    return gu, gl


# ----------------------------------------------------------------------------
# the five configurations
# ----------------------------------------------------------------------------

def config1(seed: int = DEFAULT_SEED, n: int = 4096):
    """Single pair, int32: f = cumsum of U{0..8} increments, g = 3*(D-100)^+."""
    inc = uniform_int(stream(seed, 1, 0, n - 1), 0, 8) if n > 1 else np.zeros(0, np.int64)
    f = np.concatenate([[0], np.cumsum(inc)]).astype(np.int32)
    g = rate_latency(n, 3, 100, np.int32)
    return {"f": f[None, :].copy(), "g": g[None, :].copy()}


def config2(seed: int = DEFAULT_SEED, batch: int = 1024, n: int = 4096):
    """Batch of pairs, int32: periodic-with-jitter alpha^u and TDMA beta^l."""
    P = uniform_int(stream(seed, 2, 0, batch), 20, 200)
    J = uniform_int(stream(seed, 2, 1, batch), 0, P)
    s = uniform_int(stream(seed, 2, 2, batch), 10, 50)
    c = uniform_int(stream(seed, 2, 3, batch), s, 4 * s)
    alpha = np.empty((batch, n), np.int32)
    beta = np.empty((batch, n), np.int32)
    for b in range(batch):
        alpha[b] = periodic_jitter_upper(n, int(P[b]), int(J[b]))
        beta[b] = tdma_lower(n, int(s[b]), int(c[b]))
    return {"alpha_u": alpha, "beta_l": beta, "P": P, "J": J, "s": s, "c": c}


def _mixture_increments(words_sel: np.ndarray, words_val: np.ndarray) -> np.ndarray:
    sel = words_sel % np.uint64(100)
    small = uniform_int(words_val, 0, 4)
    burst = uniform_int(words_val, 50, 500)
    return np.where(sel < np.uint64(70), small, burst)


def config3(seed: int = DEFAULT_SEED, batch: int = 64, n: int = 65536, dtype=np.int64):
    """Pairs with 70% U{0..4} / 30% U{50..500} increments, f[0] = g[0] = 0."""
    out = {}
    for k, name in enumerate(("f", "g")):
        cur = np.zeros((batch, n), dtype)
        for b in range(batch):
            ws = stream(seed, 3, 4 * b + 2 * k, n - 1)
            wv = stream(seed, 3, 4 * b + 2 * k + 1, n - 1)
            cur[b, 1:] = np.cumsum(_mixture_increments(ws, wv))
        out[name] = cur
    return out


def config4(seed: int = DEFAULT_SEED, chains: int = 256, components: int = 16, n: int = 16384):
    """Chains of greedy processing components, int32.

    Per chain: event-domain arrival curve alpha_bar^u (periodic with jitter), a demand
    sequence of n-1 events in U{100..1000} cycles giving gamma^u / gamma^l with n samples.
    Per (component, chain): a TDMA resource (slot s, cycle c) of bandwidth Bw cycles per
    tick, Bw in U{200..400}, giving beta^u and beta^l in cycles.
    """
    P = uniform_int(stream(seed, 4, 0, chains), 20, 200)
    J = uniform_int(stream(seed, 4, 1, chains), 0, P)
    alpha_bar = np.empty((chains, n), np.int32)
    gamma_u = np.empty((chains, n), np.int32)
    gamma_l = np.empty((chains, n), np.int32)
    for ch in range(chains):
        alpha_bar[ch] = periodic_jitter_upper(n, int(P[ch]), int(J[ch]))
        dem = uniform_int(stream(seed, 4, 16 + ch, n - 1), 100, 1000)
        gu, gl = workload_curves(dem)
        gamma_u[ch] = gu
        gamma_l[ch] = gl
    tot = chains * components
    s = uniform_int(stream(seed, 4, 2, tot), 10, 50)
    c = uniform_int(stream(seed, 4, 3, tot), s, 4 * s)
    bw = uniform_int(stream(seed, 4, 4, tot), 200, 400)
    beta_u = np.empty((components, chains, n), np.int32)
    beta_l = np.empty((components, chains, n), np.int32)
    for i in range(components):
        for ch in range(chains):
            k = i * chains + ch
            beta_u[i, ch] = tdma_upper(n, int(s[k]), int(c[k]), int(bw[k]))
            beta_l[i, ch] = tdma_lower(n, int(s[k]), int(c[k]), int(bw[k]))
    return {"alpha_bar_u": alpha_bar, "gamma_u": gamma_u, "gamma_l": gamma_l,
            "beta_u": beta_u, "beta_l": beta_l}


def config5(seed: int = DEFAULT_SEED, n: int = 262144):
    """Single fp64 pair: f = cumsum Exp(1); g = 0.8*(D-1000)^+ + 0.01*D^1.5 (running max)."""
    u = uniform_double(stream(seed, 5, 0, n - 1))
    inc = -np.log1p(-u)
    f = np.concatenate([[0.0], np.cumsum(inc)])
    d = np.arange(n, dtype=np.float64)
    g = np.maximum(0.0, 0.8 * (d - 1000.0)) + 0.01 * np.power(d, 1.5)
    g = np.maximum.accumulate(g)
    x = d.copy()
    return {"f": f[None, :].copy(), "g": g[None, :].copy(), "x": x[None, :].copy()}


def random_monotone(seed: int, stream_id: int, batch: int, n: int, dtype, max_inc: int = 9,
                    start_max: int = 5) -> np.ndarray:
    """Generic nondecreasing test curves with a random starting value (ragged-size tests)."""
    w = stream(seed, 9, stream_id, batch * n).reshape(batch, n)
    if np.dtype(dtype) == np.float64:
        inc = uniform_double(w) * max_inc
        inc[:, 0] = uniform_double(w[:, 0]) * start_max
        return np.cumsum(inc, axis=1)
    inc = uniform_int(w, 0, max_inc)
    inc[:, 0] = uniform_int(w[:, 0], 0, start_max)
    return np.cumsum(inc, axis=1).astype(dtype)
