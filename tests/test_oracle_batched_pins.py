"""Pins for the row indexing of the CPU oracle's batched entry points.

Every function of the oracle that takes [batch][n] (or [count][batch][n]) arrays is called here
with at least three rows that all differ, and compared row by row with a pure-Python evaluation
of the definition on Python lists (no numpy arithmetic, no call into the oracle).  A slip in the
oracle's row offsets (a row read from the wrong place, `[batch][count]` taken for
`[count][batch]`, a broadcast stride applied to the wrong operand, the inverse's x rows of length
m indexed with n) changes at least one row of at least one case below.
"""
import numpy as np
import pytest

from oracle import oracle

DTYPES = [np.int32, np.int64, np.float64]


# ------------------------------------------------------------------ the definitions, on lists

def bf_conv(f, g):
    return [min(f[s] + g[t - s] for s in range(t + 1)) for t in range(len(f))]


def bf_deconv(f, g):
    n = len(f)
    return [max(f[t + u] - g[u] for u in range(n - t)) for t in range(n)]


def bf_maxconv(f, g):
    return [max(f[s] + g[t - s] for s in range(t + 1)) for t in range(len(f))]


def bf_mindeconv(f, g):
    n = len(f)
    return [min(f[t + u] - g[u] for u in range(n - t)) for t in range(n)]


def bf_pinv(f, x, mode):
    if mode == 0:
        ks = [k for k in range(len(f)) if f[k] >= x]
        return min(ks) if ks else len(f)
    ks = [k for k in range(len(f)) if f[k] <= x]
    return max(ks) if ks else -1


def bf_hdev(alpha, beta):
    n = len(alpha)
    return max(max(0, bf_pinv(beta, alpha[d], 0) - d) for d in range(n))


def bf_closure(f):
    """min over k >= 1 of the k-fold power of f with f[0] read as 0: by the recursion
    c[t] = min(f[t], min_{0<s<t} c[s] + c[t-s]), c[0] = 0."""
    n = len(f)
    c = [0] * n
    for t in range(1, n):
        c[t] = min([f[t]] + [c[s] + c[t - s] for s in range(1, t)])
    return c


def rows(rng, batch, n, dtype, hi=9, start_hi=5):
    """`batch` nondecreasing rows, all different (row b also gets its own slope)."""
    out = []
    for b in range(batch):
        if np.dtype(dtype) == np.float64:
            inc = rng.random(n) * (hi + b)
            inc[0] = rng.random() * start_hi
        else:
            inc = rng.integers(0, hi + 1 + b, n)
            inc[0] = rng.integers(0, start_hi + 1)
        out.append(np.cumsum(inc))
    a = np.stack(out).astype(dtype)
    for b in range(1, batch):
        assert not np.array_equal(a[b], a[0])
    return a


# ------------------------------------------------------------------ products, broadcast operands

@pytest.mark.parametrize("dtype", DTYPES)
def test_all_four_products_batched_and_with_either_operand_broadcast(dtype):
    rng = np.random.default_rng(301)
    batch, n = 4, 23
    F = rows(rng, batch, n, dtype)
    G = rows(rng, batch, n, dtype, hi=6)
    one = rows(rng, 1, n, dtype, hi=4)
    cases = [("minplus_conv", bf_conv), ("maxplus_deconv", bf_deconv), ("maxplus_conv", bf_maxconv),
             ("minplus_deconv", bf_mindeconv)]
    for name, bf in cases:
        fn = getattr(oracle, name)
        got = fn(F, G)
        for b in range(batch):
            assert got[b].tolist() == bf(F[b].tolist(), G[b].tolist()), (name, b)
        got = fn(F, one)                     # g shared by all rows
        for b in range(batch):
            assert got[b].tolist() == bf(F[b].tolist(), one[0].tolist()), (name, "g broadcast", b)
        got = fn(one, G)                     # f shared by all rows
        for b in range(batch):
            assert got[b].tolist() == bf(one[0].tolist(), G[b].tolist()), (name, "f broadcast", b)


# ------------------------------------------------------------------ pseudo-inverse, composition

@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("mode", [0, 1])
def test_pseudo_inverse_batched_with_m_different_from_n(dtype, mode):
    rng = np.random.default_rng(302)
    for batch, n, m in ((3, 17, 29), (5, 40, 7)):
        F = rows(rng, batch, n, dtype)
        top = float(F.max()) + 3
        if np.dtype(dtype) == np.float64:
            X = rng.random((batch, m)) * top - 1
            X[:, 0] = F[:, n // 2]          # hits a sample exactly
        else:
            X = rng.integers(-1, int(top) + 1, (batch, m))
        X = X.astype(dtype)
        got = oracle.pseudo_inverse(F, X, mode)
        assert got.shape == (batch, m) and got.dtype == np.int32
        for b in range(batch):
            want = [bf_pinv(F[b].tolist(), x, mode) for x in X[b].tolist()]
            assert got[b].tolist() == want, (batch, n, m, b)


@pytest.mark.parametrize("dtype", DTYPES)
def test_compose_batched_with_n_outer_different_from_n(dtype):
    rng = np.random.default_rng(303)
    for batch, k, n in ((3, 11, 26), (4, 30, 9)):
        outer = rows(rng, batch, k, dtype)
        inner = np.sort(rng.integers(0, k, (batch, n)), axis=1).astype(np.int32)
        got, fl = oracle.compose(outer, inner)
        assert fl == 0
        for b in range(batch):
            assert got[b].tolist() == [outer[b].tolist()[i] for i in inner[b].tolist()], (batch, k, n, b)
        # out-of-range indices in one row only: clamped there, flagged, other rows untouched
        inner2 = inner.copy()
        inner2[1, 0] = -4
        inner2[1, -1] = k + 5
        got2, fl2 = oracle.compose(outer, inner2)
        assert fl2 == 2
        for b in range(batch):
            want = [outer[b].tolist()[min(max(i, 0), k - 1)] for i in inner2[b].tolist()]
            assert got2[b].tolist() == want


# ------------------------------------------------------------------ component step, both sides

@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_gpc_step_batched(dtype):
    rng = np.random.default_rng(304)
    batch, n = 4, 21
    A = rows(rng, batch, n, dtype, hi=5)
    BU = rows(rng, batch, n, dtype, hi=12, start_hi=0)
    BL = np.minimum(BU, rows(rng, batch, n, dtype, hi=8, start_hi=0)).astype(dtype)
    au, bl = oracle.gpc_step(A, BU, BL)
    for b in range(batch):
        a, u, l = A[b].tolist(), BU[b].tolist(), BL[b].tolist()
        d = bf_deconv(bf_conv(a, u), l)
        assert au[b].tolist() == [min(x, y) for x, y in zip(d, u)], b
        want = [max(0, max(l[j] - a[j] for j in range(k + 1))) for k in range(n)]
        assert bl[b].tolist() == want, b


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_gpc_step_lower_batched(dtype):
    rng = np.random.default_rng(305)
    batch, n = 3, 24
    AL = rows(rng, batch, n, dtype, hi=3, start_hi=0)
    BU = rows(rng, batch, n, dtype, hi=12, start_hi=2)
    BL = np.minimum(BU, rows(rng, batch, n, dtype, hi=8, start_hi=0)).astype(dtype)
    al, bu = oracle.gpc_step_lower(AL, BU, BL)
    for b in range(batch):
        a, u, l = AL[b].tolist(), BU[b].tolist(), BL[b].tolist()
        c = bf_conv(bf_deconv(a, u), l)
        assert al[b].tolist() == [min(x, y) for x, y in zip(c, l)], b
        want = [max(0, min(u[j] - a[j] for j in range(k, n))) for k in range(n)]
        assert bu[b].tolist() == want, b


def test_gpc_step_batched_fp64_rounds_each_candidate_once():
    """fp64 rows: the same comparison, with the brute force in Python floats (IEEE doubles: each
    candidate is one rounded add or subtract, exactly as the definition is evaluated)."""
    rng = np.random.default_rng(306)
    batch, n = 3, 19
    A = rows(rng, batch, n, np.float64, hi=5)
    BU = rows(rng, batch, n, np.float64, hi=12, start_hi=0)
    BL = np.minimum(BU, rows(rng, batch, n, np.float64, hi=8, start_hi=0))
    au, bl = oracle.gpc_step(A, BU, BL)
    for b in range(batch):
        a, u, l = A[b].tolist(), BU[b].tolist(), BL[b].tolist()
        d = bf_deconv(bf_conv(a, u), l)
        assert au[b].tolist() == [min(x, y) for x, y in zip(d, u)]
        assert bl[b].tolist() == [max(0.0, max(l[j] - a[j] for j in range(k + 1))) for k in range(n)]


# ------------------------------------------------------------------ closures, chains

@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_closures_batched(dtype):
    rng = np.random.default_rng(307)
    batch, n = 4, 18
    F = np.stack([rng.integers(0, 40 + 25 * b, n) for b in range(batch)]).astype(dtype)
    F[2, 0] = -3                                     # one row breaks the precondition: flagged, read as 0
    got, fl = oracle.closure(F)
    assert fl == 2
    for b in range(batch):
        assert got[b].tolist() == bf_closure(F[b].tolist()), b
    sup, fl = oracle.closure(-F, super_additive=True)
    assert fl == 2
    for b in range(batch):
        assert sup[b].tolist() == [-v for v in bf_closure(F[b].tolist())], b


@pytest.mark.parametrize("dtype", DTYPES)
def test_conv_chain_layout_is_count_major(dtype):
    """curves[k][b] is the k-th curve of row b.  count = 4 and batch = 3 differ, all twelve curves
    differ, and for fp64 the left-to-right order of the products is part of the result."""
    rng = np.random.default_rng(308)
    count, batch, n = 4, 3, 16
    C = rows(rng, count * batch, n, dtype, hi=7).reshape(count, batch, n)
    got = oracle.conv_chain(C)
    assert got.shape == (batch, n)
    for b in range(batch):
        acc = C[0, b].tolist()
        for k in range(1, count):
            acc = bf_conv(acc, C[k, b].tolist())
        assert got[b].tolist() == acc, b
    # and the transposed reading gives something else (so the test can tell them apart)
    wrong = C.reshape(batch, count, n)
    acc = wrong[0, 0].tolist()
    for k in range(1, count):
        acc = bf_conv(acc, wrong[0, k].tolist())
    assert got[0].tolist() != acc
    # count = 1 returns the curves themselves, count = 2 one product per row
    assert np.array_equal(oracle.conv_chain(C[:1]), C[0])
    two = oracle.conv_chain(C[:2])
    for b in range(batch):
        assert two[b].tolist() == bf_conv(C[0, b].tolist(), C[1, b].tolist())


# ------------------------------------------------------------------ deviations

@pytest.mark.parametrize("dtype", DTYPES)
def test_deviations_batched(dtype):
    rng = np.random.default_rng(309)
    batch, n = 5, 33
    A = rows(rng, batch, n, dtype, hi=4)
    B = rows(rng, batch, n, dtype, hi=9, start_hi=0)
    B[3] = np.minimum(B[3], A[3, n // 2])            # row 3 never reaches the end of alpha: unbounded
    h, fl = oracle.max_hdev(A, B)
    v = oracle.max_vdev(A, B)
    assert h.shape == (batch,) and v.shape == (batch,)
    assert fl == 4
    for b in range(batch):
        a, be = A[b].tolist(), B[b].tolist()
        assert int(h[b]) == bf_hdev(a, be), b
        assert v[b].tolist() == max(x - y for x, y in zip(a, be)), b
    # without the unbounded row the flag stays clear
    keep = [0, 1, 2, 4]
    h2, fl2 = oracle.max_hdev(A[keep], B[keep])
    if all(B[b, -1] >= A[b, -1] for b in keep):
        assert fl2 == 0
    assert h2.tolist() == [int(h[b]) for b in keep]
