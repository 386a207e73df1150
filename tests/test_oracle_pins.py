"""Pins of the CPU oracle (no GPU): the oracle is checked against things that
are not the oracle — exact rational arithmetic on tiny integer inputs, numpy
products on the explicitly completed matrix, closed forms (A = I, A = ones),
the alpha = 0 / beta = 0 conventions, transpose identities and NaN poison in
the triangle that must never be read.  Each pin names the mistake it catches.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import MODE_ABS, MODE_W, MODE_X

PRECS = "sdcz"
REAL = {"s": np.float32, "d": np.float64, "c": np.float32, "z": np.float64}
# relative tolerance of a MODE_X result against a float64/complex128 numpy product
XTOL = {"s": 1e-13, "d": 1e-13, "c": 1e-13, "z": 1e-13}


def rnd(rng, prec, shape, lo=-1.0, hi=1.0):
    dt = oracle.DTYPES[prec]
    a = rng.uniform(lo, hi, shape)
    if prec in "cz":
        a = a + 1j * rng.uniform(lo, hi, shape)
    return a.astype(dt)


def rnd_int(rng, prec, shape):
    dt = oracle.DTYPES[prec]
    a = rng.integers(-3, 4, shape).astype(np.float64)
    if prec in "cz":
        a = a + 1j * rng.integers(-3, 4, shape)
    return a.astype(dt)


def colmajor(a2d, lda=None, fill=np.nan):
    """flat column-major buffer with leading dimension lda (padding = NaN)"""
    m, n = a2d.shape
    lda = max(1, m) if lda is None else lda
    buf = np.full((n, lda), fill, dtype=a2d.dtype)
    buf[:, :m] = a2d.T
    return buf.reshape(-1), lda


def strided(v, inc, fill=np.nan):
    """storage of logical vector v with BLAS increment inc (negative = reversed)"""
    n = v.size
    ext = 0 if n == 0 else 1 + (n - 1) * abs(inc)
    buf = np.full(ext, fill, dtype=v.dtype)
    if n:
        buf[:: abs(inc)] = v if inc > 0 else v[::-1]
    return buf


def logical(buf, n, inc):
    v = buf[:: abs(inc)][:n]
    return v if inc > 0 else v[::-1]


def complete(A, uplo, herm):
    """full symmetric / Hermitian matrix from the stored triangle (numpy only)"""
    if uplo == "L":
        strict = np.tril(A, -1)
    else:
        strict = np.triu(A, 1)
    d = np.diag(np.diag(A).real if herm else np.diag(A)).astype(A.dtype)
    other = strict.conj().T if herm else strict.T
    return strict + d + other


def poison(A, uplo):
    B = A.copy()
    n = A.shape[0]
    i, j = np.indices((n, n))
    B[(i < j) if uplo == "L" else (i > j)] = np.nan
    return B


# --------------------------------------------------------------------------
# 1. exact rational brute force on tiny integer inputs: catches a dropped term,
#    a wrong index, a missing conjugation, a wrong increment rule.
# --------------------------------------------------------------------------
def frac(v):
    v = complex(v)
    return (Fraction(int(v.real)), Fraction(int(v.imag)))


def as_dtype(v, dt):
    v = np.asarray(v)
    if np.issubdtype(dt, np.complexfloating):
        return v.astype(dt)
    assert np.all(v.imag == 0)
    return v.real.astype(dt)


def cmul(a, b):
    return (a[0] * b[0] - a[1] * b[1], a[0] * b[1] + a[1] * b[0])


def cadd(a, b):
    return (a[0] + b[0], a[1] + b[1])


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("trans", "NTC")
@pytest.mark.parametrize("incx,incy", [(1, 1), (2, 3), (-1, -2)])
def test_gemv_exact_rational(prec, trans, incx, incy):
    rng = np.random.default_rng(11)
    m, n = 5, 7
    A = rnd_int(rng, prec, (m, n))
    leny, lenx = (m, n) if trans == "N" else (n, m)
    x, y = rnd_int(rng, prec, lenx), rnd_int(rng, prec, leny)
    alpha, beta = (2 - 1j, -3 + 2j) if prec in "cz" else (2, -3)
    want = []
    for k in range(leny):
        acc = (Fraction(0), Fraction(0))
        for l in range(lenx):
            a = A[k, l] if trans == "N" else A[l, k]
            if trans == "C":
                a = np.conj(a)
            acc = cadd(acc, cmul(frac(a), frac(x[l])))
        r = cadd(cmul(frac(alpha), acc), cmul(frac(beta), frac(y[k])))
        want.append(complex(float(r[0]), float(r[1])))
    want = np.array(want)
    Af, lda = colmajor(A, lda=m + 3)
    for mode in (MODE_W, MODE_X):
        got = oracle.gemv(prec, trans, m, n, alpha, Af, strided(x, incx), beta, strided(y, incy),
                          lda=lda, incx=incx, incy=incy, mode=mode)
        assert np.array_equal(logical(got, leny, incy), as_dtype(want, got.dtype))


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("uplo", "LU")
def test_symv_exact_rational(prec, uplo):
    rng = np.random.default_rng(12)
    n = 6
    herm = prec in "cz"
    A = rnd_int(rng, prec, (n, n))          # diagonal has a non-zero imaginary part for c/z
    x, y = rnd_int(rng, prec, n), rnd_int(rng, prec, n)
    alpha, beta = (1 + 2j, 3 - 1j) if herm else (-2, 3)
    want = []
    for i in range(n):
        acc = (Fraction(0), Fraction(0))
        for j in range(n):
            if i == j:
                s = frac(A[i, i].real) if herm else frac(A[i, i])
            else:
                stored = (i > j) if uplo == "L" else (i < j)
                if stored:
                    s = frac(A[i, j])
                else:
                    s = frac(np.conj(A[j, i]) if herm else A[j, i])
            acc = cadd(acc, cmul(s, frac(x[j])))
        r = cadd(cmul(frac(alpha), acc), cmul(frac(beta), frac(y[i])))
        want.append(complex(float(r[0]), float(r[1])))
    want = np.array(want)
    Af, lda = colmajor(poison(A, uplo), lda=n + 2)
    for mode in (MODE_W, MODE_X):
        got = oracle.symv(prec, uplo, n, alpha, Af, x, beta, y, lda=lda, mode=mode)
        assert np.array_equal(got, as_dtype(want, got.dtype))


# --------------------------------------------------------------------------
# 2. numpy products on random data (library routine, different code path):
#    catches a transposed operand, wrong lda handling, wrong stride handling.
# --------------------------------------------------------------------------
@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("trans", "NTC")
@pytest.mark.parametrize("m,n", [(1, 1), (3, 17), (64, 65), (129, 31), (257, 300)])
def test_gemv_vs_numpy(prec, trans, m, n):
    rng = np.random.default_rng(m * 1000 + n)
    A = rnd(rng, prec, (m, n))
    leny, lenx = (m, n) if trans == "N" else (n, m)
    x, y = rnd(rng, prec, lenx), rnd(rng, prec, leny)
    alpha, beta = (1.5 - 0.25j, 0.5 + 0.75j) if prec in "cz" else (1.5, 0.5)
    A64 = A.astype(np.complex128 if prec in "cz" else np.float64)
    op = {"N": A64, "T": A64.T, "C": A64.conj().T}[trans]
    al = oracle.DTYPES[prec].type(alpha)
    be = oracle.DTYPES[prec].type(beta)
    want = complex(al) * (op @ x.astype(A64.dtype)) + complex(be) * y.astype(A64.dtype) if prec in "cz" else \
        float(al) * (op @ x.astype(np.float64)) + float(be) * y.astype(np.float64)
    for incx, incy, lda in [(1, 1, None), (2, 1, m + 5), (-3, -2, m + 1)]:
        Af, ld = colmajor(A, lda=lda)
        got = oracle.gemv(prec, trans, m, n, alpha, Af, strided(x, incx), beta, strided(y, incy),
                          lda=ld, incx=incx, incy=incy, mode=MODE_X)
        g = logical(got, leny, incy)
        assert np.linalg.norm(g - want) <= XTOL[prec] * np.linalg.norm(want)
        # working-precision mode agrees to working precision
        gw = logical(oracle.gemv(prec, trans, m, n, alpha, Af, strided(x, incx), beta, strided(y, incy),
                                 lda=ld, incx=incx, incy=incy, mode=MODE_W), leny, incy)
        eps = np.finfo(REAL[prec]).eps
        assert np.linalg.norm(gw - want) <= 4 * (lenx + 2) * eps * np.linalg.norm(want) + 1e-30
    # the wrong operand is far away: this pin can tell N from T
    if m == n and n > 1:
        wrong = oracle.gemv(prec, "T" if trans == "N" else "N", m, n, alpha, colmajor(A)[0], x, beta, y, lda=m)
        assert np.linalg.norm(wrong - want) > 1e-3 * np.linalg.norm(want)


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("uplo", "LU")
@pytest.mark.parametrize("n", [1, 2, 5, 64, 65, 200])
def test_symv_vs_numpy_on_completed_matrix(prec, uplo, n):
    rng = np.random.default_rng(n)
    herm = prec in "cz"
    A = rnd(rng, prec, (n, n))      # complex diagonal carries a garbage imaginary part
    x, y = rnd(rng, prec, n), rnd(rng, prec, n)
    alpha, beta = (0.7 + 0.1j, 0.3 - 0.2j) if herm else (0.7, 0.3)
    wide = np.complex128 if herm else np.float64
    S = complete(A.astype(wide), uplo, herm)
    al, be = oracle.DTYPES[prec].type(alpha), oracle.DTYPES[prec].type(beta)
    want = wide(al) * (S @ x.astype(wide)) + wide(be) * y.astype(wide)
    for incx, incy, lda in [(1, 1, None), (2, -1, n + 7)]:
        Af, ld = colmajor(poison(A, uplo), lda=lda)
        got = oracle.symv(prec, uplo, n, alpha, Af, strided(x, incx), beta, strided(y, incy),
                          lda=ld, incx=incx, incy=incy, mode=MODE_X)
        g = logical(got, n, incy)
        assert np.all(np.isfinite(g)), "the poisoned triangle or padding was read"
        assert np.linalg.norm(g - want) <= XTOL[prec] * np.linalg.norm(want)
    # completed-matrix GEMV through the oracle itself gives the identical sums
    Sf, _ = colmajor(S.astype(oracle.DTYPES[prec]))
    via_gemv = oracle.gemv(prec, "N", n, n, alpha, Sf, x, beta, y, lda=n, mode=MODE_W)
    via_symv = oracle.symv(prec, uplo, n, alpha, colmajor(poison(A, uplo))[0], x, beta, y, lda=n, mode=MODE_W)
    assert np.array_equal(via_gemv, via_symv)


# --------------------------------------------------------------------------
# 3. closed forms
# --------------------------------------------------------------------------
@pytest.mark.parametrize("prec", PRECS)
def test_identity_matrix(prec):
    rng = np.random.default_rng(3)
    n = 37
    dt = oracle.DTYPES[prec]
    I = np.eye(n, dtype=dt)
    x, y = rnd(rng, prec, n), rnd(rng, prec, n)
    alpha, beta = 2.0, 0.5     # powers of two: alpha*x + beta*y has one rounding
    want = (dt.type(alpha) * x + dt.type(beta) * y).astype(dt)
    for trans in "NTC":
        got = oracle.gemv(prec, trans, n, n, alpha, colmajor(I)[0], x, beta, y, lda=n, mode=MODE_W)
        assert np.array_equal(got, want)
    for uplo in "LU":
        got = oracle.symv(prec, uplo, n, alpha, colmajor(poison(I, uplo))[0], x, beta, y, lda=n, mode=MODE_W)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("prec", PRECS)
def test_ones_matrix_integer_x_is_exact(prec):
    rng = np.random.default_rng(4)
    m, n = 70, 129
    dt = oracle.DTYPES[prec]
    x = rnd_int(rng, prec, n)
    y = rnd_int(rng, prec, m)
    A = np.ones((m, n), dtype=dt)
    want = (2 * x.sum() + 4 * y).astype(dt)
    got = oracle.gemv(prec, "N", m, n, 2, colmajor(A)[0], x, 4, y, lda=m, mode=MODE_W)
    assert np.array_equal(got, want)
    # transposed: every y_j = alpha*sum(x) + beta*y_j
    xt, yt = rnd_int(rng, prec, m), rnd_int(rng, prec, n)
    got = oracle.gemv(prec, "T", m, n, 2, colmajor(A)[0], xt, 4, yt, lda=m, mode=MODE_W)
    assert np.array_equal(got, (2 * xt.sum() + 4 * yt).astype(dt))
    S = np.ones((n, n), dtype=dt)
    for uplo in "LU":
        got = oracle.symv(prec, uplo, n, 2, colmajor(poison(S, uplo))[0], x, 4, rnd_int(rng, prec, n) * 0, lda=n, mode=MODE_W)
        assert np.array_equal(got, np.full(n, 2 * x.sum(), dtype=dt))


# --------------------------------------------------------------------------
# 4. alpha = 0 and beta = 0 conventions
# --------------------------------------------------------------------------
@pytest.mark.parametrize("prec", PRECS)
def test_alpha_zero_never_reads_A_or_x(prec):
    rng = np.random.default_rng(5)
    m, n = 9, 6
    dt = oracle.DTYPES[prec]
    A = np.full((m, n), np.nan, dtype=dt)
    y = rnd(rng, prec, m)
    got = oracle.gemv(prec, "N", m, n, 0, colmajor(A)[0], np.full(n, np.nan, dtype=dt), 0.5, y, lda=m, mode=MODE_W)
    assert np.array_equal(got, (dt.type(0.5) * y).astype(dt))
    S = np.full((m, m), np.nan, dtype=dt)
    got = oracle.symv(prec, "L", m, 0, colmajor(S)[0], np.full(m, np.nan, dtype=dt), 0.5, y, lda=m, mode=MODE_W)
    assert np.array_equal(got, (dt.type(0.5) * y).astype(dt))


@pytest.mark.parametrize("prec", PRECS)
def test_beta_zero_never_reads_y(prec):
    rng = np.random.default_rng(6)
    m, n = 8, 5
    dt = oracle.DTYPES[prec]
    A, x = rnd(rng, prec, (m, n)), rnd(rng, prec, n)
    ynan = np.full(m, np.nan, dtype=dt)
    got = oracle.gemv(prec, "N", m, n, 1.0, colmajor(A)[0], x, 0, ynan, lda=m, mode=MODE_X)
    ref = oracle.gemv(prec, "N", m, n, 1.0, colmajor(A)[0], x, 0, np.zeros(m, dtype=dt), lda=m, mode=MODE_X)
    assert np.all(np.isfinite(got)) and np.array_equal(got, ref)
    S = rnd(rng, prec, (m, m))
    xs = rnd(rng, prec, m)
    got = oracle.symv(prec, "U", m, 1.0, colmajor(poison(S, "U"))[0], xs, 0, ynan, lda=m, mode=MODE_X)
    assert np.all(np.isfinite(got))


# --------------------------------------------------------------------------
# 5. transpose identities on tiny sizes (bitwise: same sums in the same order)
# --------------------------------------------------------------------------
SIZES = [1, 2, 3, 5, 8, 31, 32, 33, 63, 64, 65, 127, 128, 129]


@pytest.mark.parametrize("prec", PRECS)
def test_trans_equals_explicit_transpose(prec):
    rng = np.random.default_rng(7)
    for m in SIZES[::2]:
        for n in SIZES[1::3]:
            A = rnd(rng, prec, (m, n))
            x, y = rnd(rng, prec, m), rnd(rng, prec, n)
            t = oracle.gemv(prec, "T", m, n, 0.7, colmajor(A)[0], x, 0.3, y, lda=m, mode=MODE_W)
            nt = oracle.gemv(prec, "N", n, m, 0.7, colmajor(np.ascontiguousarray(A.T))[0], x, 0.3, y, lda=n, mode=MODE_W)
            assert np.array_equal(t, nt)
            c = oracle.gemv(prec, "C", m, n, 0.7, colmajor(A)[0], x, 0.3, y, lda=m, mode=MODE_W)
            nc = oracle.gemv(prec, "N", n, m, 0.7, colmajor(np.ascontiguousarray(A.conj().T))[0], x, 0.3, y, lda=n, mode=MODE_W)
            assert np.array_equal(c, nc)


@pytest.mark.parametrize("prec", PRECS)
def test_symv_lower_equals_upper_equals_gemv(prec):
    rng = np.random.default_rng(8)
    herm = prec in "cz"
    for n in SIZES:
        A = rnd(rng, prec, (n, n))
        S = complete(A, "L", herm)                     # a symmetric / Hermitian matrix, real diagonal
        x, y = rnd(rng, prec, n), rnd(rng, prec, n)
        lo = oracle.symv(prec, "L", n, 0.7, colmajor(poison(S, "L"))[0], x, 0.3, y, lda=n, mode=MODE_W)
        up = oracle.symv(prec, "U", n, 0.7, colmajor(poison(S, "U"))[0], x, 0.3, y, lda=n, mode=MODE_W)
        ge = oracle.gemv(prec, "N", n, n, 0.7, colmajor(S)[0], x, 0.3, y, lda=n, mode=MODE_W)
        assert np.array_equal(lo, up) and np.array_equal(lo, ge)


# --------------------------------------------------------------------------
# 6. invariants
# --------------------------------------------------------------------------
@pytest.mark.parametrize("prec", "cz")
def test_hemv_quadratic_form_is_real_and_diag_imag_ignored(prec):
    rng = np.random.default_rng(9)
    n = 90
    A = rnd(rng, prec, (n, n))
    x = rnd(rng, prec, n)
    zero = np.zeros(n, dtype=A.dtype)
    Ax = oracle.symv(prec, "L", n, 1.0, colmajor(poison(A, "L"))[0], x, 0, zero, lda=n, mode=MODE_X)
    q = np.vdot(x.astype(np.complex128), Ax)
    assert abs(q.imag) <= 1e-12 * abs(q)
    B = A.copy()
    d = np.arange(n)
    B.imag[d, d] = np.nan                     # NaN imaginary part on the diagonal only
    assert np.all(np.isfinite(B.real[d, d]))
    Bx = oracle.symv(prec, "L", n, 1.0, colmajor(poison(B, "L"))[0], x, 0, zero, lda=n, mode=MODE_X)
    assert np.array_equal(Ax, Bx)


@pytest.mark.parametrize("prec", "sd")
def test_symv_bilinear_symmetry(prec):
    rng = np.random.default_rng(10)
    n = 77
    A = rnd(rng, prec, (n, n))
    x1, x2 = rnd(rng, prec, n), rnd(rng, prec, n)
    zero = np.zeros(n, dtype=A.dtype)
    Af = colmajor(poison(A, "U"))[0]
    a = np.dot(x1.astype(np.float64), oracle.symv(prec, "U", n, 1.0, Af, x2, 0, zero, lda=n))
    b = np.dot(x2.astype(np.float64), oracle.symv(prec, "U", n, 1.0, Af, x1, 0, zero, lda=n))
    assert abs(a - b) <= 1e-12 * max(abs(a), 1.0)


# --------------------------------------------------------------------------
# 7. the error-bound denominator and the sampled-output interface
# --------------------------------------------------------------------------
@pytest.mark.parametrize("prec", PRECS)
def test_abs_mode_and_sampling(prec):
    rng = np.random.default_rng(13)
    m, n = 40, 23
    A, x, y = rnd(rng, prec, (m, n)), rnd(rng, prec, n), rnd(rng, prec, m)
    alpha, beta = 0.7, 0.3
    dt = oracle.DTYPES[prec]
    got = oracle.gemv(prec, "N", m, n, alpha, colmajor(A)[0], x, beta, y, lda=m, mode=MODE_ABS)
    want = abs(dt.type(alpha)) * (np.abs(A).astype(np.float64) @ np.abs(x).astype(np.float64)) \
        + abs(dt.type(beta)) * np.abs(y).astype(np.float64)
    assert np.allclose(got, want, rtol=1e-6)
    full = oracle.gemv(prec, "N", m, n, alpha, colmajor(A)[0], x, beta, y, lda=m, mode=MODE_X)
    idx = np.array([0, 7, 39])
    part = oracle.gemv(prec, "N", m, n, alpha, colmajor(A)[0], x, beta, y, lda=m, mode=MODE_X, sample=idx)
    assert np.array_equal(part[idx], full[idx])
    untouched = np.setdiff1d(np.arange(m), idx)
    assert np.array_equal(part[untouched], y.astype(part.dtype)[untouched])
    S = rnd(rng, prec, (m, m))
    xs = rnd(rng, prec, m)
    fulls = oracle.symv(prec, "L", m, alpha, colmajor(poison(S, "L"))[0], xs, beta, y, lda=m, mode=MODE_X)
    parts = oracle.symv(prec, "L", m, alpha, colmajor(poison(S, "L"))[0], xs, beta, y, lda=m, mode=MODE_X, sample=idx)
    assert np.array_equal(parts[idx], fulls[idx])


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("trans", "TC")
def test_abs_mode_of_transposed_gemv(prec, trans):
    """|alpha| (|A|^T |x|) + |beta| |y| from numpy on a rectangular matrix with a padded leading dimension and
    strided vectors: an ABS loop that walked rows for columns, or used the wrong vector lengths, fails"""
    rng = np.random.default_rng(17)
    m, n = 37, 22
    A, x, y = rnd(rng, prec, (m, n)), rnd(rng, prec, m), rnd(rng, prec, n)
    alpha, beta = (-0.7 + 0.4j, 0.3 - 0.2j) if prec in "cz" else (-0.7, 0.3)
    Af, lda = colmajor(A, lda=m + 5)
    got = logical(oracle.gemv(prec, trans, m, n, alpha, Af, strided(x, 2), beta, strided(y, -3), lda=lda, incx=2, incy=-3,
                              mode=MODE_ABS), n, -3)
    want = abs(alpha) * (np.abs(A).astype(np.float64).T @ np.abs(x).astype(np.float64)) + abs(beta) * np.abs(y).astype(np.float64)
    assert np.allclose(got.real, want, rtol=1e-6) and np.all(np.isfinite(got.real))


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("uplo", "LU")
def test_abs_mode_of_symv_on_the_completed_matrix(prec, uplo):
    """ABS mode of SYMV / HEMV (and of the complex symmetric product) against numpy on |S|, S completed from the
    stored triangle, with the OTHER triangle and the padding NaN in what the oracle sees: a loop that indexed the
    wrong triangle returns NaN, one that dropped the mirrored part or counted the diagonal twice misses the
    value; HEMV takes |Re a_ii| on the diagonal, the symmetric product |a_ii|"""
    rng = np.random.default_rng(19)
    n = 61
    A, x, y = rnd(rng, prec, (n, n)), rnd(rng, prec, n), rnd(rng, prec, n)
    alpha, beta = (0.6 - 0.8j, -0.5j) if prec in "cz" else (-1.25, 0.5)
    Af, lda = colmajor(poison(A, uplo), lda=n + 3)
    variants = [(False, prec in "cz")] + ([(True, False)] if prec in "cz" else [])
    for csym, herm in variants:
        S = complete(A, uplo, herm)
        want = abs(alpha) * (np.abs(S).astype(np.float64) @ np.abs(x).astype(np.float64)) + abs(beta) * np.abs(y).astype(np.float64)
        got = oracle.symv(prec, uplo, n, alpha, Af, x, beta, y, lda=lda, mode=MODE_ABS, complex_symmetric=csym)
        assert np.all(np.isfinite(got.real)), "the ABS loop touched the unreferenced triangle or the padding"
        assert np.allclose(got.real, want, rtol=1e-6), (csym, np.max(np.abs(got.real - want)))
    if prec in "cz":
        # the two diagonal rules differ when the diagonal has an imaginary part
        h = oracle.symv(prec, uplo, n, alpha, Af, x, beta, y, lda=lda, mode=MODE_ABS)
        c = oracle.symv(prec, uplo, n, alpha, Af, x, beta, y, lda=lda, mode=MODE_ABS, complex_symmetric=True)
        assert np.all(c.real >= h.real) and np.any(c.real > h.real)


# --------------------------------------------------------------------------
# 8. complex symmetric SYMV (prec c,z): the s,d rule applied to complex data.
#    Pinned apart from HEMV so that a conjugation left in, or the diagonal's
#    imaginary part dropped, fails.
# --------------------------------------------------------------------------
@pytest.mark.parametrize("prec", "cz")
@pytest.mark.parametrize("uplo", "LU")
def test_complex_symmetric_exact_rational(prec, uplo):
    rng = np.random.default_rng(21)
    n = 6
    A = rnd_int(rng, prec, (n, n))
    x, y = rnd_int(rng, prec, n), rnd_int(rng, prec, n)
    alpha, beta = 2 - 1j, -1 + 3j
    want = []
    for i in range(n):
        acc = (Fraction(0), Fraction(0))
        for j in range(n):
            stored = (i == j) or ((i > j) if uplo == "L" else (i < j))
            acc = cadd(acc, cmul(frac(A[i, j] if stored else A[j, i]), frac(x[j])))
        r = cadd(cmul(frac(alpha), acc), cmul(frac(beta), frac(y[i])))
        want.append(complex(float(r[0]), float(r[1])))
    want = np.array(want)
    Af, lda = colmajor(poison(A, uplo), lda=n + 3)
    for mode in (MODE_W, MODE_X):
        got = oracle.csymv(prec, uplo, n, alpha, Af, x, beta, y, lda=lda, mode=mode)
        assert np.array_equal(got, as_dtype(want, got.dtype))
    herm = oracle.symv(prec, uplo, n, alpha, Af, x, beta, y, lda=lda, mode=MODE_X)
    assert not np.array_equal(herm, want), "inputs do not tell the two products apart"


@pytest.mark.parametrize("prec", "cz")
@pytest.mark.parametrize("uplo", "LU")
@pytest.mark.parametrize("n", [1, 2, 5, 64, 65, 200])
def test_complex_symmetric_vs_numpy_and_gemv(prec, uplo, n):
    rng = np.random.default_rng(100 + n)
    A = rnd(rng, prec, (n, n))
    x, y = rnd(rng, prec, n), rnd(rng, prec, n)
    alpha, beta = 0.7 + 0.1j, 0.3 - 0.2j
    S = complete(A.astype(np.complex128), uplo, herm=False)
    assert np.array_equal(S, S.T) and (n == 1 or not np.array_equal(S, S.conj().T))
    al, be = oracle.DTYPES[prec].type(alpha), oracle.DTYPES[prec].type(beta)
    want = np.complex128(al) * (S @ x.astype(np.complex128)) + np.complex128(be) * y.astype(np.complex128)
    for incx, incy, lda in [(1, 1, None), (-2, 3, n + 5)]:
        Af, ld = colmajor(poison(A, uplo), lda=lda)
        got = oracle.csymv(prec, uplo, n, alpha, Af, strided(x, incx), beta, strided(y, incy),
                           lda=ld, incx=incx, incy=incy, mode=MODE_X)
        g = logical(got, n, incy)
        assert np.all(np.isfinite(g)), "the poisoned triangle or padding was read"
        assert np.linalg.norm(g - want) <= XTOL[prec] * np.linalg.norm(want)
    Sf, _ = colmajor(S.astype(oracle.DTYPES[prec]))
    via_gemv = oracle.gemv(prec, "N", n, n, alpha, Sf, x, beta, y, lda=n, mode=MODE_W)
    via_symv = oracle.csymv(prec, uplo, n, alpha, colmajor(poison(A, uplo))[0], x, beta, y, lda=n, mode=MODE_W)
    assert np.array_equal(via_gemv, via_symv)
    # the transposed product of a symmetric matrix is the same sum in the same order
    via_gemv_t = oracle.gemv(prec, "T", n, n, alpha, Sf, x, beta, y, lda=n, mode=MODE_W)
    assert np.array_equal(via_gemv_t, via_symv)


@pytest.mark.parametrize("prec", "cz")
def test_complex_symmetric_bilinear_form_and_diagonal(prec):
    rng = np.random.default_rng(31)
    n = 83
    A = rnd(rng, prec, (n, n))
    x1, x2 = rnd(rng, prec, n), rnd(rng, prec, n)
    zero = np.zeros(n, dtype=A.dtype)
    Af = colmajor(poison(A, "L"))[0]
    # x1^T (S x2) == x2^T (S x1) without any conjugation
    a = np.dot(x1.astype(np.complex128), oracle.csymv(prec, "L", n, 1.0, Af, x2, 0, zero, lda=n))
    b = np.dot(x2.astype(np.complex128), oracle.csymv(prec, "L", n, 1.0, Af, x1, 0, zero, lda=n))
    assert abs(a - b) <= 1e-12 * max(abs(a), 1.0)
    # the imaginary part of the diagonal takes part: changing it changes exactly y_k by i*d*x_k
    B = A.copy()
    k = 17
    B[k, k] += 0.5j
    ya = oracle.csymv(prec, "L", n, 1.0, Af, x1, 0, zero, lda=n)
    yb = oracle.csymv(prec, "L", n, 1.0, colmajor(poison(B, "L"))[0], x1, 0, zero, lda=n)
    diff = yb - ya
    assert np.count_nonzero(diff) == 1
    delta = np.complex128(B[k, k]) - np.complex128(A[k, k])     # 0.5j up to the rounding of the sum
    assert delta.real == 0 and delta.imag != 0
    assert abs(diff[k] - delta * np.complex128(x1[k])) <= 1e-13
    # ABS mode uses |a_kk| of the full diagonal entry, not of its real part
    C = np.zeros((n, n), dtype=A.dtype)
    C[k, k] = 3 + 4j
    ones = np.ones(n, dtype=A.dtype)
    ab = oracle.csymv(prec, "L", n, 1.0, colmajor(C)[0], ones, 0, zero, lda=n, mode=MODE_ABS)
    assert ab[k] == 5.0 and np.count_nonzero(ab) == 1
    ab_h = oracle.symv(prec, "L", n, 1.0, colmajor(C)[0], ones, 0, zero, lda=n, mode=MODE_ABS)
    assert ab_h[k] == 3.0


def test_complex_symmetric_rejects_real_precisions():
    z = np.zeros(1, dtype=np.float64)
    with pytest.raises(ValueError):
        oracle.csymv("d", "L", 1, 1.0, z, z, 0.0, z, lda=1)
