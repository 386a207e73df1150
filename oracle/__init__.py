"""CPU oracle for GEMV / SYMV / HEMV (test infrastructure, never the product path).

Thin numpy/ctypes front end of ``mv_oracle.cpp`` (plain C++ double loops, one
left-to-right sum per output element).  Only ``tests/``, the smoke check and
the CPU-baseline leg of the benchmark may import this package; the GPU library
and its Python binding never do, and this package imports nothing of theirs.

The operation is the one of the paper's Section 5.2: ``y = alpha*op(A)*x +
beta*y`` with ``A`` general (GEMV, op = identity / transpose / conjugate
transpose) or symmetric / Hermitian with a single stored triangle (SYMV for
s,d; HEMV for c,z; Section 7 states that only one triangle is read).

Matrices are column major: a numpy array ``A`` holding the matrix must be
Fortran-ordered, or the caller passes a flat buffer together with ``lda``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mv_oracle.cpp")
_LIB = os.path.join(_HERE, "libmv_oracle.so")

MODE_W = 0    # working-precision accumulation (the timed CPU baseline)
MODE_X = 1    # extended accumulation, returns float64 / complex128
MODE_ABS = 2  # |alpha| sum |a||x| + |beta||y| in float64

DTYPES = {
    "s": np.dtype(np.float32),
    "d": np.dtype(np.float64),
    "c": np.dtype(np.complex64),
    "z": np.dtype(np.complex128),
}
_XOUT = {"s": np.float64, "d": np.float64, "c": np.complex128, "z": np.complex128}


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (g++ -O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c++11", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, vp, ch, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_char, ctypes.c_int
        lib.mvo_gemv.argtypes = [ch, ci, ch, i64, i64, vp, vp, i64, vp, i64, vp, vp, i64, vp, vp, i64]
        lib.mvo_gemv.restype = ci
        lib.mvo_symv.argtypes = [ch, ci, ch, i64, vp, vp, i64, vp, i64, vp, vp, i64, vp, vp, i64]
        lib.mvo_symv.restype = ci
        lib.mvo_symv_complex_symmetric.argtypes = lib.mvo_symv.argtypes
        lib.mvo_symv_complex_symmetric.restype = ci
        lib.mvo_num_threads.restype = ci
        lib.mvo_set_num_threads.argtypes = [ci]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().mvo_num_threads())


def set_num_threads(t: int) -> None:
    _load().mvo_set_num_threads(int(t))


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _vec_extent(length: int, inc: int) -> int:
    return 0 if length == 0 else 1 + (length - 1) * abs(inc)


def _prep(prec, A, lda, rows, cols):
    dt = DTYPES[prec]
    A = np.asarray(A)
    if A.dtype != dt:
        raise TypeError(f"A must be {dt}, got {A.dtype}")
    if A.ndim == 2:
        if not A.flags.f_contiguous and A.size:
            raise ValueError("2-D A must be Fortran (column-major) ordered")
        if lda is None:
            lda = max(1, A.shape[0])
        if A.shape[0] > lda or (cols and A.shape[1] < cols):
            raise ValueError("A too small")
    else:
        if lda is None:
            raise ValueError("flat A needs lda")
        if cols and rows and A.size < (cols - 1) * lda + rows:
            raise ValueError("flat A too small")
    return A, int(lda)


def _out_buffer(prec, mode, y):
    if mode == MODE_W:
        return np.array(y, copy=True)
    if mode == MODE_X:
        return y.astype(_XOUT[prec])
    return np.abs(y).astype(np.float64)


def gemv(prec, trans, m, n, alpha, A, x, beta, y, *, lda=None, incx=1, incy=1,
         mode=MODE_X, sample=None):
    """Return op(A)x scaled and added to y; ``y`` itself is not modified.

    The returned array has the strided layout of ``y`` (same length and
    increment); entries that are not outputs keep the (converted) input value.
    """
    lib = _load()
    dt = DTYPES[prec]
    trans = trans.upper()
    A, lda = _prep(prec, A, lda, m, n)
    x = np.ascontiguousarray(x, dtype=dt)
    y = np.ascontiguousarray(y, dtype=dt)
    leny, lenx = (m, n) if trans == "N" else (n, m)
    assert x.size >= _vec_extent(lenx, incx) and y.size >= _vec_extent(leny, incy)
    out = _out_buffer(prec, mode, y)
    al = np.array([alpha], dtype=dt)
    be = np.array([beta], dtype=dt)
    if sample is not None:
        sample = np.ascontiguousarray(sample, dtype=np.int64)
        sp, ns = _ptr(sample), sample.size
    else:
        sp, ns = None, 0
    rc = lib.mvo_gemv(prec.encode(), mode, trans.encode(), m, n, _ptr(al), _ptr(A), lda,
                      _ptr(x), incx, _ptr(be), _ptr(y), incy, _ptr(out), sp, ns)
    if rc != 0:
        raise RuntimeError(f"mvo_gemv failed: {rc}")
    return out


def symv(prec, uplo, n, alpha, A, x, beta, y, *, lda=None, incx=1, incy=1,
         mode=MODE_X, sample=None, complex_symmetric=False):
    """SYMV (prec s,d) or HEMV (prec c,z) reading only the ``uplo`` triangle.

    ``complex_symmetric=True`` (prec c,z only) gives the complex symmetric
    product instead of the Hermitian one: no conjugation, diagonal as stored.
    """
    lib = _load()
    if complex_symmetric and prec not in "cz":
        raise ValueError("complex_symmetric needs prec 'c' or 'z'")
    fn = lib.mvo_symv_complex_symmetric if complex_symmetric else lib.mvo_symv
    dt = DTYPES[prec]
    A, lda = _prep(prec, A, lda, n, n)
    x = np.ascontiguousarray(x, dtype=dt)
    y = np.ascontiguousarray(y, dtype=dt)
    assert x.size >= _vec_extent(n, incx) and y.size >= _vec_extent(n, incy)
    out = _out_buffer(prec, mode, y)
    al = np.array([alpha], dtype=dt)
    be = np.array([beta], dtype=dt)
    if sample is not None:
        sample = np.ascontiguousarray(sample, dtype=np.int64)
        sp, ns = _ptr(sample), sample.size
    else:
        sp, ns = None, 0
    rc = fn(prec.encode(), mode, uplo.upper().encode(), n, _ptr(al), _ptr(A), lda,
            _ptr(x), incx, _ptr(be), _ptr(y), incy, _ptr(out), sp, ns)
    if rc != 0:
        raise RuntimeError(f"mvo_symv failed: {rc}")
    return out


hemv = symv


def csymv(prec, uplo, n, alpha, A, x, beta, y, **kw):
    """Complex symmetric SYMV (prec c,z)."""
    return symv(prec, uplo, n, alpha, A, x, beta, y, complex_symmetric=True, **kw)
