"""What the result of a panel step has to satisfy, stated per case instead of as one flat tolerance.

A panel is a chain of nb dependent columns (Section 10's reductions call SYMV / GEMV once or twice per
column), so its rounding error is not that of one product.  Two things are required of the device's result:

1. against the oracles: its deviation from the oracle run in the next wider type is at most K_DEV times the
   deviation of the SAME oracle run in the working precision on the same input (plus a few units of
   roundoff for the tiny cases in which both are zero or nearly so).  The working-precision oracle takes
   the same steps with numpy's summation order; K_DEV covers the difference between two legitimate
   orders of summation, nothing more.
2. the factorisation identities, each to the normwise tolerance of a single product (1e-5 / 1e-13 relative
   to ||A||_F), evaluated in the wider type with the device's own reflectors, tau, d, e and companion
   panels: the leading rows / columns of Q^H A Q (Q^H A P) are tridiagonal (bidiagonal) with the
   device's d and e, the trailing block of A - V W^H - W V^H (A - V Y^H - X U^H) equals that of
   Q^H A Q (Q^H A P), and every I - tau v v^H is unitary.
"""
from __future__ import annotations

import numpy as np

K_DEV = 4.0
UNIT = {"s": 2.0 ** -24, "c": 2.0 ** -24, "d": 2.0 ** -53, "z": 2.0 ** -53}
IDENTITY_TOL = {"s": 1e-5, "c": 1e-5, "d": 1e-13, "z": 1e-13}


def wide_dtype(prec, force_complex=False):
    real = np.float64 if prec in "sc" else np.longdouble
    cplx = np.complex128 if prec in "sc" else np.clongdouble
    return cplx if (prec in "cz" or force_complex) else real


def deviation(prec, got, ref):
    """|| got - ref ||_2 / || ref ||_2 in the wider type"""
    dt = wide_dtype(prec, np.iscomplexobj(got) or np.iscomplexobj(ref))
    g, r = np.asarray(got).astype(dt).ravel(), np.asarray(ref).astype(dt).ravel()
    nrm = np.sqrt(np.sum(np.abs(r) ** 2))
    err = np.sqrt(np.sum(np.abs(g - r) ** 2))
    return float(err / nrm) if nrm > 0 else float(err)


def against_oracles(prec, what, got, wide, work, log=None):
    """requirement 1 for one output (already restricted to its defined entries)"""
    dev_gpu, dev_work = deviation(prec, got, wide), deviation(prec, work, wide)
    if log is not None:
        log.append((what, dev_gpu, dev_work))
    assert np.isfinite(dev_gpu), f"{what}: non-finite result"
    assert dev_gpu <= K_DEV * dev_work + 8 * UNIT[prec], \
        f"{what}: device deviates {dev_gpu:.3e} from the wide oracle, the working-precision oracle {dev_work:.3e}"


def _left(B, v, t):
    """B <- (I - conj(t) v v^H) B"""
    return B - np.conj(t) * np.outer(v, np.conj(v) @ B)


def _right(B, v, t):
    """B <- B (I - t v v^H)"""
    return B - t * np.outer(B @ v, np.conj(v))


def _norm(M):
    return float(np.sqrt(np.sum(np.abs(M) ** 2)))


def _unitarity(v, t):
    """| 2 Re t - |t|^2 v^H v |: zero exactly when I - t v v^H is unitary"""
    return float(abs(2 * np.real(t) - np.abs(t) ** 2 * np.real(np.conj(v) @ v)))


def affordable(prec, n, nb):
    """the identities run in long double (no BLAS) for d and z: the largest complex cases are left to c"""
    return not (prec == "z" and n * n * nb > 4e7)


def trd_identities(prec, uplo, A0, A1, tau, e, W, nb):
    """(largest defect of unitarity of a reflector, tridiagonal residual / ||S||_F, trailing-block residual /
    ||S||_F) for kmv_*trd_panel's result.
    A0: the input block (only the uplo triangle is used), A1: the block afterwards (n x n, row index first),
    W: n x nb."""
    n = A0.shape[0]
    dt = wide_dtype(prec)
    lower = uplo == "L"
    T0 = (np.tril(A0) if lower else np.triu(A0)).astype(dt)
    idx = np.arange(n)
    T0[idx, idx] = T0[idx, idx].real
    S = T0 + np.conj(np.tril(T0, -1) if lower else np.triu(T0, 1)).T
    first = 0 if lower else n - nb
    V = np.zeros((n, nb), dtype=dt)
    E = np.zeros((n, n), dtype=dt)               # the tridiagonal part the panel's columns must equal
    B = S.copy()
    order = range(nb) if lower else range(nb - 1, -1, -1)
    th, eh = np.asarray(tau).astype(dt), np.asarray(e).astype(dt)
    r0 = 0.0
    for s in order:                              # s: slot in e, tau, W; i: column
        i = first + s
        E[i, i] = np.real(A1[i, i])
        if lower and i < n - 1:
            V[i + 1:, s] = A1[i + 1:, i]
            E[i + 1, i] = E[i, i + 1] = eh[s]
        elif not lower and i > 0:
            V[:i, s] = A1[:i, i]
            E[i - 1, i] = E[i, i - 1] = eh[s]
        else:
            continue
        r0 = max(r0, _unitarity(V[:, s], th[s]))
        B = _right(_left(B, V[:, s], th[s]), V[:, s], th[s])
    cols = slice(0, nb) if lower else slice(n - nb, n)
    rest = slice(nb, n) if lower else slice(0, n - nb)
    nrm = _norm(S) or 1.0
    r1 = _norm((B - E)[:, cols]) / nrm
    Wd = np.asarray(W).astype(dt)[rest]
    Vd = V[rest]
    trailing = S[rest, rest] - Vd @ np.conj(Wd).T - Wd @ np.conj(Vd).T
    r2 = _norm(trailing - B[rest, rest]) / nrm
    return r0, r1, r2


def gebrd_identities(prec, A0, A1, d, e, tauq, taup, X, Y, nb):
    """(largest defect of unitarity, bidiagonal residual / ||A||_F, trailing-block residual / ||A||_F) for
    kmv_*gebrd_panel's result; tall (m >= n,
    upper bidiagonal) or wide (m < n, lower bidiagonal) by the shape.  X: m x nb, Y: n x nb."""
    m, n = A0.shape
    dt = wide_dtype(prec)
    tall = m >= n
    A = np.asarray(A0).astype(dt)
    B = A.copy()
    V = np.zeros((m, nb), dtype=dt)
    UH = np.zeros((nb, n), dtype=dt)             # rows u_i^H as stored
    E = np.zeros((m, n), dtype=dt)
    tq, tp = np.asarray(tauq).astype(dt), np.asarray(taup).astype(dt)
    dh, eh = np.asarray(d).astype(dt), np.asarray(e).astype(dt)
    r0 = 0.0
    for i in range(nb):
        E[i, i] = dh[i]
        if tall:
            V[i:, i] = A1[i:, i]
            B = _left(B, V[:, i], tq[i])
            r0 = max(r0, _unitarity(V[:, i], tq[i]))
            if i < n - 1:
                UH[i, i + 1:] = A1[i, i + 1:]
                E[i, i + 1] = eh[i]
                B = _right(B, np.conj(UH[i]), tp[i])
                r0 = max(r0, _unitarity(UH[i], tp[i]))
        else:
            UH[i, i:] = A1[i, i:]
            B = _right(B, np.conj(UH[i]), tp[i])
            r0 = max(r0, _unitarity(UH[i], tp[i]))
            if i < m - 1:
                V[i + 1:, i] = A1[i + 1:, i]
                E[i + 1, i] = eh[i]
                B = _left(B, V[:, i], tq[i])
                r0 = max(r0, _unitarity(V[:, i], tq[i]))
    nrm = _norm(A) or 1.0
    mask = np.zeros((m, n), dtype=bool)
    mask[:nb, :] = True
    mask[:, :nb] = True
    r1 = _norm((B - E)[mask]) / nrm
    Xd, Yd = np.asarray(X).astype(dt)[nb:], np.asarray(Y).astype(dt)[nb:]
    trailing = A[nb:, nb:] - V[nb:] @ np.conj(Yd).T - Xd @ UH[:, nb:]
    r2 = _norm(trailing - B[nb:, nb:]) / nrm
    return r0, r1, r2


def check_identities(prec, what, residuals, log=None):
    r0, r1, r2 = residuals
    if log is not None:
        log.append((what + " identities", r0, r1, r2))
    assert r0 <= IDENTITY_TOL[prec], f"{what}: a reflector misses unitarity by {r0:.3e}"
    assert r1 <= IDENTITY_TOL[prec], f"{what}: reduced rows/columns deviate from the band form by {r1:.3e}"
    assert r2 <= IDENTITY_TOL[prec], f"{what}: trailing block deviates by {r2:.3e}"
