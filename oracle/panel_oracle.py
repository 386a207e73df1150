"""CPU oracle for the panel step of the symmetric tridiagonal reduction (test
infrastructure, never the product path).

The paper's Section 10 speeds up the two-sided reductions by replacing their
matrix-vector products: the tridiagonal reduction calls SYMV on the trailing
block once per column and GEMV on the tall panels of reflectors that have
accumulated so far.  The paper does not print that algorithm; this file writes
out the published one (the "latrd" panel step of the blocked Householder
tridiagonalisation, lower storage), column by column, with plain numpy
products in extended precision and nothing blocked or fused:

for column i of the first nb columns of the symmetric n x n matrix A (lower
triangle referenced), with V = the reflector vectors and W the companion
vectors of the columns before i:

  1. bring column i up to date:   a = A[i:, i] - V[i:, :i] W[i, :i]^T - W[i:, :i] V[i, :i]^T
     (the diagonal entry d_i = a[0] is final)
  2. reflector for a[1:]:  alpha = a[1], x = a[2:], xnorm = ||x||_2;
       xnorm == 0:  tau = 0, beta = alpha
       else:        beta = -sign(alpha) * sqrt(alpha^2 + xnorm^2), tau = (beta - alpha) / beta,
                    x <- x / (alpha - beta)
     e_i = beta; v = [1, x] is stored in A[i+1:, i]  (the leading one explicitly)
  3. w = A[i+1:, i+1:] v                        (the symmetric product with the ORIGINAL trailing block)
     w <- w - V[i+1:, :i] (W[i+1:, :i]^T v) - W[i+1:, :i] (V[i+1:, :i]^T v)
     w <- tau * w;   w <- w - (tau/2) (w^T v) v
     W[i+1:, i] = w, W[:i, i] holds the last small product V[i+1:, :i]^T v (scratch, as in the published routine)

so that after the panel  A - V W^T - W V^T  restricted to the trailing block is
the orthogonally transformed trailing block, and the first nb columns are
tridiagonal with diagonal d and subdiagonal e.  No rescaling against underflow
of xnorm is done (inputs here are O(1)).

V lives in A below the diagonal of the first nb columns: V[:, j] has zeros in
rows 0..j, a one in row j+1 and the scaled x below.
"""
from __future__ import annotations

import numpy as np

_WIDE = {np.dtype(np.float32): np.float64, np.dtype(np.float64): np.longdouble,
         np.dtype(np.complex64): np.complex128, np.dtype(np.complex128): np.clongdouble}


def sytrd_panel(A, nb, *, wide=True):
    """Panel step on a copy of the symmetric matrix whose lower triangle is in
    ``A`` (n x n numpy array; the strict upper triangle is never read).

    Returns ``dict(A=..., e=..., tau=..., W=...)``: ``A`` with the first ``nb``
    columns overwritten (diagonal d, ones on the subdiagonal, reflector tails
    below), ``e`` and ``tau`` of length ``nb``, ``W`` of shape ``(n, nb)``.
    With ``wide`` all arithmetic runs in the next wider type (float64 for
    float32 input, long double for float64) and the results stay in it.
    """
    A = np.asarray(A)
    n = A.shape[0]
    assert A.shape == (n, n) and 0 <= nb <= n
    dt = _WIDE[A.dtype] if wide else A.dtype.type
    # only the lower triangle is taken from the input; work on the completed matrix so that
    # the trailing symmetric product is a plain matrix-vector product
    L = np.tril(A).astype(dt)
    S = L + np.tril(L, -1).T
    out = L.copy()
    V = np.zeros((n, nb), dtype=dt)
    W = np.zeros((n, nb), dtype=dt)
    e = np.zeros(nb, dtype=dt)
    tau = np.zeros(nb, dtype=dt)
    for i in range(nb):
        a = S[i:, i].copy()
        if i:
            a = a - V[i:, :i] @ W[i, :i] - W[i:, :i] @ V[i, :i]
        out[i:, i] = a
        if i >= n - 1:
            continue
        alpha = a[1]
        x = a[2:].copy()
        xnorm = np.sqrt(np.sum(x * x)) if x.size else dt(0)
        if xnorm == 0:
            beta, t = alpha, dt(0)
        else:
            beta = -np.copysign(np.sqrt(alpha * alpha + xnorm * xnorm), alpha)
            t = (beta - alpha) / beta
            x = x / (alpha - beta)
        e[i], tau[i] = beta, t
        v = np.concatenate(([dt(1)], x))
        V[i + 1:, i] = v
        out[i + 1:, i] = v
        w = S[i + 1:, i + 1:] @ v
        if i:
            W[:i, i] = W[i + 1:, :i].T @ v
            w = w - V[i + 1:, :i] @ W[:i, i]
            W[:i, i] = V[i + 1:, :i].T @ v
            w = w - W[i + 1:, :i] @ W[:i, i]
        w = t * w
        w = w - (t / 2) * (w @ v) * v
        W[i + 1:, i] = w
    return dict(A=out, e=e, tau=tau, W=W)


def hetrd_panel(A, nb, *, wide=True):
    """The same panel step for a complex Hermitian matrix (lower triangle referenced, the imaginary part of
    the diagonal ignored): H_i = I - tau_i v_i v_i^H with the published complex reflector (beta real:
    beta = -sign(Re alpha) ||(alpha, x)||, tau = (beta - alpha) / beta, v = [1, x / (alpha - beta)]; tau = 0 when
    x = 0 and alpha is real), column update  a = A[i:, i] - V[i:, :i] conj(W[i, :i]) - W[i:, :i] conj(V[i, :i]),
    w = tau (A22 v - V (W^H v) - W (V^H v)),  w <- w - (tau/2) (w^H v) v,  so that  A - V W^H - W V^H  on the
    trailing block is Q^H A Q there, with d and e real.  Returns the same dictionary; ``e`` is real.
    """
    A = np.asarray(A)
    n = A.shape[0]
    assert A.shape == (n, n) and 0 <= nb <= n and np.iscomplexobj(A)
    dt = _WIDE[A.dtype] if wide else A.dtype.type
    rt = np.real(dt(0)).dtype.type
    L = np.tril(A).astype(dt)
    L[np.arange(n), np.arange(n)] = L[np.arange(n), np.arange(n)].real
    S = L + np.conj(np.tril(L, -1)).T
    out = L.copy()
    V = np.zeros((n, nb), dtype=dt)
    W = np.zeros((n, nb), dtype=dt)
    e = np.zeros(nb, dtype=rt)
    tau = np.zeros(nb, dtype=dt)
    for i in range(nb):
        a = S[i:, i].copy()
        if i:
            a = a - V[i:, :i] @ np.conj(W[i, :i]) - W[i:, :i] @ np.conj(V[i, :i])
        a[0] = a[0].real
        out[i:, i] = a
        if i >= n - 1:
            continue
        alpha = a[1]
        x = a[2:].copy()
        xnorm = np.sqrt(np.sum(x.real * x.real + x.imag * x.imag)) if x.size else rt(0)
        if xnorm == 0 and alpha.imag == 0:
            beta, t = alpha.real, dt(0)
        else:
            beta = -np.copysign(np.sqrt(alpha.real * alpha.real + alpha.imag * alpha.imag + xnorm * xnorm), alpha.real)
            t = dt((beta - alpha.real) / beta + 1j * (-alpha.imag / beta))
            x = x / (alpha - beta)
        e[i], tau[i] = beta, t
        v = np.concatenate(([dt(1)], x))
        V[i + 1:, i] = v
        out[i + 1:, i] = v
        w = S[i + 1:, i + 1:] @ v
        if i:
            W[:i, i] = np.conj(W[i + 1:, :i]).T @ v
            w = w - V[i + 1:, :i] @ W[:i, i]
            W[:i, i] = np.conj(V[i + 1:, :i]).T @ v
            w = w - W[i + 1:, :i] @ W[:i, i]
        w = t * w
        w = w - (t / 2) * (np.conj(w) @ v) * v
        W[i + 1:, i] = w
    return dict(A=out, e=e, tau=tau, W=W)


def trd_panel_upper(A, nb, *, wide=True):
    """The panel step for UPPER storage, real symmetric or complex Hermitian (decided by the dtype): the
    mirror image of the steps above.  The LAST nb columns are reduced, from column n-1 down to n-nb; with
    iw = i - (n - nb) the slot of column i in e, tau and W, and J the slots of the columns already done:

      1. a = A[:i+1, i] - V[:i+1, J] conj(W[i, J]) - W[:i+1, J] conj(V[i, J])     (a[i] = d_i is final, real)
      2. reflector for a[:i]: alpha = a[i-1] (its LAST element), x = a[:i-1]; beta, tau and the scaled x as
         above; e[iw] = beta; v = [x, 1] is stored in A[:i, i] (the one explicitly, at row i-1)
      3. w = A[:i, :i] v - V[:i, J] (W[:i, J]^H v) - W[:i, J] (V[:i, J]^H v);  w <- tau w;
         w <- w - (tau/2) (w^H v) v;   W[:i, iw] = w  (rows i+1.. of that column hold the last small product)

    so that  A - V W^H - W V^H  on the leading (n-nb) x (n-nb) block is Q^H A Q there and the last nb columns
    are tridiagonal with diagonal d and superdiagonal e.  Column 0 has no reflector (e = tau = 0; only when
    nb = n).  Only the upper triangle of ``A`` is read (and not the imaginary part of a complex diagonal).
    Returns ``dict(A=..., e=..., tau=..., W=...)`` with ``e`` real, all of length / width ``nb``.
    """
    A = np.asarray(A)
    n = A.shape[0]
    assert A.shape == (n, n) and 0 <= nb <= n
    cplx = np.iscomplexobj(A)
    dt = _WIDE[A.dtype] if wide else A.dtype.type
    rt = np.real(dt(0)).dtype.type
    U = np.triu(A).astype(dt)
    if cplx:
        U[np.arange(n), np.arange(n)] = U[np.arange(n), np.arange(n)].real
    S = U + np.conj(np.triu(U, 1)).T
    out = U.copy()
    V = np.zeros((n, nb), dtype=dt)
    W = np.zeros((n, nb), dtype=dt)
    e = np.zeros(nb, dtype=rt)
    tau = np.zeros(nb, dtype=dt)
    for i in range(n - 1, n - nb - 1, -1):
        iw = i - (n - nb)
        J = slice(iw + 1, nb)
        a = S[:i + 1, i].copy()
        if i < n - 1:
            a = a - V[:i + 1, J] @ np.conj(W[i, J]) - W[:i + 1, J] @ np.conj(V[i, J])
        if cplx:
            a[i] = a[i].real
        out[:i + 1, i] = a
        if i == 0:
            continue
        alpha = a[i - 1]
        x = a[:i - 1].copy()
        xnorm = np.sqrt(np.sum((x * np.conj(x)).real)) if x.size else rt(0)
        if xnorm == 0 and (not cplx or alpha.imag == 0):
            beta, t = (alpha.real if cplx else alpha), dt(0)
        else:
            are = alpha.real if cplx else alpha
            beta = -np.copysign(np.sqrt((alpha * np.conj(alpha)).real + xnorm * xnorm), are)
            t = dt((beta - alpha) / beta)
            x = x / (alpha - beta)
        e[iw], tau[iw] = beta, t
        v = np.concatenate((x, [dt(1)]))
        V[:i, iw] = v
        out[:i, i] = v
        w = S[:i, :i] @ v
        if i < n - 1:
            W[i + 1:, iw] = np.conj(W[:i, J]).T @ v
            w = w - V[:i, J] @ W[i + 1:, iw]
            W[i + 1:, iw] = np.conj(V[:i, J]).T @ v
            w = w - W[:i, J] @ W[i + 1:, iw]
        w = t * w
        w = w - (t / 2) * (np.conj(w) @ v) * v
        W[:i, iw] = w
    return dict(A=out, e=e, tau=tau, W=W)
