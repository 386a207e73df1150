"""CPU oracle for the panel step of the bidiagonal reduction (test infrastructure,
never the product path).

The paper's Section 10 names the bidiagonal reduction as the consumer of GEMV on
sub-blocks: every column of a panel multiplies the trailing block once from the
left (transposed) and once from the right, and several tall or wide panels of
accumulated vectors besides.  The paper prints no algorithm; this file writes out
the published "labrd" panel step (m >= n, upper bidiagonal) from its definition,
column by column, with plain numpy products in extended precision:

for i = 0 .. nb-1, with V, U the reflector vectors so far and X, Y the companion
panels (A is m x n; everything not yet reduced keeps its input values):

  1. column i up to date:   a = A[i:, i] - V[i:, :i] Y[i, :i]^T - X[i:, :i] Ubar[:i, i]
     where V[i:, :i] lives in A[i:, :i] and Ubar[:i, i] = A[:i, i] (the rows 0..i-1 of column i, which
     hold the row reflectors' entries)
  2. column reflector for a:  alpha = a[0], x = a[1:];  beta = -sign(alpha) ||a||,  tauq = (beta - alpha)/beta,
     v = [1, x / (alpha - beta)];  d_i = beta   (x = 0 gives tauq = 0, beta = alpha)
  3. if i < n-1:
       y = A[i:, i+1:]^T v                                  (trailing block, transposed)
       y -= Y[i+1:, :i] (A[i:, :i]^T v) + A[:i, i+1:]^T (X[i:, :i]^T v);   y *= tauq
       row i up to date:    r = A[i, i+1:] - Y[i+1:, :i+1] A[i, :i+1]^T - A[:i, i+1:]^T X[i, :i]^T
       row reflector for r: taup, u = [1, ...], e_i = beta
       x = A[i+1:, i+1:] u                                  (trailing block)
       x -= A[i+1:, :i+1] (Y[i+1:, :i+1]^T u) + X[i+1:, :i] (A[:i, i+1:] u);   x *= taup
     Y[i+1:, i] = y,  X[i+1:, i] = x

so that afterwards  A - V Y^T - X U^T  on the trailing block equals Q^T A P there, and the leading nb
rows and columns of Q^T A P are upper bidiagonal with diagonal d and superdiagonal e.  V is stored in
A on and below the diagonal of the first nb columns (leading ones explicit), U in A right of the diagonal
of the first nb rows (leading ones explicit, at column i+1).  No rescaling of the norms.

Complex matrices (``gebrd_panel`` accepts complex64 / complex128): the same steps with H_i = I - tauq v v^H
applied as H_i^H from the left and G_i = I - taup u u^H from the right, so that every transpose above
becomes a conjugate transpose and the update reads  A - V Y^H - X U^H:
  y = tauq (A^H v - Y (V^H v) - U (X^H v)),      x = taup (A u - V (Y^H u) - X (U^H u)),
a reflector for the complex vector (alpha, x) has beta = -sign(Re alpha) ||(alpha, x)|| real (so d and e are
real), tau = (beta - alpha)/beta complex, and is skipped (tau = 0) only when x = 0 and alpha is real; the
row reflector is generated from the conjugate of the updated row (that makes r G_i = beta e_1^T), and row i
of A right of the diagonal stores u^H, the rows of U^H.
"""
from __future__ import annotations

import numpy as np

_WIDE = {np.dtype(np.float32): np.float64, np.dtype(np.float64): np.longdouble,
         np.dtype(np.complex64): np.complex128, np.dtype(np.complex128): np.clongdouble}


def _reflector(alpha, x, dt):
    """(beta, tau, scaled x) with H^H (alpha, x) = (beta, 0), H = I - tau v v^H, v = (1, scaled x)"""
    if np.iscomplexobj(x) or np.iscomplexobj(alpha):
        rt = np.real(dt(0)).dtype.type
        xnorm = np.sqrt(np.sum(x.real * x.real + x.imag * x.imag)) if x.size else rt(0)
        if xnorm == 0 and alpha.imag == 0:
            return alpha.real, dt(0), x
        beta = -np.copysign(np.sqrt(alpha.real * alpha.real + alpha.imag * alpha.imag + xnorm * xnorm), alpha.real)
        return beta, dt((beta - alpha) / beta), x / (alpha - beta)
    xnorm = np.sqrt(np.sum(x * x)) if x.size else dt(0)
    if xnorm == 0:
        return alpha, dt(0), x
    beta = -np.copysign(np.sqrt(alpha * alpha + xnorm * xnorm), alpha)
    return beta, (beta - alpha) / beta, x / (alpha - beta)


def gebrd_panel(A, nb, *, wide=True):
    """Panel step on a copy of the m x n matrix ``A`` (m >= n, 0 <= nb <= n).

    Returns ``dict(A=..., d=..., e=..., tauq=..., taup=..., X=..., Y=...)``: ``A`` with the first nb
    columns and rows overwritten by the reflector vectors (ones explicit), ``X`` (m x nb) and ``Y``
    (n x nb) with rows 0..i of column i zero (scratch in the device routine).
    """
    A = np.asarray(A)
    m, n = A.shape
    assert m >= n and 0 <= nb <= n
    dt = _WIDE[A.dtype] if wide else A.dtype.type
    rt = np.real(dt(0)).dtype.type          # d and e are real
    W = A.astype(dt).copy()
    X = np.zeros((m, nb), dtype=dt)
    Y = np.zeros((n, nb), dtype=dt)
    d = np.zeros(nb, dtype=rt)
    e = np.zeros(nb, dtype=rt)
    tauq = np.zeros(nb, dtype=dt)
    taup = np.zeros(nb, dtype=dt)
    H = lambda M: M.conj().T                # (conjugate) transpose
    for i in range(nb):
        # 1. column i
        a = W[i:, i].copy()
        if i:
            a = a - W[i:, :i] @ Y[i, :i].conj() - X[i:, :i] @ W[:i, i]
        # 2. column reflector
        beta, tq, tail = _reflector(a[0], a[1:].copy(), dt)
        d[i], tauq[i] = beta, tq
        v = np.concatenate(([dt(1)], tail))
        W[i:, i] = v
        if i >= n - 1:
            continue
        # 3. y
        y = H(W[i:, i + 1:]) @ v
        if i:
            y = y - Y[i + 1:, :i] @ (H(W[i:, :i]) @ v) - H(W[:i, i + 1:]) @ (H(X[i:, :i]) @ v)
        y = tq * y
        Y[i + 1:, i] = y
        # row i (W[i, :i+1] ends with the explicit one of v)
        r = W[i, i + 1:].copy()
        r = r - Y[i + 1:, :i + 1].conj() @ W[i, :i + 1]
        if i:
            r = r - X[i, :i] @ W[:i, i + 1:]
        beta, tp, tail = _reflector(r[0].conj(), r[1:].conj().copy(), dt)
        e[i], taup[i] = beta, tp
        u = np.concatenate(([dt(1)], tail))
        W[i, i + 1:] = u.conj()
        # x
        x = W[i + 1:, i + 1:] @ u
        x = x - W[i + 1:, :i + 1] @ (H(Y[i + 1:, :i + 1]) @ u)
        if i:
            x = x - X[i + 1:, :i] @ (W[:i, i + 1:] @ u)
        x = tp * x
        X[i + 1:, i] = x
    return dict(A=W, d=d, e=e, tauq=tauq, taup=taup, X=X, Y=Y)


def gebrd_panel_wide(A, nb, *, wide=True):
    """The panel step for m < n (more columns than rows): the reduction is to LOWER bidiagonal form, with the
    roles of rows and columns exchanged.  For i = 0 .. nb-1 (0 <= nb <= m), with the update A - V Y^H - X U^H of
    the reflectors so far (V: column reflectors v_k, support rows k+1.., stored in A[k+1:, k]; U: row reflectors
    u_k, support columns k.., stored conjugated in A[k, k:]):

      1. row i up to date:      r = A[i, i:] - V[i, :i] Y[i:, :i]^H - X[i, :i] U^H[:i, i:]
      2. row reflector from conj(r): beta = d_i, taup_i, u_i (one at column i); A[i, i:] = u_i^H
      3. if i < m-1:
           x = taup (A[i+1:, i:] u - V[i+1:, :i] (Y[i:, :i]^H u) - X[i+1:, :i] (U^H[:i, i:] u));   X[i+1:, i] = x
           column i up to date:  c = A[i+1:, i] - V[i+1:, :i] conj(Y[i, :i]) - X[i+1:, :i+1] U^H[:i+1, i]
           column reflector from c: beta = e_i, tauq_i, v_i (one at row i+1); A[i+1:, i] = v_i
           y = tauq (A[i+1:, i+1:]^H v - Y[i+1:, :i] (V[i+1:, :i]^H v) - U[i+1:, :i+1] (X[i+1:, :i+1]^H v));  Y[i+1:, i] = y

    so that the first nb rows and columns of Q^H A P are lower bidiagonal (diagonal d, subdiagonal e) and
    A - V Y^H - X U^H on the trailing block equals Q^H A P there.  The last row of the matrix has no column
    reflector (e = tauq = 0).  Returns the same dictionary as ``gebrd_panel``; X is m x nb, Y is n x nb.
    """
    A = np.asarray(A)
    m, n = A.shape
    assert m < n and 0 <= nb <= m
    dt = _WIDE[A.dtype] if wide else A.dtype.type
    rt = np.real(dt(0)).dtype.type
    W = A.astype(dt).copy()
    X = np.zeros((m, nb), dtype=dt)
    Y = np.zeros((n, nb), dtype=dt)
    d = np.zeros(nb, dtype=rt)
    e = np.zeros(nb, dtype=rt)
    tauq = np.zeros(nb, dtype=dt)
    taup = np.zeros(nb, dtype=dt)
    H = lambda M: M.conj().T
    for i in range(nb):
        # 1. row i (W[i, :i] holds the entries of v_0 .. v_{i-1} in row i; W[:i, i:] the rows u_k^H)
        r = W[i, i:].copy()
        if i:
            r = r - Y[i:, :i].conj() @ W[i, :i] - X[i, :i] @ W[:i, i:]
        # 2. row reflector
        beta, tp, tail = _reflector(r[0].conj(), r[1:].conj().copy(), dt)
        d[i], taup[i] = beta, tp
        u = np.concatenate(([dt(1)], tail))
        W[i, i:] = u.conj()
        if i >= m - 1:
            continue
        # 3. x
        x = W[i + 1:, i:] @ u
        if i:
            x = x - W[i + 1:, :i] @ (H(Y[i:, :i]) @ u) - X[i + 1:, :i] @ (W[:i, i:] @ u)
        x = tp * x
        X[i + 1:, i] = x
        # column i
        c = W[i + 1:, i].copy()
        if i:
            c = c - W[i + 1:, :i] @ Y[i, :i].conj()
        c = c - X[i + 1:, :i + 1] @ W[:i + 1, i]
        beta, tq, tail = _reflector(c[0], c[1:].copy(), dt)
        e[i], tauq[i] = beta, tq
        v = np.concatenate(([dt(1)], tail))
        W[i + 1:, i] = v
        # y
        y = H(W[i + 1:, i + 1:]) @ v
        if i:
            y = y - Y[i + 1:, :i] @ (H(W[i + 1:, :i]) @ v)
        y = y - H(W[:i + 1, i + 1:]) @ (H(X[i + 1:, :i + 1]) @ v)
        y = tq * y
        Y[i + 1:, i] = y
    return dict(A=W, d=d, e=e, tauq=tauq, taup=taup, X=X, Y=Y)
