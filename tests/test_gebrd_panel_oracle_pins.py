"""Pins of the bidiagonal panel oracle (`oracle/gebrd_panel_oracle.py`) against numpy linear algebra on the
explicitly formed reflectors: orthogonality, the bidiagonal leading rows and columns of Q^T A P, the
trailing-block identity A - V Y^T - X U^T = Q^T A P, singular values of a full reduction, and a 2 x 2 case
worked by hand; the same for complex matrices (unitary H_i and G_i, real d and e, conjugate transposes), plus
the complex panel on real data against the real one."""
import numpy as np
import pytest

from oracle import gebrd_panel_oracle as go


def reflectors(res, m, n, nb):
    A = np.asarray(res["A"], dtype=np.float64)
    V = np.zeros((m, nb))
    U = np.zeros((n, nb))
    for i in range(nb):
        V[i:, i] = A[i:, i]
        if i < n - 1:
            U[i + 1:, i] = A[i, i + 1:]
    return V, U


def products(V, U, tauq, taup):
    m, n, nb = V.shape[0], U.shape[0], V.shape[1]
    Q, P = np.eye(m), np.eye(n)
    for i in range(nb):
        Q = Q @ (np.eye(m) - tauq[i] * np.outer(V[:, i], V[:, i]))
        P = P @ (np.eye(n) - taup[i] * np.outer(U[:, i], U[:, i]))
    return Q, P


def test_hand_worked_two_by_two():
    # column (3, 4): beta = -5, tauq = 8/5, v = (1, 1/2);  y = tauq * (row of A^T v) = 1.6 * (1*1 + 2*0.5) = 3.2
    # row 0 right of the diagonal: 1 - y * 1 = -2.2: a single entry, nothing to annihilate: taup = 0, e = -2.2
    A = np.array([[3.0, 1.0], [4.0, 2.0]])
    r = go.gebrd_panel(A, 1)
    assert float(r["d"][0]) == -5.0 and abs(float(r["tauq"][0]) - 1.6) < 1e-18
    assert float(r["A"][0, 0]) == 1.0 and float(r["A"][1, 0]) == 0.5
    assert abs(float(r["Y"][1, 0]) - 3.2) < 1e-15
    assert abs(float(r["e"][0]) + 2.2) < 1e-15 and float(r["taup"][0]) == 0.0 and float(r["A"][0, 1]) == 1.0
    # x = taup * (...) = 0
    assert float(r["X"][1, 0]) == 0.0


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("m,n,nb", [(2, 2, 1), (5, 3, 2), (40, 40, 8), (97, 61, 32), (64, 64, 64), (50, 33, 33)])
def test_two_sided_identities(dtype, m, n, nb):
    rng = np.random.default_rng(m * 1000 + n * 10 + nb)
    A0 = rng.uniform(-1, 1, (m, n)).astype(dtype)
    r = go.gebrd_panel(A0, nb)
    A64 = A0.astype(np.float64)
    V, U = reflectors(r, m, n, nb)
    tauq = np.asarray(r["tauq"], dtype=np.float64)
    taup = np.asarray(r["taup"], dtype=np.float64)
    d = np.asarray(r["d"], dtype=np.float64)
    e = np.asarray(r["e"], dtype=np.float64)
    X = np.asarray(r["X"], dtype=np.float64)
    Y = np.asarray(r["Y"], dtype=np.float64)
    for i in range(nb):
        assert V[i, i] == 1.0 and np.all(V[:i, i] == 0)
        assert tauq[i] == 0 or abs(tauq[i] * (V[:, i] @ V[:, i]) - 2) < 1e-13
        if i < n - 1:
            assert U[i + 1, i] == 1.0 and np.all(U[:i + 1, i] == 0)
            assert taup[i] == 0 or abs(taup[i] * (U[:, i] @ U[:, i]) - 2) < 1e-13
    Q, P = products(V, U, tauq, taup)
    B = Q.T @ A64 @ P
    scale = np.linalg.norm(A64)
    for i in range(nb):
        assert abs(B[i, i] - d[i]) < 1e-13 * scale
        assert np.all(np.abs(B[i + 1:, i]) < 1e-13 * scale), "column not reduced"
        if i < n - 1:
            assert abs(B[i, i + 1] - e[i]) < 1e-13 * scale
            assert np.all(np.abs(B[i, i + 2:]) < 1e-13 * scale), "row not reduced"
        assert np.all(np.abs(B[i, :i]) < 1e-13 * scale)
    upd = A64 - V @ Y.T - X @ U.T
    assert np.allclose(upd[nb:, nb:], B[nb:, nb:], atol=1e-12 * scale)
    # everything outside the first nb rows and columns keeps its input values
    assert np.array_equal(np.asarray(r["A"])[nb:, nb:].astype(np.float64), A64[nb:, nb:])


def test_full_reduction_keeps_singular_values():
    rng = np.random.default_rng(3)
    m, n = 45, 30
    A0 = rng.uniform(-1, 1, (m, n))
    r = go.gebrd_panel(A0, n)
    d = np.asarray(r["d"], dtype=np.float64)
    e = np.asarray(r["e"], dtype=np.float64)[: n - 1]
    B = np.diag(d) + np.diag(e, 1)
    assert np.allclose(np.linalg.svd(B, compute_uv=False), np.linalg.svd(A0, compute_uv=False), atol=1e-12)


# ---- complex matrices: H_i = I - tauq v v^H applied as H_i^H from the left, G_i = I - taup u u^H from the right

def complex_reflectors(res, m, n, nb):
    A = np.asarray(res["A"], dtype=np.complex128)
    V = np.zeros((m, nb), dtype=np.complex128)
    U = np.zeros((n, nb), dtype=np.complex128)
    for i in range(nb):
        V[i:, i] = A[i:, i]
        if i < n - 1:
            U[i + 1:, i] = A[i, i + 1:].conj()        # the row stores u^H
    return V, U


def test_hand_worked_complex_column():
    # column (3i, 4): Re alpha = 0 counts as positive, beta = -5, tauq = (beta - alpha)/beta = 1 + 0.6i,
    # v = (1, 4/(3i + 5)) = (1, (20 - 12i)/34)
    A = np.array([[3j, 1.0], [4.0, 2.0]], dtype=np.complex128)
    r = go.gebrd_panel(A, 1)
    assert float(r["d"][0]) == -5.0
    assert abs(complex(r["tauq"][0]) - (1 + 0.6j)) < 1e-17
    assert complex(r["A"][0, 0]) == 1.0 and abs(complex(r["A"][1, 0]) - (20 - 12j) / 34) < 1e-17
    # H^H (3i, 4) = (-5, 0) with H = I - tauq v v^H
    v = np.array([1.0, (20 - 12j) / 34])
    Hm = np.eye(2) - (1 + 0.6j) * np.outer(v, v.conj())
    assert np.allclose(Hm.conj().T @ np.array([3j, 4.0]), [-5.0, 0.0], atol=1e-15)
    assert np.allclose(Hm.conj().T @ Hm, np.eye(2), atol=1e-15)
    # a single real element right of the diagonal would need no reflector; this one is complex, so the
    # reflector turns it onto the real axis: |e| = |updated element|
    y = complex(r["Y"][1, 0])
    assert abs(abs(float(r["e"][0])) - abs(1.0 - np.conj(y))) < 1e-15
    assert np.isrealobj(r["d"]) and np.isrealobj(r["e"])


@pytest.mark.parametrize("dtype", [np.complex64, np.complex128])
@pytest.mark.parametrize("m,n,nb", [(2, 2, 1), (5, 3, 2), (40, 40, 8), (97, 61, 32), (64, 64, 64), (50, 33, 33)])
def test_complex_two_sided_identities(dtype, m, n, nb):
    rng = np.random.default_rng(m * 1000 + n * 10 + nb + 7)
    A0 = (rng.uniform(-1, 1, (m, n)) + 1j * rng.uniform(-1, 1, (m, n))).astype(dtype)
    r = go.gebrd_panel(A0, nb)
    A128 = A0.astype(np.complex128)
    V, U = complex_reflectors(r, m, n, nb)
    tauq = np.asarray(r["tauq"], dtype=np.complex128)
    taup = np.asarray(r["taup"], dtype=np.complex128)
    d = np.asarray(r["d"], dtype=np.float64)
    e = np.asarray(r["e"], dtype=np.float64)
    X = np.asarray(r["X"], dtype=np.complex128)
    Y = np.asarray(r["Y"], dtype=np.complex128)
    Q, P = np.eye(m, dtype=np.complex128), np.eye(n, dtype=np.complex128)
    for i in range(nb):
        assert V[i, i] == 1.0 and np.all(V[:i, i] == 0)
        Hi = np.eye(m) - tauq[i] * np.outer(V[:, i], V[:, i].conj())
        assert np.allclose(Hi.conj().T @ Hi, np.eye(m), atol=1e-13), "H_i not unitary"
        Q = Q @ Hi
        if i < n - 1:
            assert U[i + 1, i] == 1.0 and np.all(U[:i + 1, i] == 0)
        Gi = np.eye(n) - taup[i] * np.outer(U[:, i], U[:, i].conj())
        assert np.allclose(Gi.conj().T @ Gi, np.eye(n), atol=1e-13), "G_i not unitary"
        P = P @ Gi
    B = Q.conj().T @ A128 @ P
    scale = np.linalg.norm(A128)
    for i in range(nb):
        assert abs(B[i, i] - d[i]) < 1e-13 * scale, "diagonal is not the real d"
        assert np.all(np.abs(B[i + 1:, i]) < 1e-13 * scale), "column not reduced"
        if i < n - 1:
            assert abs(B[i, i + 1] - e[i]) < 1e-13 * scale, "superdiagonal is not the real e"
            assert np.all(np.abs(B[i, i + 2:]) < 1e-13 * scale), "row not reduced"
        assert np.all(np.abs(B[i, :i]) < 1e-13 * scale)
    upd = A128 - V @ Y.conj().T - X @ U.conj().T
    assert np.allclose(upd[nb:, nb:], B[nb:, nb:], atol=1e-12 * scale)
    assert np.array_equal(np.asarray(r["A"])[nb:, nb:].astype(np.complex128), A128[nb:, nb:])


def test_complex_full_reduction_keeps_singular_values():
    rng = np.random.default_rng(4)
    m, n = 45, 30
    A0 = rng.uniform(-1, 1, (m, n)) + 1j * rng.uniform(-1, 1, (m, n))
    r = go.gebrd_panel(A0, n)
    d = np.asarray(r["d"], dtype=np.float64)
    e = np.asarray(r["e"], dtype=np.float64)[: n - 1]
    B = np.diag(d) + np.diag(e, 1)
    assert np.allclose(np.linalg.svd(B, compute_uv=False), np.linalg.svd(A0, compute_uv=False), atol=1e-12)


def test_complex_panel_reduces_to_the_real_one_on_real_data():
    rng = np.random.default_rng(5)
    A0 = rng.uniform(-1, 1, (30, 20))
    rr, rc = go.gebrd_panel(A0, 8), go.gebrd_panel(A0.astype(np.complex128), 8)
    for key in ("A", "d", "e", "tauq", "taup", "X", "Y"):
        got = np.asarray(rc[key], dtype=np.complex128)
        assert np.max(np.abs(got.imag)) == 0
        assert np.allclose(got.real, np.asarray(rr[key], dtype=np.float64), atol=1e-14)


# ---- more columns than rows: lower bidiagonal form

@pytest.mark.parametrize("dtype", [np.float32, np.float64, np.complex64, np.complex128])
@pytest.mark.parametrize("m,n,nb", [(1, 2, 1), (2, 3, 2), (3, 5, 2), (40, 41, 8), (61, 97, 32), (33, 50, 33)])
def test_wide_matrices_lower_bidiagonal_identities(dtype, m, n, nb):
    rng = np.random.default_rng(m * 1000 + n * 10 + nb + 11)
    A0 = rng.uniform(-1, 1, (m, n))
    if np.issubdtype(dtype, np.complexfloating):
        A0 = A0 + 1j * rng.uniform(-1, 1, (m, n))
    A0 = A0.astype(dtype)
    r = go.gebrd_panel_wide(A0, nb)
    Aw = A0.astype(np.complex128)
    out = np.asarray(r["A"], dtype=np.complex128)
    tauq = np.asarray(r["tauq"], dtype=np.complex128)
    taup = np.asarray(r["taup"], dtype=np.complex128)
    d = np.asarray(r["d"], dtype=np.float64)
    e = np.asarray(r["e"], dtype=np.float64)
    X = np.asarray(r["X"], dtype=np.complex128)
    Y = np.asarray(r["Y"], dtype=np.complex128)
    assert np.isrealobj(r["d"]) and np.isrealobj(r["e"])
    V = np.zeros((m, nb), dtype=np.complex128)
    U = np.zeros((n, nb), dtype=np.complex128)
    Q, P = np.eye(m, dtype=np.complex128), np.eye(n, dtype=np.complex128)
    for i in range(nb):
        U[i:, i] = out[i, i:].conj()             # the row stores u^H
        assert U[i, i] == 1.0
        if i < m - 1:
            V[i + 1:, i] = out[i + 1:, i]
            assert V[i + 1, i] == 1.0
        Gi = np.eye(n) - taup[i] * np.outer(U[:, i], U[:, i].conj())
        Hi = np.eye(m) - tauq[i] * np.outer(V[:, i], V[:, i].conj())
        assert np.allclose(Gi.conj().T @ Gi, np.eye(n), atol=1e-13) and np.allclose(Hi.conj().T @ Hi, np.eye(m), atol=1e-13)
        P, Q = P @ Gi, Q @ Hi
    B = Q.conj().T @ Aw @ P
    scale = np.linalg.norm(Aw)
    for i in range(nb):
        assert abs(B[i, i] - d[i]) < 1e-13 * scale, "diagonal is not the real d"
        assert np.all(np.abs(B[i, i + 1:]) < 1e-13 * scale), "row not reduced"
        if i < m - 1:
            assert abs(B[i + 1, i] - e[i]) < 1e-13 * scale, "subdiagonal is not the real e"
            assert np.all(np.abs(B[i + 2:, i]) < 1e-13 * scale), "column not reduced"
        assert np.all(np.abs(B[:i, i]) < 1e-13 * scale)
    upd = Aw - V @ Y.conj().T - X @ U.conj().T
    assert np.allclose(upd[nb:, nb:], B[nb:, nb:], atol=1e-12 * scale)
    assert np.array_equal(out[nb:, nb:], Aw[nb:, nb:])


def test_wide_panel_is_the_tall_panel_of_the_conjugate_transpose():
    """lower bidiagonal reduction of A (m < n) = upper bidiagonal reduction of A^H, with the roles of the
    row and the column reflectors (and of X and Y) exchanged"""
    rng = np.random.default_rng(21)
    m, n, nb = 30, 45, 9
    A0 = rng.uniform(-1, 1, (m, n)) + 1j * rng.uniform(-1, 1, (m, n))
    w, t = go.gebrd_panel_wide(A0, nb), go.gebrd_panel(A0.conj().T.copy(), nb)
    c = lambda a: np.asarray(a, dtype=np.complex128)
    assert np.allclose(c(w["d"]), c(t["d"]), atol=1e-13) and np.allclose(c(w["e"]), c(t["e"]), atol=1e-13)
    # row i of A is the conjugate of column i of A^H, and the row reflector is generated from the conjugated row:
    # the same vector, the same tau; what differs is the storage (a row holds u^H, a column holds v)
    assert np.allclose(c(w["taup"]), c(t["tauq"]), atol=1e-13) and np.allclose(c(w["tauq"]), c(t["taup"]), atol=1e-13)
    wa, ta = c(w["A"]), c(t["A"])
    for i in range(nb):
        assert np.allclose(wa[i, i:], ta[i:, i].conj(), atol=1e-13)
        assert np.allclose(wa[i + 1:, i], ta[i, i + 1:].conj(), atol=1e-13)
    assert np.allclose(c(w["X"]), c(t["Y"]), atol=1e-12) and np.allclose(c(w["Y"]), c(t["X"]), atol=1e-12)


def test_wide_full_reduction_keeps_singular_values():
    rng = np.random.default_rng(22)
    m, n = 30, 45
    A0 = rng.uniform(-1, 1, (m, n))
    r = go.gebrd_panel_wide(A0, m)
    d = np.asarray(r["d"], dtype=np.float64)
    e = np.asarray(r["e"], dtype=np.float64)[: m - 1]
    B = np.diag(d) + np.diag(e, -1)
    assert np.allclose(np.linalg.svd(B, compute_uv=False), np.linalg.svd(A0, compute_uv=False), atol=1e-12)
