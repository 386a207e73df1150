"""Pins of the panel-step oracle (`oracle/panel_oracle.py`) against things it does not compute itself:
a hand-worked 3 x 3 case, and numpy linear algebra on the explicitly formed reflectors (orthogonality,
tridiagonal leading columns, the trailing-block identity, eigenvalues of a full reduction); the upper-storage
panel additionally against the lower-storage one on the matrix with rows and columns reversed."""
import numpy as np
import pytest

from oracle import panel_oracle as po


def sym_lower(rng, n, dtype=np.float64):
    """random symmetric matrix given by its lower triangle; the strict upper triangle is NaN"""
    A = rng.uniform(-1, 1, (n, n)).astype(dtype)
    A[np.triu_indices(n, 1)] = np.nan
    return A


def completed(A):
    L = np.tril(A).astype(np.float64)
    return L + np.tril(L, -1).T


def reflectors(res, n, nb):
    """V (n x nb, zero above the leading ones) from the panel result"""
    V = np.zeros((n, nb))
    for j in range(min(nb, n - 1)):
        V[j + 1:, j] = np.asarray(res["A"][j + 1:, j], dtype=np.float64)
    return V


def q_of(V, tau):
    n, nb = V.shape
    Q = np.eye(n)
    for j in range(nb):
        Q = Q @ (np.eye(n) - float(tau[j]) * np.outer(V[:, j], V[:, j]))
    return Q


def test_hand_worked_three_by_three():
    # a = (4,3,4): alpha = 3, x = (4), beta = -5, tau = 8/5, v = (1, 1/2);
    # S22 v = (5/2, 7/2), times tau = (4, 28/5), w.v = 34/5, w - (4/5)(34/5) v = (-36/25, 72/25)
    A = np.array([[4.0, np.nan, np.nan], [3.0, 2.0, np.nan], [4.0, 1.0, 5.0]])
    r = po.sytrd_panel(A, 1)
    assert float(r["e"][0]) == -5.0 and abs(float(r["tau"][0]) - 1.6) < 1e-18
    assert float(r["A"][0, 0]) == 4.0 and float(r["A"][1, 0]) == 1.0 and float(r["A"][2, 0]) == 0.5
    assert np.allclose(np.asarray(r["W"][:, 0], dtype=np.float64), [0.0, -1.44, 2.88], rtol=0, atol=1e-15)
    # the untouched trailing columns keep their input values
    assert float(r["A"][1, 1]) == 2.0 and float(r["A"][2, 1]) == 1.0 and float(r["A"][2, 2]) == 5.0


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("n,nb", [(2, 1), (5, 2), (40, 8), (97, 32), (64, 64), (33, 33)])
def test_similarity_transform_identities(dtype, n, nb):
    rng = np.random.default_rng(n * 100 + nb)
    A = sym_lower(rng, n, dtype)
    S = completed(A)
    r = po.sytrd_panel(A, nb)
    assert np.all(np.isfinite(np.asarray(r["W"], dtype=np.float64))), "the NaN triangle was read"
    V = reflectors(r, n, nb)
    tau = np.asarray(r["tau"], dtype=np.float64)
    W = np.asarray(r["W"], dtype=np.float64).copy()
    for j in range(nb):
        W[: j + 1, j] = 0.0                   # rows 0..j of column j are scratch / not part of w_j
        vv = V[:, j] @ V[:, j]
        assert tau[j] == 0 or abs(tau[j] * vv - 2.0) < 1e-13, "H_j is not orthogonal"
        if j < n - 1:
            assert V[j + 1, j] == 1.0
    Q = q_of(V, tau)
    assert np.allclose(Q.T @ Q, np.eye(n), atol=1e-13)
    T = Q.T @ S @ Q
    d = np.asarray(np.diag(r["A"]), dtype=np.float64)
    e = np.asarray(r["e"], dtype=np.float64)
    scale = np.linalg.norm(S)
    for j in range(nb):
        assert abs(T[j, j] - d[j]) < 1e-13 * scale
        if j < n - 1:
            assert abs(T[j + 1, j] - e[j]) < 1e-13 * scale
            assert np.all(np.abs(T[j + 2:, j]) < 1e-13 * scale), "column is not reduced"
    # trailing block: A - V W^T - W V^T equals the transformed matrix there
    upd = S - V @ W.T - W @ V.T
    assert np.allclose(upd[nb:, nb:], T[nb:, nb:], atol=1e-12 * scale)


def test_full_reduction_keeps_eigenvalues():
    rng = np.random.default_rng(5)
    n = 48
    A = sym_lower(rng, n)
    r = po.sytrd_panel(A, n)
    d = np.asarray(np.diag(r["A"]), dtype=np.float64)
    e = np.asarray(r["e"], dtype=np.float64)[: n - 1]
    T = np.diag(d) + np.diag(e, -1) + np.diag(e, 1)
    assert np.allclose(np.linalg.eigvalsh(T), np.linalg.eigvalsh(completed(A)), atol=1e-12)


def test_already_reduced_inputs():
    n = 12
    rng = np.random.default_rng(6)
    # diagonal matrix: nothing to annihilate, alpha = 0: tau = 0, e = 0
    D = np.diag(rng.uniform(1, 2, n))
    r = po.sytrd_panel(D, 5)
    assert np.all(np.asarray(r["tau"], dtype=np.float64) == 0) and np.all(np.asarray(r["e"], dtype=np.float64) == 0)
    # tridiagonal matrix: tau = 0 and e is the subdiagonal, d the diagonal
    sub = rng.uniform(1, 2, n - 1)
    T = D + np.diag(sub, -1)
    r = po.sytrd_panel(T, 6)
    assert np.all(np.asarray(r["tau"], dtype=np.float64) == 0)
    assert np.array_equal(np.asarray(r["e"], dtype=np.float64), sub[:6])
    assert np.array_equal(np.asarray(np.diag(r["A"]), dtype=np.float64)[:6], np.diag(D)[:6])
    assert np.all(np.asarray(r["W"], dtype=np.float64) == 0)


def test_working_precision_mode_is_close_to_the_wide_one():
    rng = np.random.default_rng(7)
    A = sym_lower(rng, 60, np.float32)
    a = po.sytrd_panel(A, 16, wide=False)
    b = po.sytrd_panel(A, 16, wide=True)
    assert a["W"].dtype == np.float32 and b["W"].dtype == np.float64
    assert np.linalg.norm(a["W"] - b["W"]) < 1e-5 * np.linalg.norm(b["W"])


# ---------------------------------------------------------------- complex Hermitian ----
def herm_lower(rng, n, dtype=np.complex128):
    A = (rng.uniform(-1, 1, (n, n)) + 1j * rng.uniform(-1, 1, (n, n))).astype(dtype)
    A[np.triu_indices(n, 1)] = np.nan       # never read; the diagonal keeps a garbage imaginary part
    return A


def completed_h(A):
    L = np.tril(A).astype(np.complex128)
    L[np.arange(len(L)), np.arange(len(L))] = L.diagonal().real
    return L + np.conj(np.tril(L, -1)).T


def test_hermitian_hand_worked_two_by_two():
    # n = 2: column 0 has nothing below the subdiagonal: x is empty, alpha = 3 + 4i is not real, so the
    # reflector is a phase: beta = -|alpha| = -5, tau = (beta - alpha)/beta = 1.6 + 0.8i, v = (1)
    A = np.array([[2.0 + 9j, np.nan], [3.0 + 4j, 7.0 - 5j]])
    r = po.hetrd_panel(A, 1)
    assert float(r["e"][0]) == -5.0
    assert abs(complex(r["tau"][0]) - (1.6 + 0.8j)) < 1e-15
    assert complex(r["A"][0, 0]) == 2.0 and complex(r["A"][1, 0]) == 1.0
    # w = tau * 7 * 1 - (tau/2) * conj(tau * 7) * 1 ... evaluated directly
    t = 1.6 + 0.8j
    w = t * 7.0
    w = w - (t / 2) * np.conj(w)
    assert abs(complex(r["W"][1, 0]) - w) < 1e-14


@pytest.mark.parametrize("dtype", [np.complex64, np.complex128])
@pytest.mark.parametrize("n,nb", [(2, 1), (5, 2), (40, 8), (97, 32), (48, 48)])
def test_hermitian_similarity_identities(dtype, n, nb):
    rng = np.random.default_rng(n * 7 + nb)
    A = herm_lower(rng, n, dtype)
    S = completed_h(A)
    r = po.hetrd_panel(A, nb)
    W = np.asarray(r["W"], dtype=np.complex128).copy()
    assert np.all(np.isfinite(W)), "the NaN triangle was read"
    tau = np.asarray(r["tau"], dtype=np.complex128)
    e = np.asarray(r["e"], dtype=np.float64)
    V = np.zeros((n, nb), dtype=np.complex128)
    for j in range(min(nb, n - 1)):
        V[j + 1:, j] = np.asarray(r["A"][j + 1:, j], dtype=np.complex128)
        assert V[j + 1, j] == 1.0
    Q = np.eye(n, dtype=np.complex128)
    for j in range(nb):
        W[: j + 1, j] = 0.0
        H = np.eye(n) - tau[j] * np.outer(V[:, j], np.conj(V[:, j]))
        assert np.allclose(np.conj(H).T @ H, np.eye(n), atol=1e-13), "H_j is not unitary"
        Q = Q @ H
    T = np.conj(Q).T @ S @ Q
    d = np.asarray(np.diag(r["A"]), dtype=np.complex128)
    scale = np.linalg.norm(S)
    for j in range(nb):
        assert d[j].imag == 0 and abs(T[j, j] - d[j]) < 1e-13 * scale
        if j < n - 1:
            assert abs(T[j + 1, j] - e[j]) < 1e-13 * scale, "subdiagonal is not the real e"
            assert np.all(np.abs(T[j + 2:, j]) < 1e-13 * scale), "column is not reduced"
    upd = S - V @ np.conj(W).T - W @ np.conj(V).T
    assert np.allclose(upd[nb:, nb:], T[nb:, nb:], atol=1e-12 * scale)
    if nb == n:
        Tm = np.diag(d.real) + np.diag(e[: n - 1], -1) + np.diag(e[: n - 1], 1)
        assert np.allclose(np.linalg.eigvalsh(Tm), np.linalg.eigvalsh(S), atol=1e-12)


# ---------------------------------------------------------------- upper storage ----
def upper_input(rng, n, dtype):
    if np.issubdtype(dtype, np.complexfloating):
        A = (rng.uniform(-1, 1, (n, n)) + 1j * rng.uniform(-1, 1, (n, n))).astype(dtype)
    else:
        A = rng.uniform(-1, 1, (n, n)).astype(dtype)
    A[np.tril_indices(n, -1)] = np.nan       # the strict lower triangle is never read
    return A


def completed_upper(A):
    U = np.triu(A).astype(np.complex128 if np.iscomplexobj(A) else np.float64)
    if np.iscomplexobj(A):
        U[np.arange(len(U)), np.arange(len(U))] = U.diagonal().real
    return U + np.conj(np.triu(U, 1)).T


def test_upper_hand_worked_three_by_three():
    # last column a = (4, 3, 4) from the top: d = 4 (bottom), alpha = a[1] = 3, x = (a[0]) = (4), beta = -5,
    # tau = 8/5, v = (1/2, 1): the mirror image of the lower 3 x 3 case, so w = (2.88, -1.44) from the top
    A = np.array([[5.0, 1.0, 4.0], [np.nan, 2.0, 3.0], [np.nan, np.nan, 4.0]])
    r = po.trd_panel_upper(A, 1)
    assert float(r["e"][0]) == -5.0 and abs(float(r["tau"][0]) - 1.6) < 1e-18
    assert float(r["A"][2, 2]) == 4.0 and float(r["A"][1, 2]) == 1.0 and float(r["A"][0, 2]) == 0.5
    assert np.allclose(np.asarray(r["W"][:, 0], dtype=np.float64), [2.88, -1.44, 0.0], rtol=0, atol=1e-15)
    assert float(r["A"][0, 0]) == 5.0 and float(r["A"][0, 1]) == 1.0 and float(r["A"][1, 1]) == 2.0


@pytest.mark.parametrize("dtype", [np.float32, np.float64, np.complex64, np.complex128])
@pytest.mark.parametrize("n,nb", [(1, 1), (2, 1), (2, 2), (5, 2), (40, 8), (97, 32), (48, 48)])
def test_upper_panel_is_the_mirror_image_of_the_lower_one(dtype, n, nb):
    """Reversing the order of rows and columns turns the upper triangle into the lower one and the last nb
    columns into the first nb: the lower-storage oracle on the reversed matrix must give the reversed results."""
    rng = np.random.default_rng(n * 100 + nb + 3)
    A = upper_input(rng, n, dtype)
    cplx = np.iscomplexobj(A)
    up = po.trd_panel_upper(A, nb)
    lo = (po.hetrd_panel if cplx else po.sytrd_panel)(A[::-1, ::-1].copy(), nb)
    wt = np.complex128 if cplx else np.float64
    assert np.allclose(np.asarray(up["e"], dtype=np.float64), np.asarray(lo["e"], dtype=np.float64)[::-1], atol=1e-13)
    assert np.allclose(np.asarray(up["tau"], dtype=wt), np.asarray(lo["tau"], dtype=wt)[::-1], atol=1e-13)
    Au, Al = np.asarray(up["A"], dtype=wt), np.asarray(lo["A"], dtype=wt)[::-1, ::-1]
    iu = np.triu_indices(n)
    assert np.allclose(Au[iu], Al[iu], atol=1e-13)
    Wu, Wl = np.asarray(up["W"], dtype=wt), np.asarray(lo["W"], dtype=wt)[::-1, ::-1]
    for iw in range(nb):
        i = n - nb + iw
        assert np.allclose(Wu[:i, iw], Wl[:i, iw], atol=1e-13)


@pytest.mark.parametrize("dtype", [np.float64, np.complex128])
@pytest.mark.parametrize("n,nb", [(5, 2), (40, 8), (33, 33)])
def test_upper_similarity_identities(dtype, n, nb):
    rng = np.random.default_rng(n * 100 + nb + 4)
    A = upper_input(rng, n, dtype)
    S = completed_upper(A)
    r = po.trd_panel_upper(A, nb)
    wt = S.dtype
    W = np.asarray(r["W"], dtype=wt).copy()
    assert np.all(np.isfinite(W)), "the NaN triangle was read"
    tau = np.asarray(r["tau"], dtype=wt)
    e = np.asarray(r["e"], dtype=np.float64)
    out = np.asarray(r["A"], dtype=wt)
    V = np.zeros((n, nb), dtype=wt)
    Q = np.eye(n, dtype=wt)
    for iw in range(nb - 1, -1, -1):
        i = n - nb + iw
        W[i:, iw] = 0                          # rows i.. of that column are scratch
        if i > 0:
            V[:i, iw] = out[:i, i]
            assert V[i - 1, iw] == 1.0
        Hi = np.eye(n, dtype=wt) - tau[iw] * np.outer(V[:, iw], np.conj(V[:, iw]))
        assert np.allclose(np.conj(Hi).T @ Hi, np.eye(n), atol=1e-13), "H_i is not unitary"
        Q = Q @ Hi
    T = np.conj(Q).T @ S @ Q
    scale = np.linalg.norm(S)
    for iw in range(nb):
        i = n - nb + iw
        assert abs(T[i, i] - out[i, i]) < 1e-13 * scale and out[i, i].imag == 0
        if i > 0:
            assert abs(T[i - 1, i] - e[iw]) < 1e-13 * scale, "superdiagonal is not the real e"
            assert np.all(np.abs(T[:i - 1, i]) < 1e-13 * scale), "column is not reduced"
    upd = S - V @ np.conj(W).T - W @ np.conj(V).T
    m = n - nb
    assert np.allclose(upd[:m, :m], T[:m, :m], atol=1e-12 * scale)
    # columns before the panel keep their input values (of a complex diagonal the real part: the rest is not read)
    iu = np.triu_indices(n)
    keep = iu[1] < m
    ref = np.triu(A).astype(wt)
    ref[np.arange(n), np.arange(n)] = ref.diagonal().real
    assert np.array_equal(out[iu][keep], ref[iu][keep])
