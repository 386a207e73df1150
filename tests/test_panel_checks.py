"""The checks that the GPU panel tests apply (tests/panel_checks.py), tried on the CPU: the wide oracle's own
results satisfy every identity to the roundoff of the wider type, and a planted mistake in any output (a
companion-panel entry, an off-diagonal element, a tau, a reflector entry) is caught at the tolerance of a single
product; the deviation rule accepts the working-precision oracle and rejects a result that is off by more than
the stated factor."""
import numpy as np
import pytest

from oracle import gebrd_panel_oracle as go
from oracle import panel_oracle as po

import panel_checks as pc

DT = {"s": np.float32, "d": np.float64, "c": np.complex64, "z": np.complex128}


def matrix(prec, m, n, seed):
    rng = np.random.default_rng(seed)
    a = rng.uniform(-1, 1, (m, n))
    if prec in "cz":
        a = a + 1j * rng.uniform(-1, 1, (m, n))
    return a.astype(DT[prec])


@pytest.mark.parametrize("prec", "sdcz")
@pytest.mark.parametrize("uplo", "LU")
@pytest.mark.parametrize("n,nb", [(1, 1), (2, 2), (5, 2), (40, 40), (150, 12)])
def test_trd_identities_hold_for_the_oracle_and_catch_mistakes(prec, uplo, n, nb):
    A0 = matrix(prec, n, n, 10 * n + nb)
    if uplo == "U":
        w = po.trd_panel_upper(A0, nb)
    else:
        w = (po.sytrd_panel if prec in "sd" else po.hetrd_panel)(A0, nb)
    A1, tau, e, W = np.asarray(w["A"]), np.asarray(w["tau"]), np.asarray(w["e"]), np.asarray(w["W"])
    eps = 1e-14 if prec in "sc" else 1e-17
    assert max(pc.trd_identities(prec, uplo, A0, A1, tau, e, W, nb)) <= eps
    pc.check_identities(prec, "oracle", pc.trd_identities(prec, uplo, A0, A1, tau, e, W, nb))
    if n < 5:
        return
    slot = min(nb - 1, n - 3) if uplo == "L" else max(0, 2 - (n - nb))   # a slot whose reflector has a tail
    col = slot if uplo == "L" else n - nb + slot
    tol = pc.IDENTITY_TOL[prec]
    if nb < n:                                                # a companion-panel entry that the trailing block uses
        Wb = W.copy()
        Wb[(n - 1) if uplo == "L" else 0, slot] += 1e-3
        assert pc.trd_identities(prec, uplo, A0, A1, tau, e, Wb, nb)[2] > tol
    eb = e.copy()
    eb[slot] *= 1 + 1e-3
    assert pc.trd_identities(prec, uplo, A0, A1, tau, eb, W, nb)[1] > tol
    tb = tau.copy()
    tb[slot] *= 1 + 1e-3
    assert pc.trd_identities(prec, uplo, A0, A1, tb, e, W, nb)[0] > tol
    Ab = A1.copy()
    row = n - 1 if uplo == "L" else 0
    if row != col and abs(row - col) > 1:
        Ab[row, col] += 1e-3                                  # a reflector entry
        assert max(pc.trd_identities(prec, uplo, A0, Ab, tau, e, W, nb)) > tol


@pytest.mark.parametrize("prec", "sdcz")
@pytest.mark.parametrize("m,n,nb", [(1, 1, 1), (5, 3, 3), (90, 70, 8), (3, 5, 3), (70, 90, 8), (40, 41, 40)])
def test_gebrd_identities_hold_for_the_oracle_and_catch_mistakes(prec, m, n, nb):
    A0 = matrix(prec, m, n, 7 * m + n)
    w = (go.gebrd_panel if m >= n else go.gebrd_panel_wide)(A0, nb)
    args = [np.asarray(w[k]) for k in ("A", "d", "e", "tauq", "taup", "X", "Y")]
    eps = 1e-14 if prec in "sc" else 1e-17
    assert max(pc.gebrd_identities(prec, A0, *args, nb)) <= eps
    if min(m, n) < 50:
        return
    tol = pc.IDENTITY_TOL[prec]
    for k, pos, which in ((5, (m - 1, 0), 2), (6, (n - 1, 1), 2), (1, (2,), 1), (2, (2,), 1), (3, (2,), 0), (4, (2,), 0)):
        bad = [a.copy() for a in args]
        if k >= 5:
            bad[k][pos] += 1e-3
        else:
            bad[k][pos] *= 1 + 1e-3
        assert pc.gebrd_identities(prec, A0, *bad, nb)[which] > tol, (k, pos)


@pytest.mark.parametrize("prec", "sd")
def test_deviation_rule(prec):
    A0 = matrix(prec, 200, 200, 3)
    wide, work = po.sytrd_panel(A0, 16), po.sytrd_panel(A0, 16, wide=False)
    pc.against_oracles(prec, "the working-precision oracle itself", work["W"], wide["W"], work["W"])
    dev = pc.deviation(prec, work["W"], wide["W"])
    assert 0 < dev < pc.IDENTITY_TOL[prec]
    off = np.asarray(wide["W"], dtype=np.float64) * (1 + 2 * pc.K_DEV * dev + 64 * pc.UNIT[prec])
    with pytest.raises(AssertionError):
        pc.against_oracles(prec, "a result off by twice the allowed factor", off, wide["W"], work["W"])
