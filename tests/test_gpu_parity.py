"""GPU parity tests: every product goes through the C ABI (ctypes binding) and is
compared with the CPU oracle on the same seeded inputs.

Bars: integer-valued inputs (every summation order is exact) must match
bitwise; random inputs must match the extended-accumulation oracle within a
normwise relative error of 1e-5 (s, c) / 1e-13 (d, z), and every component
within the order-independent bound gamma_{n+2} * (|alpha||A||x| + |beta||y|).
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1410_1726_amd import workloads as wl

from gpu_util import DEV, check, errors, gemv_case, kmv, logical, symv_case

pytestmark = pytest.mark.gpu

PRECS = "sdcz"
TINY = [1, 2, 3, 5, 8, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257]


def scalars(prec, a, b):
    """complex routines get scalars with an imaginary part"""
    if prec in "cz":
        return complex(a, 0.25 * a), complex(b, -0.5 * b)
    return a, b


# ------------------------------------------------------------------ GEMV ----
@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("trans", "NTC")
def test_gemv_tiny_shapes_bitwise(prec, trans):
    """small integers: exact in any order, so GPU == oracle bit for bit; covers
    every combination of head / tail / single-tile shapes"""
    alpha, beta = scalars(prec, 2, -3)
    for i, m in enumerate(TINY):
        for n in TINY[i % 3:: 3]:
            got, err, ex = gemv_case(prec, trans, m, n, alpha, beta, dist="smallint", seed=m * 7 + n, lda=m + (n % 4))
            assert np.array_equal(got.astype(ex["want"].dtype), ex["want"]), (m, n, err)


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("trans", "NT")
@pytest.mark.parametrize("m,n", [(1024, 1024), (1000, 1000), (4099, 4099), (2500, 700), (700, 2500), (5000, 33), (33, 5000)])
def test_gemv_medium_full_oracle(prec, trans, m, n):
    """several tiles, ragged tails, lda == m (per-column alignment drift for the odd sizes)"""
    alpha, beta = scalars(prec, 1.0, 1.0)
    _, err, _ = gemv_case(prec, trans, m, n, alpha, beta, seed=1)
    check(prec, err, f"{prec}gemv {trans} {m}x{n}")


def test_dgemv_config1():
    """DGEMV N, m = n = lda = 1024, U[-1,1], alpha 1.5, beta 0.5, seed 0"""
    _, err, _ = gemv_case("d", "N", 1024, 1024, 1.5, 0.5, seed=0)
    check("d", err, "config 1")


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("trans", "NC")
@pytest.mark.parametrize("incx,incy", [(2, 1), (1, 2), (-1, -1), (-3, 2)])
def test_gemv_strides(prec, trans, incx, incy):
    alpha, beta = scalars(prec, 0.7, 0.3)
    _, err, _ = gemv_case(prec, trans, 777, 1301, alpha, beta, incx=incx, incy=incy, lda=800, seed=2)
    check(prec, err, f"{prec}gemv {trans} inc {incx},{incy}")


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("trans", "NT")
@pytest.mark.parametrize("off", [1, 17, 63, 1000])
def test_gemv_subblock_offsets(prec, trans, off):
    """sub-block at (off, off) of a parent whose lda keeps columns 128-byte
    aligned; everything outside the block is NaN"""
    m, n, lda = 1500, 900, 2560
    alpha, beta = scalars(prec, -1.0, 1.0)
    _, err, _ = gemv_case(prec, trans, m, n, alpha, beta, lda=lda, row_off=off, col_off=off, seed=3)
    check(prec, err, f"{prec}gemv {trans} offset {off}")
    # and with a leading dimension that drifts the alignment column by column
    _, err, _ = gemv_case(prec, trans, 600, 500, alpha, beta, lda=600 + off + 3, row_off=off, col_off=2, seed=4)
    check(prec, err, f"{prec}gemv {trans} offset {off} odd lda")


@pytest.mark.parametrize("prec", PRECS)
def test_gemv_alpha_beta_special_cases(prec):
    k = kmv()
    m, n = 300, 200
    dt = wl.TORCH_DTYPES[prec]
    nan = float("nan")
    A = torch.full((n, m), nan, dtype=dt, device=DEV)
    x = torch.full((n,), nan, dtype=dt, device=DEV)
    y0 = wl.vector(prec, m, seed=5, which=2, device=DEV)
    # alpha = 0: A and x (all NaN) are not read, y = beta*y exactly
    y = y0.clone()
    k.GEMV[prec]("N", m, n, 0.0, A, m, x, 1, 0.5, y, 1)
    assert torch.equal(y, y0 * 0.5)
    # alpha = 0 and beta = 0: zeros even from a NaN y
    y = torch.full((m,), nan, dtype=dt, device=DEV)
    k.GEMV[prec]("N", m, n, 0.0, A, m, x, 1, 0.0, y, 1)
    assert torch.equal(y, torch.zeros_like(y))
    # alpha = 0 and beta = 1: y untouched
    y = y0.clone()
    k.GEMV[prec]("T", n, m, 0.0, A, n, x, 1, 1.0, y, 1)
    assert torch.equal(y, y0)
    # beta = 0: a NaN y is overwritten, never read (both the direct and the split path)
    for (mm, nn, trans) in [(300, 200, "N"), (300, 200, "T"), (64, 5000, "N"), (5000, 64, "T")]:
        Ar = wl.matrix(prec, mm, nn, seed=6, device=DEV)
        lenx, leny = (nn, mm) if trans == "N" else (mm, nn)
        xr = wl.vector(prec, lenx, seed=6, device=DEV)
        ynan = torch.full((leny,), nan, dtype=dt, device=DEV)
        yzero = torch.zeros((leny,), dtype=dt, device=DEV)
        k.GEMV[prec](trans, mm, nn, 1.0, Ar, mm, xr, 1, 0.0, ynan, 1)
        k.GEMV[prec](trans, mm, nn, 1.0, Ar, mm, xr, 1, 0.0, yzero, 1)
        assert torch.isfinite(torch.view_as_real(ynan) if ynan.is_complex() else ynan).all()
        assert torch.equal(ynan, yzero)


@pytest.mark.parametrize("prec", PRECS)
def test_identity_and_ones_closed_forms(prec):
    """A = I gives alpha*x + beta*y exactly; A = ones with integer x gives
    alpha*sum(x) + beta*y exactly, in every precision and summation order"""
    k = kmv()
    dt = wl.TORCH_DTYPES[prec]
    n = 1300
    I = torch.eye(n, dtype=dt, device=DEV)
    x = wl.vector(prec, n, seed=7, device=DEV)
    y0 = wl.vector(prec, n, seed=7, which=2, device=DEV)
    want = 2.0 * x + 0.5 * y0
    for trans in "NTC":
        y = y0.clone()
        k.GEMV[prec](trans, n, n, 2.0, I, n, x, 1, 0.5, y, 1)
        assert torch.equal(y, want)
    for uplo in "LU":
        y = y0.clone()
        k.SYMV[prec](uplo, n, 2.0, wl.poison_triangle(I.clone(), n, uplo), n, x, 1, 0.5, y, 1)
        assert torch.equal(y, want)
    m = 2100
    ones = torch.ones((n, m), dtype=dt, device=DEV)          # m x n matrix of ones
    xi = wl.vector(prec, n, dist="smallint", seed=8, device=DEV)
    yi = wl.vector(prec, m, dist="smallint", seed=8, which=2, device=DEV)
    y = yi.clone()
    k.GEMV[prec]("N", m, n, 2.0, ones, m, xi, 1, 4.0, y, 1)
    assert torch.equal(y, 2.0 * xi.sum() + 4.0 * yi)
    xt = wl.vector(prec, m, dist="smallint", seed=9, device=DEV)
    yt = wl.vector(prec, n, dist="smallint", seed=9, which=2, device=DEV)
    y = yt.clone()
    k.GEMV[prec]("T", m, n, 2.0, ones, m, xt, 1, 4.0, y, 1)
    assert torch.equal(y, 2.0 * xt.sum() + 4.0 * yt)
    sq = torch.ones((n, n), dtype=dt, device=DEV)
    for uplo in "LU":
        y = torch.zeros(n, dtype=dt, device=DEV)
        k.SYMV[prec](uplo, n, 2.0, wl.poison_triangle(sq.clone(), n, uplo), n, xi, 1, 0.0, y, 1)
        assert torch.equal(y, (2.0 * xi.sum()).expand(n))


# ------------------------------------------------------------- SYMV / HEMV ----
@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("uplo", "LU")
def test_symv_tiny_shapes_bitwise(prec, uplo):
    alpha, beta = scalars(prec, 2, -3)
    for n in TINY + [300, 513]:
        got, err, ex = symv_case(prec, uplo, n, alpha, beta, dist="smallint", seed=n, lda=n + (n % 5),
                                 nan_imag_diag=True)
        assert np.array_equal(got.astype(ex["want"].dtype), ex["want"]), (n, err)


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("uplo", "LU")
@pytest.mark.parametrize("n", [1024, 1000, 2048, 4099])
def test_symv_medium_full_oracle(prec, uplo, n):
    """config 3 shape: referenced triangle random, other triangle NaN, beta = 0
    with a NaN y; n = 1000 / 4099 add ragged panels and alignment drift"""
    _, err, _ = symv_case(prec, uplo, n, 1.0, 0.0, seed=10, nan_imag_diag=True)
    check(prec, err, f"symv {prec} {uplo} n={n}")


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("uplo", "LU")
@pytest.mark.parametrize("incx,incy", [(2, 1), (-1, 3), (1, -2)])
def test_symv_strides_and_scalars(prec, uplo, incx, incy):
    alpha, beta = scalars(prec, 0.7, 0.3)
    _, err, _ = symv_case(prec, uplo, 1237, alpha, beta, incx=incx, incy=incy, lda=1300, seed=11)
    check(prec, err, f"symv {prec} {uplo} inc {incx},{incy}")


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("uplo", "LU")
@pytest.mark.parametrize("off", [1, 17, 63, 1000])
def test_symv_subblock_offsets(prec, uplo, off):
    alpha, beta = scalars(prec, -1.0, 1.0)
    _, err, _ = symv_case(prec, uplo, 1100, alpha, beta, lda=2304, off=off, seed=12)
    check(prec, err, f"symv {prec} {uplo} offset {off}")


@pytest.mark.parametrize("prec", PRECS)
def test_symv_alpha_zero(prec):
    k = kmv()
    n = 500
    dt = wl.TORCH_DTYPES[prec]
    A = torch.full((n, n), float("nan"), dtype=dt, device=DEV)
    x = torch.full((n,), float("nan"), dtype=dt, device=DEV)
    y0 = wl.vector(prec, n, seed=13, which=2, device=DEV)
    y = y0.clone()
    k.SYMV[prec]("L", n, 0.0, A, n, x, 1, 0.5, y, 1)
    assert torch.equal(y, y0 * 0.5)


# ------------------------------------------------------------ determinism ----
@pytest.mark.parametrize("prec", PRECS)
def test_bitwise_reproducible(prec):
    """partial sums meet in a workspace in a fixed order: repeated calls agree bit for bit"""
    k = kmv()
    n = 3000
    A = wl.matrix(prec, n, n, seed=14, device=DEV)
    x = wl.vector(prec, n, seed=14, device=DEV)
    y0 = wl.vector(prec, n, seed=14, which=2, device=DEV)
    for call in (lambda y: k.GEMV[prec]("N", n, n, 0.7, A, n, x, 1, 0.3, y, 1),
                 lambda y: k.GEMV[prec]("T", n, n, 0.7, A, n, x, 1, 0.3, y, 1),
                 lambda y: k.SYMV[prec]("L", n, 0.7, A, n, x, 1, 0.3, y, 1),
                 lambda y: k.SYMV[prec]("U", n, 0.7, A, n, x, 1, 0.3, y, 1)):
        ref = y0.clone()
        call(ref)
        for _ in range(5):
            y = y0.clone()
            call(y)
            assert torch.equal(y, ref)


def test_split_variants_agree_with_oracle():
    """every cross-workgroup split count goes through the same fixed-order reduction"""
    k = kmv()
    try:
        for key, trans in (("gemv_n_splits", "N"), ("gemv_t_splits", "T")):
            for s in (1, 2, 3, 7, 16):
                k.set_tuning(key, s)
                _, err, _ = gemv_case("d", trans, 2100, 1900, 0.7, 0.3, seed=15)
                check("d", err, f"{key}={s}")
        # GEMV-T with fewer workgroups than column groups (each takes several), alone, with row splits, and with
        # alignment classes
        for wgs, splits, lda in ((1, 0, 2100), (7, 0, 2100), (100, 3, 2100), (192, 0, 2100), (5, 2, 2111)):
            k.set_tuning("gemv_t_wgs", wgs)
            k.set_tuning("gemv_t_splits", splits)
            for prec, trans in (("d", "T"), ("c", "C"), ("s", "T")):
                _, err, _ = gemv_case(prec, trans, 2100, 1900, 0.7, 0.3, lda=lda, seed=17)
                check(prec, err, f"gemv_t_wgs={wgs} splits={splits} lda={lda} {prec}gemv {trans}")
        k.set_tuning("gemv_t_wgs", 0)
        k.set_tuning("gemv_t_splits", 0)
        # columns grouped by alignment class (leading dimension no multiple of 128 bytes), forced on for small
        # and ragged shapes, with few and many splits, classes with no column at all (n below the period)
        k.set_tuning("gemv_align_classes", 2)
        for prec, m, n, lda in (("d", 2100, 1900, 2111), ("s", 700, 45, 701), ("z", 300, 9, 333), ("c", 4099, 260, 4100),
                                ("d", 3, 50, 5), ("s", 1, 7, 3)):
            for key, trans, splits in (("gemv_n_splits", "N", 0), ("gemv_n_splits", "N", 64), ("gemv_t_splits", "T", 0),
                                       ("gemv_t_splits", "C", 3)):
                k.set_tuning(key, splits)
                _, err, _ = gemv_case(prec, trans, m, n, 0.7, 0.3, lda=lda, row_off=1, col_off=2, seed=19)
                check(prec, err, f"alignment classes {prec}gemv {trans} {m}x{n} lda={lda} splits={splits}")
                k.set_tuning(key, 0)
        k.set_tuning("gemv_align_classes", 1)
        for trans in "NT":
            _, err, _ = gemv_case("d", trans, 4099, 4099, 0.7, 0.3, lda=4099, seed=20)
            check("d", err, f"dgemv {trans} without alignment classes")
        k.set_tuning("gemv_align_classes", 0)
        k.set_tuning("symv_variant", 2)
        for tpw, workers, fixed, edge in ((1, 1, 1, 1), (2, 3, 4, 1), (1, 8, 1, 9), (2, 5, 17, 17), (2, 256, 2, 3), (1, 16, 3, 2),
                                          (3, 1, 1, 1), (3, 7, 2, 3), (3, 256, 0, 0), (4, 1, 1, 1), (4, 6, 3, 2), (4, 256, 0, 0)):
            k.set_tuning("symv_tiles_per_wave", tpw)
            k.set_tuning("wg_target", workers)
            k.set_tuning("symv_piece_fixed", fixed)
            k.set_tuning("symv_edge_weight", edge)
            for prec, n in (("z", 1500), ("s", 2300), ("d", 3001)):
                for uplo in "LU":
                    _, err, _ = symv_case(prec, uplo, n, 0.7, 0.3, seed=16)
                    check(prec, err, f"symv tiles_per_wave={tpw} workers={workers} fixed={fixed} edge={edge} {prec} {uplo}")
    finally:
        for key in k.tuning_keys():
            k.set_tuning(key, 0)


@pytest.mark.parametrize("prec", list("sdcz"))
def test_oracle_is_handed_the_poisoned_matrix(prec):
    """medium sizes with the host copy for the oracle taken AFTER the poisoning: NaN in the unreferenced triangle,
    in the lda padding and everywhere outside the block, so an oracle loop that left the stored triangle would
    return NaN and fail the comparison (the GPU result is checked against it element by element as usual)"""
    for n, off, lda in ((3001, 0, 3008), (4099, 5, 4200), (2500, 17, 2600)):
        for uplo in "LU":
            _, err, _ = symv_case(prec, uplo, n, 0.7, 0.3, lda=lda, off=off, seed=n, oracle_sees_poison=True)
            check(prec, err, f"symv/hemv {prec} {uplo} n={n} off={off}, oracle on the poisoned copy")
            if prec in "cz":
                _, err, _ = symv_case(prec, uplo, n, 0.7 - 0.2j, 0.3j, lda=lda, off=off, seed=n, oracle_sees_poison=True,
                                      complex_symmetric=True)
                check(prec, err, f"complex symmetric symv {prec} {uplo} n={n} off={off}, oracle on the poisoned copy")


@pytest.mark.parametrize("prec", list("sdcz"))
def test_other_entry_points_against_the_oracle(prec):
    """the entry points that share kernels with the plain calls, each compared with the ORACLE (not with the
    plain GPU call): scalars in device memory, the parent + offset forms, also for the complex symmetric product"""
    k = kmv()
    dt = wl.TORCH_DTYPES[prec]
    al_v, be_v = (0.7 - 0.2j, 0.3 + 0.1j) if prec in "cz" else (0.7, 0.3)
    al = torch.tensor([al_v], dtype=dt, device=DEV)
    be = torch.tensor([be_v], dtype=dt, device=DEV)

    def dev_gemv(trans, m, n, alpha, A, lda, x, incx, beta, y, incy):
        k.GEMV_DEVSCALARS[prec](trans, m, n, al, A, lda, x, incx, be, y, incy)

    def dev_symv(uplo, n, alpha, A, lda, x, incx, beta, y, incy):
        k.SYMV_DEVSCALARS[prec](uplo, n, al, A, lda, x, incx, be, y, incy)

    for trans in "NTC":
        _, err, _ = gemv_case(prec, trans, 2100, 1900, al_v, be_v, lda=2111, seed=41, call=dev_gemv)
        check(prec, err, f"{prec}gemv_devscalars {trans}")
    for n in (900, 3001):            # one-launch kernel and the two-kernel path
        for uplo in "LU":
            _, err, _ = symv_case(prec, uplo, n, al_v, be_v, lda=n + 7, seed=42, call=dev_symv)
            check(prec, err, f"{prec} symv/hemv_devscalars {uplo} n={n}")
    # parent + offset: the call names the parent (size n + off) and the offset; the oracle gets the block
    off = 37
    for n in (800, 2900):
        def off_symv(uplo, nn, alpha, A, lda, x, incx, beta, y, incy, csym=False):
            # A, x, y as symv_case passes them describe the block; step back to the parent's first element
            Ap = A.as_strided((1,), (1,), A.storage_offset() - off * lda - off)
            xp, yp = torch.zeros(nn + off, dtype=dt, device=DEV), torch.zeros(nn + off, dtype=dt, device=DEV)
            xp[off:], yp[off:] = x, y
            (k.CSYMV_OFFSET if csym else k.SYMV_OFFSET)[prec](uplo, nn + off, alpha, Ap, lda, xp, 1, beta, yp, 1, off)
            assert torch.equal(yp[:off], torch.zeros(off, dtype=dt, device=DEV)), "wrote before the offset"
            y.copy_(yp[off:])
        for uplo in "LU":
            _, err, _ = symv_case(prec, uplo, n, al_v, be_v, lda=n + off + 3, off=off, seed=43, call=off_symv)
            check(prec, err, f"{prec} symv/hemv_offset {uplo} n={n}")
            if prec in "cz":
                _, err, _ = symv_case(prec, uplo, n, al_v, be_v, lda=n + off + 3, off=off, seed=44, complex_symmetric=True,
                                      call=lambda *a: off_symv(*a, csym=True))
                check(prec, err, f"{prec} complex symmetric symv_offset {uplo} n={n}")


@pytest.mark.parametrize("variant", [2, 3])
@pytest.mark.parametrize("prec", list("sdcz"))
def test_symv_main_kernel_variants(prec, variant):
    """the SYMV/HEMV main kernels (balanced shares of pieces; one launch for small matrices), forced
    through the tuning key, over ragged sizes, sub-block offsets, chunk heights and
    workgroup counts that make one share span several row chunks"""
    k = kmv()
    try:
        k.set_tuning("symv_variant", variant)
        for tpw, target, unit in ((0, 0, 0), (1, 3, 1), (2, 1, 2), (1, 256, 2), (2, 7, 1), (3, 5, 1), (3, 256, 0), (4, 3, 1), (4, 256, 0)):
            k.set_tuning("symv_tiles_per_wave", tpw)
            k.set_tuning("wg_target", target)
            k.set_tuning("symv_unit_tiles", unit)
            for n, off, lda in ((1, 0, None), (63, 0, None), (257, 0, 300), (1500, 17, 1792), (2048, 0, 2048),
                                (3001, 0, 3008), (4099, 1, 4112)):
                for uplo in "LU":
                    beta = 0.0 if (n + off) % 2 else 0.3
                    _, err, _ = symv_case(prec, uplo, n, 0.7, beta, lda=lda, off=off, seed=n + off, nan_imag_diag=True)
                    check(prec, err, f"variant={variant} tiles_per_wave={tpw} target={target} unit={unit} {prec} {uplo} n={n} off={off}")
    finally:
        for key in k.tuning_keys():
            k.set_tuning(key, 0)


@pytest.mark.parametrize("prec", "cz")
@pytest.mark.parametrize("uplo", "LU")
def test_complex_symmetric_symv(prec, uplo):
    """csymv / zsymv: the HEMV kernels without conjugation and with the diagonal as stored; integer data
    bitwise, then every main kernel on ragged sizes, sub-block offsets, strides and complex scalars"""
    k = kmv()
    for n in TINY + [300, 513]:
        got, err, ex = symv_case(prec, uplo, n, 2 - 1j, -3 + 2j, dist="smallint", seed=n, lda=n + (n % 5),
                                 complex_symmetric=True)
        assert np.array_equal(got.astype(ex["want"].dtype), ex["want"]), (n, err)
    # the inputs tell the two products apart: the Hermitian call gives another result
    got_s, _, ex = symv_case(prec, uplo, 300, 1.0, 0.0, dist="smallint", seed=5, complex_symmetric=True)
    got_h, _, _ = symv_case(prec, uplo, 300, 1.0, 0.0, dist="smallint", seed=5)
    assert not np.array_equal(got_s, got_h)
    try:
        for variant, unit in ((0, 0), (2, 1), (2, 2), (3, 0)):
            k.set_tuning("symv_variant", variant)
            k.set_tuning("symv_unit_tiles", unit)
            for n, off, lda, incx, incy in ((1000, 0, None, 1, 1), (1500, 17, 1792, -2, 1), (2048, 0, 2048, 1, 3),
                                            (4099, 1, 4112, 1, 1)):
                beta = 0.0 if n % 2 else 0.3 - 0.2j
                _, err, _ = symv_case(prec, uplo, n, 0.7 + 0.1j, beta, lda=lda, off=off, incx=incx, incy=incy,
                                      seed=n + off, complex_symmetric=True)
                check(prec, err, f"complex symmetric variant={variant} unit={unit} {prec} {uplo} n={n} off={off}")
    finally:
        for key in k.tuning_keys():
            k.set_tuning(key, 0)


def _bits(a):
    return np.ascontiguousarray(a).view(np.uint8)


def _sub_vector(buf, off, inc):
    """storage of the logical elements off.. of a strided parent vector (BLAS rule)"""
    return buf[off * inc:] if inc > 0 else buf[: buf.size - off * (-inc)] if off else buf


@pytest.mark.parametrize("prec", PRECS)
def test_offset_calls_name_the_parent(prec):
    """GEMV/SYMV/HEMV `_offset` entry points: parent matrix and parent vectors plus offsets.  The oracle
    computes the product with the block; parent elements outside the block are NaN, the vector elements
    before the offsets are NaN in x and must stay bit-unchanged in y."""
    k = kmv()
    alpha, beta = scalars(prec, 0.7, -0.4)
    M, N, lda = 1400, 1100, 1536
    for trans, offr, offc, incx, incy in (("N", 1, 17, 1, 1), ("T", 63, 5, 2, 1), ("C", 100, 1000, -1, -2),
                                          ("N", 0, 0, 1, 1), ("N", M, 3, 1, 1), ("T", 7, N, 1, 1)):
        parent = wl.matrix(prec, M, N, lda, seed=41, device=DEV)
        keep = parent[offc:, offr:M].clone()
        parent.fill_(float("nan"))
        parent[offc:, offr:M] = keep
        lenx, leny, offx, offy = (N, M, offc, offr) if trans == "N" else (M, N, offr, offc)
        x = wl.vector(prec, lenx, incx, seed=41, which=1, device=DEV, gap_value=float("nan"))
        y0 = wl.vector(prec, leny, incy, seed=41, which=2, device=DEV, gap_value=float("nan"))
        xl = x[:: abs(incx)]
        (xl[:offx] if incx > 0 else xl[lenx - offx:]).fill_(float("nan"))      # logical elements before the offset
        y = y0.clone()
        k.GEMV_OFFSET[prec](trans, M, N, alpha, parent, lda, x, incx, beta, y, incy, offr, offc)
        torch.cuda.synchronize()
        yh, y0h, xh = y.cpu().numpy(), y0.cpu().numpy(), x.cpu().numpy()
        m, n = M - offr, N - offc
        got_all, y0_all = logical(yh, leny, incy), logical(y0h, leny, incy)
        assert np.array_equal(_bits(got_all[:offy]), _bits(y0_all[:offy])), "wrote before the offset"
        untouched = np.ones(yh.size, dtype=bool)
        untouched[:: abs(incy)] = False
        assert np.array_equal(yh[untouched].view(np.uint8), y0h[untouched].view(np.uint8))
        if m == 0 or n == 0:
            assert np.array_equal(yh.view(np.uint8), y0h.view(np.uint8))
            continue
        Ah = parent.cpu().numpy().reshape(-1)[offc * lda + offr:]
        xs, ys = _sub_vector(xh, offx, incx), _sub_vector(y0h, offy, incy)
        kw = dict(lda=lda, incx=incx, incy=incy)
        lo, lx = (m, n) if trans == "N" else (n, m)
        want = logical(oracle.gemv(prec, trans, m, n, alpha, Ah, xs, beta, ys, mode=oracle.MODE_X, **kw), lo, incy)
        den = logical(oracle.gemv(prec, trans, m, n, alpha, Ah, xs, beta, ys, mode=oracle.MODE_ABS, **kw), lo, incy)
        check(prec, errors(prec, got_all[offy:], want, den, lx), f"{prec}gemv_offset {trans} ({offr},{offc})")
    n, lda = 1300, 1408
    for uplo, off, incx, incy in (("L", 1, 1, 1), ("U", 63, -1, 2), ("L", 1000, 2, -1), ("U", 0, 1, 1), ("L", n, 1, 1)):
        parent = wl.matrix(prec, n, n, lda, seed=42, device=DEV)
        keep = parent[off:, off:n].clone()
        parent.fill_(float("nan"))
        parent[off:, off:n] = keep
        host = parent.cpu().numpy().reshape(-1)
        if n - off:
            wl.poison_triangle(parent[off:, off:], n - off, uplo, real_diag=False)
        x = wl.vector(prec, n, incx, seed=42, which=1, device=DEV, gap_value=float("nan"))
        y0 = wl.vector(prec, n, incy, seed=42, which=2, device=DEV, gap_value=float("nan"))
        xl = x[:: abs(incx)]
        (xl[:off] if incx > 0 else xl[n - off:]).fill_(float("nan"))
        y = y0.clone()
        k.SYMV_OFFSET[prec](uplo, n, alpha, parent, lda, x, incx, beta, y, incy, off)
        torch.cuda.synchronize()
        yh, y0h, xh = y.cpu().numpy(), y0.cpu().numpy(), x.cpu().numpy()
        got_all, y0_all = logical(yh, n, incy), logical(y0h, n, incy)
        assert np.array_equal(_bits(got_all[:off]), _bits(y0_all[:off])), "wrote before the offset"
        untouched = np.ones(yh.size, dtype=bool)
        untouched[:: abs(incy)] = False
        assert np.array_equal(yh[untouched].view(np.uint8), y0h[untouched].view(np.uint8))
        nb = n - off
        if nb == 0:
            assert np.array_equal(yh.view(np.uint8), y0h.view(np.uint8))
            continue
        Ah = host[off * lda + off:]
        xs, ys = _sub_vector(xh, off, incx), _sub_vector(y0h, off, incy)
        kw = dict(lda=lda, incx=incx, incy=incy)
        want = logical(oracle.symv(prec, uplo, nb, alpha, Ah, xs, beta, ys, mode=oracle.MODE_X, **kw), nb, incy)
        den = logical(oracle.symv(prec, uplo, nb, alpha, Ah, xs, beta, ys, mode=oracle.MODE_ABS, **kw), nb, incy)
        check(prec, errors(prec, got_all[off:], want, den, nb), f"symv/hemv_offset {prec} {uplo} offset {off}")


@pytest.mark.parametrize("prec", "cz")
def test_complex_symmetric_offset_and_device_scalars(prec):
    """csymv / zsymv `_offset` and `_devscalars` forms run the kernels of the plain call (held against the
    oracle above): same bits as that call on the sub-block pointer, nothing written before the offset."""
    k = kmv()
    dt = wl.TORCH_DTYPES[prec]
    alpha, beta = scalars(prec, 0.7, -0.4)
    for n, lda, off, uplo in ((1300, 1408, 63, "L"), (1300, 1408, 1, "U"), (5000, 5000, 1000, "L"), (700, 701, 0, "U")):
        parent = wl.matrix(prec, n, n, lda, seed=52, device=DEV)
        wl.poison_triangle(parent[off:, off:], n - off, uplo, real_diag=False)
        x = wl.vector(prec, n, 1, seed=52, which=1, device=DEV)
        y0 = wl.vector(prec, n, 1, seed=52, which=2, device=DEV)
        want, got, got_dev = y0.clone(), y0.clone(), y0.clone()
        k.CSYMV[prec](uplo, n - off, alpha, parent[off:, off:], lda, x[off:], 1, beta, want[off:], 1)
        k.CSYMV_OFFSET[prec](uplo, n, alpha, parent, lda, x, 1, beta, got, 1, off)
        al = torch.tensor([alpha], dtype=dt, device=DEV)
        be = torch.tensor([beta], dtype=dt, device=DEV)
        k.CSYMV_DEVSCALARS[prec](uplo, n - off, al, parent[off:, off:], lda, x[off:], 1, be, got_dev[off:], 1)
        torch.cuda.synchronize()
        assert not torch.isnan(torch.view_as_real(want)).any()
        assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), (n, off, uplo)
        assert torch.equal(got_dev.view(torch.uint8), want.view(torch.uint8)), (n, off, uplo)


@pytest.mark.parametrize("prec", PRECS)
def test_scalars_in_device_memory(prec):
    """`_devscalars` entry points: alpha and beta are read from device memory by every kernel that ends a
    product (fused epilogues of the GEMV-N, short GEMV-N, GEMV-T and small SYMV kernels, the GEMV and SYMV
    final passes).  Same kernels and arithmetic as the host-scalar calls, so results are compared bitwise
    with those (which the other tests hold against the oracle); the value-dependent cases alpha = 0 and
    beta = 0 are checked against their definition."""
    k = kmv()
    dt = wl.TORCH_DTYPES[prec]
    al_v, be_v = scalars(prec, 0.7, -0.3)
    al = torch.tensor([al_v], dtype=dt, device=DEV)
    be = torch.tensor([be_v], dtype=dt, device=DEV)
    zero = torch.zeros(1, dtype=dt, device=DEV)
    one = torch.ones(1, dtype=dt, device=DEV)
    nan = float("nan")

    def has_nan(t):
        return bool(torch.isnan(torch.view_as_real(t) if t.is_complex() else t).any())

    try:
        # (tuning, trans, m, n): every way a GEMV ends
        for tune, trans, m, n in (({}, "N", 3000, 2000), ({"gemv_n_splits": 1}, "N", 1500, 700), ({}, "N", 64, 9000),
                                  ({"gemv_n_splits": 1}, "N", 64, 3000),
                                  ({}, "T", 2000, 3000), ({}, "C", 5000, 40), ({}, "T", 100, 5000)):
            for key, v in tune.items():
                k.set_tuning(key, v)
            A = wl.matrix(prec, m, n, m + 3, seed=7, device=DEV)
            lenx, leny = (n, m) if trans == "N" else (m, n)
            x = wl.vector(prec, lenx, 1, seed=7, which=1, device=DEV)
            y0 = wl.vector(prec, leny, 2, seed=7, which=2, device=DEV, gap_value=nan)
            want, got = y0.clone(), y0.clone()
            k.GEMV[prec](trans, m, n, al_v, A, m + 3, x, 1, be_v, want, 2)
            k.GEMV_DEVSCALARS[prec](trans, m, n, al, A, m + 3, x, 1, be, got, 2)
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), (trans, m, n, tune)
            # alpha = 0 on the device: beta*y exactly, although A and x hold NaN
            An, xn = torch.full_like(A, nan), torch.full_like(x, nan)
            got = y0.clone()
            k.GEMV_DEVSCALARS[prec](trans, m, n, zero, An, m + 3, xn, 1, be, got, 2)
            want = y0.clone()
            k.GEMV[prec](trans, m, n, 0.0, An, m + 3, xn, 1, be_v, want, 2)
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
            assert not has_nan(got[::2])
            # beta = 0 on the device: y is not read
            got = torch.full_like(y0, nan)
            want = torch.full_like(y0, nan)
            k.GEMV_DEVSCALARS[prec](trans, m, n, al, A, m + 3, x, 1, zero, got, 2)
            k.GEMV[prec](trans, m, n, al_v, A, m + 3, x, 1, 0.0, want, 2)
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
            assert not has_nan(got[::2])
            # alpha = 0, beta = 1: y keeps its values
            got = y0.clone()
            k.GEMV_DEVSCALARS[prec](trans, m, n, zero, An, m + 3, xn, 1, one, got, 2)
            assert torch.equal(got.view(torch.uint8), y0.view(torch.uint8))
            for key in tune:
                k.set_tuning(key, 0)
        for variant, n in ((3, 700), (2, 2500)):
            k.set_tuning("symv_variant", variant)
            for uplo in "LU":
                A = wl.poison_triangle(wl.matrix(prec, n, n, n + 5, seed=8, device=DEV), n, uplo)
                x = wl.vector(prec, n, 1, seed=8, which=1, device=DEV)
                y0 = wl.vector(prec, n, 1, seed=8, which=2, device=DEV)
                want, got = y0.clone(), y0.clone()
                k.SYMV[prec](uplo, n, al_v, A, n + 5, x, 1, be_v, want, 1)
                k.SYMV_DEVSCALARS[prec](uplo, n, al, A, n + 5, x, 1, be, got, 1)
                assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), (variant, uplo)
                assert not has_nan(got)
                got = y0.clone()
                k.SYMV_DEVSCALARS[prec](uplo, n, zero, torch.full_like(A, nan), n + 5, torch.full_like(x, nan), 1, be, got, 1)
                want = y0.clone()
                k.SYMV[prec](uplo, n, 0.0, A, n + 5, x, 1, be_v, want, 1)
                assert torch.equal(got, want)
                got = torch.full_like(y0, nan)
                want = torch.full_like(y0, nan)
                k.SYMV_DEVSCALARS[prec](uplo, n, al, A, n + 5, x, 1, zero, got, 1)
                k.SYMV[prec](uplo, n, al_v, A, n + 5, x, 1, 0.0, want, 1)
                assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
        # a scalar produced by an earlier kernel on the stream is seen without a host synchronisation
        k.set_tuning("symv_variant", 0)
        n = 1000
        A = wl.matrix(prec, n, n, n, seed=9, device=DEV)
        x = wl.vector(prec, n, 1, seed=9, which=1, device=DEV)
        y0 = wl.vector(prec, n, 1, seed=9, which=2, device=DEV)
        dyn = torch.zeros(1, dtype=dt, device=DEV)
        got = y0.clone()
        dyn.copy_(x[:1] * 2)                 # device-side producer
        k.GEMV_DEVSCALARS[prec]("N", n, n, dyn, A, n, x, 1, one, got, 1)
        want = y0.clone()
        k.GEMV[prec]("N", n, n, complex(dyn.cpu()[0]) if dt.is_complex else float(dyn.cpu()[0]), A, n, x, 1, 1.0, want, 1)
        assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
    finally:
        for key in k.tuning_keys():
            k.set_tuning(key, 0)


def test_runs_on_a_side_stream_with_explicit_workspace():
    k = kmv()
    n = 2000
    A = wl.matrix("d", n, n, seed=17, device=DEV)
    x = wl.vector("d", n, seed=17, device=DEV)
    y0 = wl.vector("d", n, seed=17, which=2, device=DEV)
    ref = y0.clone()
    k.dgemv("N", n, n, 1.0, A, n, x, 1, 1.0, ref, 1)
    ws = torch.empty(k.gemv_workspace_bytes("d", "N", n, n), dtype=torch.uint8, device=DEV)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    y = y0.clone()
    torch.cuda.synchronize()
    k.dgemv("N", n, n, 1.0, A, n, x, 1, 1.0, y, 1, workspace=ws, stream=st)
    st.synchronize()
    assert torch.equal(y, ref)
    # a workspace that is too small is refused before anything is enqueued
    k.set_tuning("gemv_n_splits", 8)
    try:
        rc = k.dgemv("N", n, n, 1.0, A, n, x, 1, 1.0, y, 1, workspace=ws[:512], check=False)
    finally:
        k.set_tuning("gemv_n_splits", 0)
    assert rc == k.ERR_WORKSPACE and torch.equal(y, ref)


def test_prepared_calls_match_plain_calls():
    """a prepared call (arguments marshalled once) gives the bits of the plain wrapper"""
    k = kmv()
    n = 1500
    A = wl.matrix("d", n, n, seed=21, device=DEV)
    x = wl.vector("d", n, seed=21, device=DEV)
    y0 = wl.vector("d", n, seed=21, which=2, device=DEV)
    for make, plain in ((lambda y: k.prepare_gemv("d", "N", n, n, 0.7, A, n, x, 1, 0.3, y, 1),
                         lambda y: k.dgemv("N", n, n, 0.7, A, n, x, 1, 0.3, y, 1)),
                        (lambda y: k.prepare_gemv("d", "T", n, n, 0.7, A, n, x, 1, 0.3, y, 1),
                         lambda y: k.dgemv("T", n, n, 0.7, A, n, x, 1, 0.3, y, 1)),
                        (lambda y: k.prepare_symv("d", "U", n, 0.7, A, n, x, 1, 0.3, y, 1),
                         lambda y: k.dsymv("U", n, 0.7, A, n, x, 1, 0.3, y, 1))):
        ref = y0.clone()
        plain(ref)
        y = y0.clone()
        call = make(y)
        call()
        torch.cuda.synchronize()
        assert torch.equal(y, ref)
        y.copy_(y0)
        call()                       # a prepared call can be repeated
        torch.cuda.synchronize()
        assert torch.equal(y, ref)


@pytest.mark.parametrize("prec", PRECS)
def test_gemv_short_matrix_kernels(prec):
    """matrices of a few row tiles: the kernels in which waves split columns, forced on
    (2) and off (1), with sub-block offsets that move the tile grid, against the oracle"""
    k = kmv()
    alpha, beta = scalars(prec, 0.7, 0.3)
    try:
        for mode in (1, 2):
            k.set_tuning("gemv_short", mode)
            for m, n, off, lda in ((100, 9000, 0, None), (200, 3000, 3, 256), (64, 70000, 0, 64), (500, 5000, 1, 512),
                                   (1000, 4100, 17, 1024), (3, 1000, 0, None), (130, 37, 5, 144)):
                for trans in "NTC":
                    _, err, _ = gemv_case(prec, trans, m, n, alpha, beta, lda=lda, row_off=off, col_off=off, seed=31)
                    check(prec, err, f"gemv_short={mode} {prec}gemv {trans} {m}x{n} off={off}")
    finally:
        k.set_tuning("gemv_short", 0)


@pytest.mark.parametrize("prec", PRECS)
def test_random_shapes_against_oracle(prec):
    """seeded random shapes, leading dimensions, offsets, increments and scalars for every
    routine: whatever combination of kernels and edge cases they hit must match the oracle
    (KMV_FUZZ_CASES / KMV_FUZZ_SEED in the environment lengthen or reseed the series)"""
    rng = np.random.default_rng({"s": 11, "d": 12, "c": 13, "z": 14}[prec] + 100 * int(os.environ.get("KMV_FUZZ_SEED", "0")))
    incs = (1, 1, 1, 2, -1, 3, -2)
    for case in range(int(os.environ.get("KMV_FUZZ_CASES", "24"))):
        m = int(rng.choice([1, 7, 64, 300, 1000, 2500]) + rng.integers(0, 130))
        n = int(rng.choice([1, 5, 96, 500, 1500, 3000]) + rng.integers(0, 130))
        off = int(rng.choice([0, 0, 1, 3, 16, 33]))
        pad = int(rng.choice([0, 1, 7, 32]))
        alpha, beta = scalars(prec, float(rng.choice([1.0, -0.5, 0.7])), float(rng.choice([0.0, 1.0, 0.3])))
        incx, incy = int(rng.choice(incs)), int(rng.choice(incs))
        trans = "NTC"[case % 3]
        _, err, _ = gemv_case(prec, trans, m, n, alpha, beta, lda=m + off + pad, row_off=off, col_off=off, incx=incx,
                              incy=incy, seed=100 + case)
        check(prec, err, f"case {case}: {prec}gemv {trans} {m}x{n} off={off} pad={pad} inc={incx},{incy}")
        uplo = "LU"[case % 2]
        beta_s = beta if case % 4 else 0.0
        _, err, _ = symv_case(prec, uplo, n, alpha, beta_s, lda=n + off + pad, off=off, incx=incx, incy=incy,
                              seed=200 + case, nan_imag_diag=True)
        check(prec, err, f"case {case}: symv/hemv {prec} {uplo} n={n} off={off} pad={pad} inc={incx},{incy}")


@pytest.mark.parametrize("prec", PRECS)
def test_mid_size_shapes_against_oracle(prec):
    """seeded shapes of 4000 ... 9000 rows and columns with odd leading dimensions and offsets: the sizes at which the
    transposed kernel changes between its forms (row splits, one workgroup per compute unit, banded loop) and the
    non-transposed one between its split rules; sampled outputs against the oracle"""
    rng = np.random.default_rng({"s": 31, "d": 32, "c": 33, "z": 34}[prec])
    for case in range(10):
        m = int(rng.integers(4000, 9000))
        n = int(rng.integers(4000, 9000))
        off = int(rng.choice([0, 0, 1, 16, 33]))
        pad = int(rng.choice([0, 0, 5, 32, 96]))
        if case % 3 == 0:       # a leading dimension on the 128-byte grid
            pad += (-(m + off + pad)) % 32
        trans = ("N", "T", "C")[case % 3] if prec in "cz" else ("N", "T")[case % 2]
        alpha, beta = scalars(prec, 0.7, 0.3)
        leny = m if trans == "N" else n
        _, err, _ = gemv_case(prec, trans, m, n, alpha, beta, lda=m + off + pad, row_off=off, col_off=off % 7, seed=300 + case,
                              sample=wl.sample_indices(leny, 64, case).numpy())
        check(prec, err, f"case {case}: {prec}gemv {trans} {m}x{n} off={off} pad={pad}")


@pytest.mark.parametrize("n", [2, 2048, 1_000_002, 40_000_000])
def test_stream_probe_moves_what_it_says(n):
    """the calibration kernels (STREAM read / copy / triad, and the read pass with few workgroups) really read and write
    every element: the per-workgroup sums add up to the array's sum, the copy and the triad equal their definitions"""
    k = kmv()
    g = torch.Generator(device=DEV).manual_seed(n)
    a = torch.randint(-8, 9, (n,), generator=g, device=DEV).to(torch.float64)     # sums are exact in any order
    b = torch.full((n,), float("nan"), dtype=torch.float64, device=DEV)
    c = torch.full((n,), float("nan"), dtype=torch.float64, device=DEV)
    want = float(a.sum().item())
    for kind, wgs in ((0, 0), (3, 0), (3, 7), (3, 8192)):
        sink = torch.zeros(8192, dtype=torch.float64, device=DEV)
        k.set_tuning("wg_target", wgs)
        try:
            k.stream_probe(kind, n, a, None, None, sink)
        finally:
            k.set_tuning("wg_target", 0)
        torch.cuda.synchronize()
        assert float(sink.sum().item()) == want, (kind, wgs)
    k.stream_probe(1, n, a, b, None, None)
    torch.cuda.synchronize()
    assert torch.equal(b, a)
    k.stream_probe(2, n, a, b, c, None)
    torch.cuda.synchronize()
    assert torch.equal(c, a + 3.0 * b)


def test_calls_can_be_captured_in_a_graph():
    """the entry points only enqueue kernels (no allocation, no memset, no host
    synchronisation), so a sequence of calls can be recorded once and replayed;
    every replay, with new vector contents and eager work in between, must give
    the bits of the eager calls"""
    k = kmv()
    n = 1800
    A = wl.matrix("d", n, n, seed=41, device=DEV)
    x = wl.vector("d", n, seed=41, device=DEV)
    y1, y2, y3, y4, y5, y6, y7 = (torch.zeros(n, dtype=torch.float64, device=DEV) for _ in range(7))
    ws = torch.empty(max(k.gemv_workspace_bytes("d", "N", n, n), k.symv_workspace_bytes("d", "L", n)),
                     dtype=torch.uint8, device=DEV)
    dev_alpha = torch.zeros(1, dtype=torch.float64, device=DEV)
    dev_beta = torch.zeros(1, dtype=torch.float64, device=DEV)
    nb, bn = 9, 200                              # a batch of nine 200 x 200 blocks inside A's buffer
    idx = torch.arange(nb, dtype=torch.int64, device=DEV)
    Ap, xp, yp = A.data_ptr() + idx * (bn * bn * 8), x.data_ptr() + idx * (bn * 8), y7.data_ptr() + idx * (bn * 8)

    def run():
        k.dgemv("N", n, n, 0.7, A, n, x, 1, 0.0, y1, 1, workspace=ws)
        k.dgemv("T", n, n, 1.0, A, n, y1, 1, 0.0, y2, 1, workspace=ws)
        k.dsymv("L", n, -0.5, A, n, y2, 1, 0.0, y3, 1, workspace=ws)
        # the other families: offsets, scalars written by a kernel of the same capture, a strided batch
        k.dgemv_offset("N", n, n, 1.0, A, n, x, 1, 0.0, y4, 1, 17, 5, workspace=ws)
        dev_alpha.copy_(y1[:1])                  # device-side producer of alpha
        k.dsymv_devscalars("U", n, dev_alpha, A, n, x, 1, dev_beta, y5, 1, workspace=ws)
        k.dgemv_strided_batched("T", bn, bn, 1.0, A, bn, bn * bn, x, 1, bn, 0.0, y6, 1, bn, nb)
        k.dsymv_batched("L", bn, 1.0, Ap, bn, xp, 1, 0.0, yp, 1, nb)       # the same members through pointer arrays

    run()                                   # warm up outside the capture (occupancy queries, module load)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for rep in range(4):
        x.copy_(wl.vector("d", n, seed=50 + rep, device=DEV))
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (y1, y2, y3, y4, y5, y6, y7)]
        run()
        torch.cuda.synchronize()
        assert float(y5.abs().sum()) > 0 and float(y6.abs().sum()) > 0 and float(y7.abs().sum()) > 0
        for a_, b_ in zip(got, (y1, y2, y3, y4, y5, y6, y7)):
            assert torch.equal(a_, b_), f"replay {rep} differs from the eager calls"


@pytest.mark.parametrize("prec", PRECS)
def test_shrinking_trailing_blocks(prec):
    """the trailing blocks A[o:, o:] of one parent for consecutive offsets o, as the panel
    loop of a blocked reduction visits them: every misalignment of the block's first column
    (0..127 bytes), with the rest of the parent set to NaN, for GEMV N/T and SYMV/HEMV L/U"""
    alpha, beta = scalars(prec, -1.0, 1.0)
    N, lda = 900, 1024           # lda*sizeof(T) is a multiple of 128: one shift for all columns
    per_line = 128 // {"s": 4, "d": 8, "c": 8, "z": 16}[prec]
    offsets = list(range(0, per_line + 2)) + [per_line * 3 + 1, 333]
    for o in offsets:
        n = N - o
        for trans in "NT":
            _, err, _ = gemv_case(prec, trans, n, n - 7, alpha, beta, lda=lda, row_off=o, col_off=o, seed=70 + o % 5)
            check(prec, err, f"{prec}gemv {trans} trailing block at {o}")
        for variant in (0, 2):       # default (the small-matrix kernel at this size) and the balanced kernel
            kmv().set_tuning("symv_variant", variant)
            try:
                for uplo in "LU":
                    _, err, _ = symv_case(prec, uplo, n, alpha, beta, lda=lda, off=o, seed=80 + o % 5)
                    check(prec, err, f"symv/hemv {prec} {uplo} trailing block at {o}, variant {variant}")
            finally:
                kmv().set_tuning("symv_variant", 0)


@pytest.mark.parametrize("prec", PRECS)
def test_workspace_bound_is_enough_and_respected(prec):
    """A workspace of exactly the queried size serves every pointer alignment, increment and tuning value:
    the call is accepted, the bytes behind the workspace keep their pattern, and the result has the bits of
    the call that lets the binding provide the workspace."""
    k = kmv()
    alpha, beta = scalars(prec, 0.9, 0.2)
    guard = 4096
    tunings = [{}, {"gemv_n_splits": 256, "gemv_t_splits": 256}, {"gemv_n_splits": 1, "gemv_t_splits": 1},
               {"gemv_n_row_tiles": 4, "wg_target": 1 << 20}, {"gemv_short": 1}, {"gemv_short": 2},
               {"symv_variant": 2, "symv_tiles_per_wave": 1, "wg_target": 800},
               {"symv_variant": 2, "wg_target": 1 << 20, "symv_unit_tiles": 1},
               {"symv_variant": 2, "wg_target": 1, "symv_unit_tiles": 2, "symv_tiles_per_wave": 2},
               {"symv_variant": 3}]
    try:
        for tune in tunings:
            for key, v in tune.items():
                k.set_tuning(key, v)
            for m, n, off, incx in ((2500, 1900, 0, 1), (1900, 2500, 1, -2), (100, 7000, 3, 3), (6000, 130, 2, 1)):
                lda = m + off + 5
                parent = wl.matrix(prec, m + off, n, lda, seed=61, device=DEV)
                A = parent[:, off:]
                for trans in "NT":
                    lenx, leny = (n, m) if trans == "N" else (m, n)
                    x = wl.vector(prec, lenx, incx, seed=61, which=1, device=DEV)
                    y0 = wl.vector(prec, leny, 1, seed=61, which=2, device=DEV)
                    nbytes = k.gemv_workspace_bytes(prec, trans, m, n)
                    ws = torch.full((nbytes + guard,), 0xA5, dtype=torch.uint8, device=DEV)
                    want, got = y0.clone(), y0.clone()
                    k.GEMV[prec](trans, m, n, alpha, A, lda, x, incx, beta, want, 1)
                    rc = k.GEMV[prec](trans, m, n, alpha, A, lda, x, incx, beta, got, 1, workspace=ws[:nbytes], check=False)
                    assert rc == 0, (tune, trans, m, n, rc)
                    torch.cuda.synchronize()
                    assert bool((ws[nbytes:] == 0xA5).all()), ("wrote behind the workspace", tune, trans, m, n)
                    assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
            for n, off, incx in ((2300, 0, 1), (3001, 1, 2), (700, 3, -1), (5200, 2, 1)):
                lda = n + off + 3
                parent = wl.matrix(prec, n + off, n, lda, seed=62, device=DEV)
                A = parent[:, off:]
                for uplo in "LU":
                    x = wl.vector(prec, n, incx, seed=62, which=1, device=DEV)
                    y0 = wl.vector(prec, n, 1, seed=62, which=2, device=DEV)
                    nbytes = k.symv_workspace_bytes(prec, uplo, n)
                    ws = torch.full((nbytes + guard,), 0xA5, dtype=torch.uint8, device=DEV)
                    want, got = y0.clone(), y0.clone()
                    k.SYMV[prec](uplo, n, alpha, A, lda, x, incx, beta, want, 1)
                    rc = k.SYMV[prec](uplo, n, alpha, A, lda, x, incx, beta, got, 1, workspace=ws[:nbytes], check=False)
                    assert rc == 0, (tune, uplo, n, rc)
                    torch.cuda.synchronize()
                    assert bool((ws[nbytes:] == 0xA5).all()), ("wrote behind the workspace", tune, uplo, n)
                    assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
            for key in tune:
                k.set_tuning(key, 0)
    finally:
        for key in k.tuning_keys():
            k.set_tuning(key, 0)
