"""Parity at the full benchmark sizes, in the launch configuration the benchmark
times (default tuning): the oracle computes a sample of output elements one by
one (both ends, tile-boundary neighbourhoods, seeded random picks) and every
sampled element must meet the normwise tolerance and the componentwise bound.
Inputs follow the benchmark configurations: the size sweep (lda = n, U[-1,1]),
the symmetric sweep with the unreferenced triangle set to NaN, sub-blocks of a
20000 x 20000 fp64 parent at unaligned offsets, and the largest shapes with
lda = n + 32, N(0,1) entries and a strided x."""
import gc

import numpy as np
import pytest
import torch

from paper_1410_1726_amd import workloads as wl

from gpu_util import DEV, check, gemv_case, symv_case

pytestmark = pytest.mark.gpu

NSAMPLE = 48


def samples(n, seed):
    return wl.sample_indices(n, NSAMPLE, seed).numpy()


def free():
    gc.collect()
    torch.cuda.empty_cache()


# ---- size sweep: SGEMV / DGEMV, N and T, lda = n, alpha = beta = 1 ------------
@pytest.mark.parametrize("prec", "sd")
@pytest.mark.parametrize("n", [16384, 17001, 20001, 32768])     # 17001, 20001: leading dimension off the 128-byte grid
def test_gemv_sweep_sizes(prec, n):
    parent = wl.matrix(prec, n, n, n, seed=0, device=DEV)
    for trans in "NT":
        _, err, _ = gemv_case(prec, trans, n, n, 1.0, 1.0, lda=n, seed=0, parent=parent, sample=samples(n, 1),
                              poison_outside=False)
        check(prec, err, f"{prec}gemv {trans} n={n}")
    del parent
    free()


# ---- symmetric sweep: DSYMV / ZHEMV, L and U, other triangle NaN, beta = 0 -----
@pytest.mark.parametrize("prec", "dz")
def test_symv_sweep_largest(prec):
    n = 32768
    host = None
    for uplo in "LU":
        parent = wl.matrix(prec, n, n, n, seed=0, device=DEV)      # regenerated: the run poisons it
        _, err, ex = symv_case(prec, uplo, n, 1.0, 0.0, lda=n, seed=0, parent=parent, parent_host=host,
                               sample=samples(n, 2), nan_imag_diag=True)
        host = ex["parent_host"]
        check(prec, err, f"symv/hemv {prec} {uplo} n={n}")
        del parent
        free()


# ---- EVERY output element at the largest sweep size, in the launch configuration the benchmark times: a
# mistake confined to one workgroup's share of the work (one row chunk, one 16-column panel) cannot hide
# between samples
def test_gemv_every_output_at_32768():
    n = 32768
    parent = wl.matrix("d", n, n, n, seed=0, device=DEV)
    for trans in "NT":
        _, err, _ = gemv_case("d", trans, n, n, 1.0, 1.0, lda=n, seed=0, parent=parent, poison_outside=False)
        check("d", err, f"dgemv {trans} n={n}, all outputs")
    del parent
    free()


@pytest.mark.parametrize("prec", "dz")
def test_symv_every_output_at_32768(prec):
    n = 32768
    host = None
    for uplo in "LU":
        parent = wl.matrix(prec, n, n, n, seed=0, device=DEV)      # regenerated: the run poisons it
        _, err, ex = symv_case(prec, uplo, n, 1.0, 0.0, lda=n, seed=0, parent=parent, parent_host=host, nan_imag_diag=True)
        host = ex["parent_host"]
        check(prec, err, f"symv/hemv {prec} {uplo} n={n}, all outputs")
        del parent
        free()
    del host
    free()


# ---- sub-blocks of a 20000 x 20000 fp64 parent, alpha = -1, beta = 1 -----------
PARENT_N = 20000
_parent_host = {}


def parent20k():
    p = wl.matrix("d", PARENT_N, PARENT_N, PARENT_N, seed=4, device=DEV)
    if "h" not in _parent_host:
        _parent_host["h"] = p.cpu().numpy().reshape(-1)
    return p, _parent_host["h"]


@pytest.mark.parametrize("off", [1, 17, 63, 1000])
def test_subblocks_of_20000_parent(off):
    for n in (2048, 8192, 19000 - off):
        for trans in "NT":
            parent, _ = parent20k()
            _, err, _ = gemv_case("d", trans, n, n, -1.0, 1.0, lda=PARENT_N, row_off=off, col_off=off, seed=4,
                                  parent=parent, sample=samples(n, 3))
            check("d", err, f"dgemv {trans} block n={n} at offset {off}")
            del parent
        parent, host = parent20k()
        _, err, _ = symv_case("d", "L", n, -1.0, 1.0, lda=PARENT_N, off=off, seed=4, parent=parent,
                              parent_host=host, sample=samples(n, 3))
        check("d", err, f"dsymv L block n={n} at offset {off}")
        del parent
        free()


def test_subblock_every_output():
    """the largest block at offset 17 of the 20000 x 20000 parent, every output element, and the oracle is handed
    the parent as the device sees it: NaN outside the block (and in the unreferenced triangle for DSYMV)"""
    off, n = 17, 19000 - 17
    for trans in "NT":
        parent, _ = parent20k()
        _, err, _ = gemv_case("d", trans, n, n, -1.0, 1.0, lda=PARENT_N, row_off=off, col_off=off, seed=4, parent=parent)
        check("d", err, f"dgemv {trans} block n={n} at offset {off}, all outputs")
        del parent
        free()
    parent, _ = parent20k()
    _, err, _ = symv_case("d", "L", n, -1.0, 1.0, lda=PARENT_N, off=off, seed=4, parent=parent, oracle_sees_poison=True)
    check("d", err, f"dsymv L block n={n} at offset {off}, all outputs")
    del parent
    free()


@pytest.mark.parametrize("prec", "sc")
def test_large_subblocks_on_the_grid(prec):
    """blocks of more than 256 MB at (1, 1) and (33, 5) of a parent whose leading dimension is a multiple of 128 bytes,
    with ragged row counts: the planner's large-matrix forms with a shifted row grid and cut first and last tiles
    (4-byte elements leave the one-workgroup-per-compute-unit form of GEMV-N there), NaN around the block"""
    n, lda = (9000, 9056) if prec == "s" else (6100, 6144)
    for row_off, col_off in ((1, 1), (33, 5)):
        m = lda - row_off - 7
        for trans in ("N", "C" if prec == "c" else "T"):
            _, err, _ = gemv_case(prec, trans, m, n, 0.7, 0.3, lda=lda, row_off=row_off, col_off=col_off, seed=23,
                                  sample=samples(m if trans == "N" else n, 3))
            check(prec, err, f"{prec}gemv {trans} {m}x{n} block at ({row_off}, {col_off}), lda={lda}")
        free()


def test_release_parent_host_copy():
    _parent_host.clear()
    free()


# ---- largest shapes: lda = n + 32, N(0,1), alpha 0.7, beta 0.3, incx 1 and 2 ---
@pytest.mark.parametrize("prec", "sdcz")
def test_largest_shapes(prec):
    n = 49152 if prec in "sc" else 40960
    lda = n + 32
    parent = wl.matrix(prec, n, n, lda, dist="normal", seed=5, device=DEV, pad_nan=True)
    host = parent.cpu().numpy().reshape(-1)
    for incx in (1, 2):
        for trans in "NT":
            _, err, _ = gemv_case(prec, trans, n, n, 0.7, 0.3, lda=lda, incx=incx, dist="normal", seed=5,
                                  parent=parent, sample=samples(n, 4), poison_outside=False)
            check(prec, err, f"{prec}gemv {trans} n={n} incx={incx}")
        for uplo in "LU":
            _, err, _ = symv_case(prec, uplo, n, 0.7, 0.3, lda=lda, incx=incx, dist="normal", seed=5,
                                  parent=parent, parent_host=host, sample=samples(n, 4), poison=False)
            check(prec, err, f"symv/hemv {prec} {uplo} n={n} incx={incx}")
            if prec in "cz" and incx == 1:
                _, err, _ = symv_case(prec, uplo, n, 0.7, 0.3, lda=lda, dist="normal", seed=5, parent=parent,
                                      parent_host=host, sample=samples(n, 4), poison=False, complex_symmetric=True)
                check(prec, err, f"complex symmetric symv {prec} {uplo} n={n}")
    del parent, host
    free()


# ---- panels of the rectangular benchmark workload (tall-skinny, short-wide) ------
@pytest.mark.parametrize("prec", "ds")
def test_rectangular_panels(prec):
    for m, n in ((65536, 512), (16384, 64), (128, 65536), (512, 65536), (4096, 16384)):
        for trans in "NT":
            leny = m if trans == "N" else n
            _, err, _ = gemv_case(prec, trans, m, n, 1.0, 1.0, lda=m, seed=6, sample=samples(leny, 6),
                                  poison_outside=False)
            check(prec, err, f"{prec}gemv {trans} {m}x{n}")
        free()


# ---- a large size whose columns are not 16-byte aligned against each other (lda = n odd): unaligned 16-byte
# loads and a ragged last row tile in every column
def test_symv_drifting_alignment_large():
    from paper_1410_1726_amd import binding as k
    n = 17001
    assert k.symv_kernel_variant("d", "L", n, 256, n) == 2
    for uplo in "LU":
        _, err, _ = symv_case("d", uplo, n, 1.0, 0.0, lda=n, seed=8, sample=samples(n, 8))
        check("d", err, f"dsymv {uplo} n={n}")
        free()
