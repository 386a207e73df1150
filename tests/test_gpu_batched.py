"""Strided-batched GEMV / SYMV / HEMV against the oracle, member by member: shapes around the tile sizes,
member strides that keep and that break the 128-byte alignment of the members, shared inputs (stride 0),
strided and reversed y, NaN canaries between the outputs, the other triangle NaN, and a batch longer than one
launch can hold."""
import numpy as np
import pytest
import torch

import oracle
from paper_1410_1726_amd import workloads as wl

from gpu_util import DEV, check, errors, kmv, logical

pytestmark = pytest.mark.gpu
PRECS = "sdcz"
NAN = float("nan")


def scal(prec, a, b):
    return (complex(a, 0.25), complex(b, -0.5)) if prec in "cz" else (a, b)


def rand(prec, count, seed):
    t = torch.empty(count, dtype=wl.TORCH_DTYPES[prec], device=DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return wl.fill_random(t, "uniform", g)


def y_buffer(prec, leny, incy, stridey, batch, seed):
    """batch strided vectors, NaN in every position that is not an element of one of them"""
    y = torch.full((max(batch * stridey, 1),), NAN, dtype=wl.TORCH_DTYPES[prec], device=DEV)
    vals = rand(prec, batch * leny, seed).view(batch, leny)
    for b in range(batch):
        y[b * stridey: b * stridey + 1 + (leny - 1) * abs(incy): abs(incy)] = vals[b]
    return y


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("trans", "NTC")
@pytest.mark.parametrize("tiny_rows", [0, 1, 1024])     # the library's choice, never, up to a whole row tile
def test_gemv_strided_batched(prec, trans, tiny_rows):
    k = kmv()
    k.set_tuning("gemv_tiny_rows", tiny_rows)
    try:
        _gemv_batched_cases(k, prec, trans)
    finally:
        k.set_tuning("gemv_tiny_rows", 0)


def _gemv_batched_cases(k, prec, trans, cases=None):
    alpha, beta = scal(prec, 0.7, -0.3)
    # up to one row tile (256 / 128 / 128 / 64 rows): one wave per member with 8, 16, 32 or 64 lanes per column
    cases = cases or [(1, 1, 1, 0, 1), (2, 9, 3, 0, 1), (3, 3, 2, 1, 1), (4, 1, 5, 0, 1), (5, 17, 2, 2, -1), (7, 5, 3, 1, 1),
             (8, 8, 9, 0, 1), (9, 40, 3, 1, 1), (16, 16, 6, 0, 1), (17, 3, 2, 0, 2), (31, 33, 3, 3, 1), (32, 100, 5, 0, 1),
             (33, 7, 2, 1, 1), (63, 64, 3, 0, 1), (64, 64, 4, 0, 2), (65, 200, 7, 16, 1), (100, 300, 5, 3, -1),
             (127, 50, 2, 0, 1), (128, 128, 3, 0, 1), (129, 31, 2, 1, 1), (255, 20, 3, 0, 1), (256, 256, 2, 0, 1),
             (257, 9, 2, 0, 1), (513, 129, 17, 0, 1), (1000, 40, 2, 8, 1), (300, 700, 3, 16, -2)]
    for m, n, batch, pad, incy in cases:
        lda = m + (pad % 5)
        strideA = lda * n + pad                       # pad = 0 or 16: members equally aligned; else not
        lenx, leny = (n, m) if trans == "N" else (m, n)
        stridex = 0 if batch % 2 else lenx + 3        # odd batches share one x
        exty = 1 + (leny - 1) * abs(incy)
        stridey = exty + 2
        A = rand(prec, (batch - 1) * strideA + lda * n, 11 + m)
        x = rand(prec, (batch - 1) * stridex + lenx, 12 + m)
        y0 = y_buffer(prec, leny, incy, stridey, batch, 13 + m)
        y = y0.clone()
        k.GEMV_STRIDED_BATCHED[prec](trans, m, n, alpha, A, lda, strideA, x, 1, stridex, beta, y, incy, stridey, batch)
        torch.cuda.synchronize()
        Ah, xh, yh, y0h = A.cpu().numpy(), x.cpu().numpy(), y.cpu().numpy(), y0.cpu().numpy()
        is_out = np.zeros(yh.size, dtype=bool)
        for b in range(batch):
            sl = slice(b * stridey, b * stridey + exty)
            is_out[b * stridey: b * stridey + exty: abs(incy)] = True
            kw = dict(lda=lda, incy=incy)
            want = oracle.gemv(prec, trans, m, n, alpha, Ah[b * strideA:], xh[b * stridex: b * stridex + lenx], beta,
                               y0h[sl], mode=oracle.MODE_X, **kw)
            den = oracle.gemv(prec, trans, m, n, alpha, Ah[b * strideA:], xh[b * stridex: b * stridex + lenx], beta,
                              y0h[sl], mode=oracle.MODE_ABS, **kw)
            err = errors(prec, logical(yh[sl], leny, incy), logical(want, leny, incy), logical(den, leny, incy), lenx)
            check(prec, err, f"{prec}gemv_strided_batched {trans} {m}x{n} member {b}/{batch}")
        assert np.array_equal(yh[~is_out].view(np.uint8), y0h[~is_out].view(np.uint8)), "wrote between outputs"


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("uplo", "LU")
def test_symv_strided_batched(prec, uplo):
    _symv_batched_case(prec, uplo, False)


@pytest.mark.parametrize("prec", "cz")
@pytest.mark.parametrize("uplo", "LU")
def test_complex_symmetric_strided_batched(prec, uplo):
    """csymv / zsymv batches: no conjugation, the diagonal as stored"""
    _symv_batched_case(prec, uplo, True)


def _symv_batched_case(prec, uplo, csym, cases=None):
    k = kmv()
    alpha, beta = scal(prec, -1.1, 0.4)
    for n, batch, pad, incy in cases or [(1, 1, 0, 1), (2, 3, 0, 1), (3, 2, 1, 1), (4, 2, 0, -1), (5, 2, 2, 1), (8, 4, 0, 1), (9, 3, 1, -1), (16, 5, 0, 1), (17, 3, 1, 1), (31, 2, 0, 1), (32, 6, 3, -1),
                                 (33, 2, 0, 1), (63, 5, 16, 2), (64, 2, 0, 1), (65, 3, 2, 1), (100, 3, 1, 1), (127, 2, 0, 1), (128, 9, 0, 1),
                                 (129, 4, 0, -2), (200, 6, 3, 1), (257, 2, 5, 1), (511, 2, 0, 1), (512, 3, 0, 1),
                                 (513, 2, 1, 1), (640, 2, 0, 1), (777, 2, 0, 1), (1024, 2, 0, 1), (1100, 3, 0, 1)]:   # small members: one workgroup each; beyond: small-matrix kernel
        lda = n + (pad % 4)
        strideA = lda * n + pad
        stridex = 0 if batch % 2 else n + 1
        exty = 1 + (n - 1) * abs(incy)
        stridey = exty + 1
        A = rand(prec, (batch - 1) * strideA + lda * n, 21 + n)
        host = A.cpu().numpy()                         # the oracle reads the stored triangle only
        for b in range(batch):
            blk = A[b * strideA: b * strideA + lda * n].view(n, lda)
            wl.poison_triangle(blk, n, uplo, real_diag=False)
            if prec in "cz" and not csym:
                d = torch.arange(n, device=DEV)
                torch.view_as_real(blk)[d, d, 1] = NAN      # HEMV ignores the diagonal's imaginary part
        x = rand(prec, (batch - 1) * stridex + n, 22 + n)
        y0 = y_buffer(prec, n, incy, stridey, batch, 23 + n)
        y = y0.clone()
        (k.CSYMV_STRIDED_BATCHED if csym else k.SYMV_STRIDED_BATCHED)[prec](
            uplo, n, alpha, A, lda, strideA, x, 1, stridex, beta, y, incy, stridey, batch)
        torch.cuda.synchronize()
        xh, yh, y0h = x.cpu().numpy(), y.cpu().numpy(), y0.cpu().numpy()
        is_out = np.zeros(yh.size, dtype=bool)
        for b in range(batch):
            sl = slice(b * stridey, b * stridey + exty)
            is_out[b * stridey: b * stridey + exty: abs(incy)] = True
            args = (prec, uplo, n, alpha, host[b * strideA:], xh[b * stridex: b * stridex + n], beta, y0h[sl])
            want = oracle.symv(*args, lda=lda, incy=incy, mode=oracle.MODE_X, complex_symmetric=csym)
            den = oracle.symv(*args, lda=lda, incy=incy, mode=oracle.MODE_ABS, complex_symmetric=csym)
            err = errors(prec, logical(yh[sl], n, incy), logical(want, n, incy), logical(den, n, incy), n)
            check(prec, err, f"symv/hemv_strided_batched {prec} {uplo} n={n} member {b}/{batch}")
        assert np.array_equal(yh[~is_out].view(np.uint8), y0h[~is_out].view(np.uint8)), "wrote between outputs"


def test_batch_longer_than_one_launch_and_special_scalars():
    k = kmv()
    m, n, batch = 4, 3, 70000                           # 65535 members per launch: two launches
    A = rand("d", batch * m * n, 1)
    x = rand("d", batch * n, 2)
    y0 = rand("d", batch * m, 3)
    y = y0.clone()
    k.dgemv_strided_batched("N", m, n, 2.0, A, m, m * n, x, 1, n, -1.0, y, 1, m, batch)
    torch.cuda.synchronize()
    Ah = A.cpu().numpy().reshape(batch, n, m)           # member, column, row
    want = 2.0 * np.einsum("bji,bj->bi", Ah, x.cpu().numpy().reshape(batch, n)) - y0.cpu().numpy().reshape(batch, m)
    got = y.cpu().numpy().reshape(batch, m)
    assert np.max(np.abs(got - want)) <= 1e-14
    for b in (0, 65534, 65535, 65536, batch - 1):       # around the launch boundary, through the oracle
        w = oracle.gemv("d", "N", m, n, 2.0, A.cpu().numpy()[b * m * n:], x.cpu().numpy()[b * n: b * n + n], -1.0,
                        y0.cpu().numpy()[b * m: b * m + m], lda=m, mode=oracle.MODE_X)
        assert np.max(np.abs(got[b] - w)) <= 1e-14
    # alpha = 0: y <- beta*y, A and x (NaN here) are not referenced; beta = 0 with NaN in y
    y = y0.clone()
    k.dgemv_strided_batched("T", n, m, 0.0, torch.full_like(A, NAN), n, m * n, torch.full_like(x, NAN), 1, n, 3.0, y, 1, m, batch)
    assert torch.equal(y, 3.0 * y0)
    y = torch.full_like(y0, NAN)
    k.dgemv_strided_batched("N", m, n, 2.0, A, m, m * n, x, 1, n, 0.0, y, 1, m, batch)
    torch.cuda.synchronize()
    want0 = 2.0 * np.einsum("bji,bj->bi", Ah, x.cpu().numpy().reshape(batch, n))
    assert np.max(np.abs(y.cpu().numpy().reshape(batch, m) - want0)) <= 1e-14
    # batch = 0 and alpha = 0, beta = 1: nothing happens
    y = y0.clone()
    k.dgemv_strided_batched("N", m, n, 2.0, A, m, m * n, x, 1, n, 0.5, y, 1, m, 0)
    k.dsymv_strided_batched("L", 3, 0.0, A, 3, 9, x, 1, 3, 1.0, y, 1, 3, 100)
    assert torch.equal(y, y0)


# ------------------------------------------------------------ pointer-array batches ----
def _member_offsets(batch, extent, rng):
    """start offsets of `batch` members of `extent` elements in one buffer, in shuffled order and with gaps
    of 0..5 elements, so that the members are neither equally spaced nor equally aligned"""
    gaps = rng.integers(0, 6, size=batch)
    starts = np.concatenate(([0], np.cumsum(extent + gaps)[:-1])) + 1      # +1: the first one is unaligned too
    order = rng.permutation(batch)
    return [int(starts[i]) for i in order], int(starts[-1] + extent + 8)


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("trans", "NTC")
def test_gemv_pointer_array_batched(prec, trans):
    k = kmv()
    alpha, beta = scal(prec, 0.7, -0.3)
    rng = np.random.default_rng(5)
    for m, n, batch, pad, incy in [(1, 1, 1, 0, 1), (3, 9, 4, 0, 1), (8, 8, 9, 1, -1), (31, 33, 3, 3, 1), (64, 64, 4, 0, 2),
                                   (100, 300, 5, 3, -1), (129, 31, 2, 1, 1), (256, 256, 3, 0, 1), (257, 9, 2, 0, 1),
                                   (513, 129, 7, 0, 1), (1000, 40, 2, 8, 1), (300, 700, 3, 16, -2)]:
        lda = m + (pad % 5)
        lenx, leny = (n, m) if trans == "N" else (m, n)
        exty = 1 + (leny - 1) * abs(incy)
        offA, sizeA = _member_offsets(batch, lda * n, rng)
        offy, sizey = _member_offsets(batch, exty, rng)
        A = rand(prec, sizeA, 31 + m)
        x = rand(prec, lenx * batch + 1, 32 + m)
        y0 = torch.full((sizey,), NAN, dtype=wl.TORCH_DTYPES[prec], device=DEV)
        vals = rand(prec, batch * leny, 33 + m).view(batch, leny)
        for b in range(batch):
            y0[offy[b]: offy[b] + exty: abs(incy)] = vals[b]
        y = y0.clone()
        offx = [0 if b % 2 else 1 + b * lenx - lenx * (b > 0) for b in range(batch)]        # odd members share one x
        offx = [min(o, x.numel() - lenx) for o in offx]
        Ap = k.pointer_array([A[o:] for o in offA])
        xp = k.pointer_array([x[o:] for o in offx])
        yp = k.pointer_array([y[o:] for o in offy])
        k.GEMV_BATCHED[prec](trans, m, n, alpha, Ap, lda, xp, 1, beta, yp, incy, batch)
        torch.cuda.synchronize()
        Ah, xh, yh, y0h = A.cpu().numpy(), x.cpu().numpy(), y.cpu().numpy(), y0.cpu().numpy()
        is_out = np.zeros(yh.size, dtype=bool)
        for b in range(batch):
            sl = slice(offy[b], offy[b] + exty)
            is_out[offy[b]: offy[b] + exty: abs(incy)] = True
            kw = dict(lda=lda, incy=incy)
            args = (prec, trans, m, n, alpha, Ah[offA[b]:], xh[offx[b]: offx[b] + lenx], beta, y0h[sl])
            want = oracle.gemv(*args, mode=oracle.MODE_X, **kw)
            den = oracle.gemv(*args, mode=oracle.MODE_ABS, **kw)
            err = errors(prec, logical(yh[sl], leny, incy), logical(want, leny, incy), logical(den, leny, incy), lenx)
            check(prec, err, f"{prec}gemv_batched {trans} {m}x{n} member {b}/{batch}")
        assert np.array_equal(yh[~is_out].view(np.uint8), y0h[~is_out].view(np.uint8)), "wrote between outputs"


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("uplo", "LU")
@pytest.mark.parametrize("csym", [False, True])
def test_symv_pointer_array_batched(prec, uplo, csym):
    if csym and prec not in "cz":
        pytest.skip("complex symmetric exists for c and z")
    k = kmv()
    alpha, beta = scal(prec, -1.1, 0.4)
    rng = np.random.default_rng(6)
    for n, batch, pad, incy in [(1, 2, 0, 1), (3, 3, 1, 1), (9, 3, 1, -1), (17, 3, 1, 1), (33, 4, 0, 1), (64, 2, 0, 2),
                                (100, 3, 1, 1), (129, 4, 0, -2), (257, 2, 5, 1), (512, 3, 0, 1), (640, 2, 0, 1),
                                (1024, 2, 0, 1), (1100, 3, 0, 1)]:
        lda = n + (pad % 4)
        exty = 1 + (n - 1) * abs(incy)
        offA, sizeA = _member_offsets(batch, lda * n, rng)
        offy, sizey = _member_offsets(batch, exty, rng)
        A = rand(prec, sizeA, 41 + n)
        host = A.cpu().numpy()
        for b in range(batch):
            blk = A[offA[b]: offA[b] + lda * n].view(n, lda)
            wl.poison_triangle(blk, n, uplo, real_diag=False)
            if prec in "cz" and not csym:
                d = torch.arange(n, device=DEV)
                torch.view_as_real(blk)[d, d, 1] = NAN
        x = rand(prec, n * batch, 42 + n)
        y0 = torch.full((sizey,), NAN, dtype=wl.TORCH_DTYPES[prec], device=DEV)
        vals = rand(prec, batch * n, 43 + n).view(batch, n)
        for b in range(batch):
            y0[offy[b]: offy[b] + exty: abs(incy)] = vals[b]
        y = y0.clone()
        Ap = k.pointer_array([A[o:] for o in offA])
        xp = k.pointer_array([x[b * n:] for b in range(batch)])
        yp = k.pointer_array([y[o:] for o in offy])
        (k.CSYMV_BATCHED if csym else k.SYMV_BATCHED)[prec](uplo, n, alpha, Ap, lda, xp, 1, beta, yp, incy, batch)
        torch.cuda.synchronize()
        xh, yh, y0h = x.cpu().numpy(), y.cpu().numpy(), y0.cpu().numpy()
        is_out = np.zeros(yh.size, dtype=bool)
        for b in range(batch):
            sl = slice(offy[b], offy[b] + exty)
            is_out[offy[b]: offy[b] + exty: abs(incy)] = True
            args = (prec, uplo, n, alpha, host[offA[b]:], xh[b * n: b * n + n], beta, y0h[sl])
            want = oracle.symv(*args, lda=lda, incy=incy, mode=oracle.MODE_X, complex_symmetric=csym)
            den = oracle.symv(*args, lda=lda, incy=incy, mode=oracle.MODE_ABS, complex_symmetric=csym)
            err = errors(prec, logical(yh[sl], n, incy), logical(want, n, incy), logical(den, n, incy), n)
            check(prec, err, f"symv/hemv_batched {prec} {uplo} n={n} member {b}/{batch}")
        assert np.array_equal(yh[~is_out].view(np.uint8), y0h[~is_out].view(np.uint8)), "wrote between outputs"


def test_pointer_array_batch_longer_than_one_launch_and_special_scalars():
    k = kmv()
    m, n, batch = 4, 3, 70000
    A = rand("d", batch * m * n, 1)
    x = rand("d", batch * n, 2)
    y0 = rand("d", batch * m, 3)
    y = y0.clone()
    base = torch.arange(batch, dtype=torch.int64, device=DEV)
    Ap = A.data_ptr() + base * (m * n * 8)
    xp = x.data_ptr() + base * (n * 8)
    yp = y.data_ptr() + base * (m * 8)
    k.dgemv_batched("N", m, n, 2.0, Ap, m, xp, 1, -1.0, yp, 1, batch)
    torch.cuda.synchronize()
    Ah = A.cpu().numpy().reshape(batch, n, m)
    want = 2.0 * np.einsum("bji,bj->bi", Ah, x.cpu().numpy().reshape(batch, n)) - y0.cpu().numpy().reshape(batch, m)
    assert np.max(np.abs(y.cpu().numpy().reshape(batch, m) - want)) <= 1e-14
    # alpha = 0: y <- beta*y, the arrays of A and x are not looked at
    y.copy_(y0)
    k.dgemv_batched("T", n, m, 0.0, None, n, None, 1, 3.0, yp, 1, batch)
    assert torch.equal(y, 3.0 * y0)
    k.dsymv_batched("L", 2, 0.0, None, 2, None, 1, 1.0, yp, 1, batch)          # alpha = 0, beta = 1: nothing happens
    k.dsymv_batched("U", 2, 1.0, Ap, 2, xp, 1, 0.0, yp, 1, 0)                  # empty batch
    assert torch.equal(y, 3.0 * y0)


@pytest.mark.parametrize("prec", PRECS)
def test_random_batched_shapes(prec):
    """seeded random member sizes, batch counts, paddings and increments through the strided forms
    (KMV_FUZZ_CASES / KMV_FUZZ_SEED in the environment lengthen or reseed the series)"""
    import os
    rng = np.random.default_rng({"s": 21, "d": 22, "c": 23, "z": 24}[prec] + 100 * int(os.environ.get("KMV_FUZZ_SEED", "0")))
    count = int(os.environ.get("KMV_FUZZ_CASES", "12"))
    k = kmv()
    sizes = [1, 2, 3, 5, 8, 13, 16, 24, 32, 47, 64, 96, 128, 200, 256, 300, 511, 700, 1030]
    gemv_cases, symv_cases = [], []
    for _ in range(count):
        m = int(rng.choice(sizes) + rng.integers(0, 3))
        n = int(rng.choice(sizes) + rng.integers(0, 3))
        gemv_cases.append((m, n, int(rng.integers(1, 6)), int(rng.choice([0, 1, 3, 16])), int(rng.choice([1, 1, 2, -1]))))
        symv_cases.append((n, int(rng.integers(1, 5)), int(rng.choice([0, 1, 2, 16])), int(rng.choice([1, 1, 2, -1]))))
    for trans in "NTC":
        _gemv_batched_cases(k, prec, trans, gemv_cases)
    for uplo in "LU":
        _symv_batched_case(prec, uplo, False, symv_cases)
        if prec in "cz":
            _symv_batched_case(prec, uplo, True, symv_cases)
