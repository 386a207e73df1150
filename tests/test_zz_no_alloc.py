"""kmv_dsymv_static (the entry point for callers that cannot allocate: its workspace is a static device array
of the library) against kmv_dsymv with a caller's workspace, through the C ABI: two calls in a row, the second
on a smaller input, each compared bit for bit (same plan, same kernels, same summation order) and against the
oracle to the parity tolerance; sizes beyond the array are refused before anything is enqueued."""
import numpy as np
import pytest
import torch

import oracle
from paper_1410_1726_amd import binding as kmv
from paper_1410_1726_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pair(uplo, n, lda, incx, alpha, beta, seed):
    A = wl.poison_triangle(wl.matrix("d", n, n, lda, seed=seed, device=DEV), n, uplo)
    x = wl.vector("d", n, incx, seed=seed, which=1, device=DEV)
    y0 = wl.vector("d", n, 1, seed=seed, which=2, device=DEV)
    want, got = y0.clone(), y0.clone()
    kmv.dsymv(uplo, n, alpha, A, lda, x, incx, beta, want, 1)
    rc = kmv.dsymv_static(uplo, n, alpha, A, lda, x, incx, beta, got, 1)
    torch.cuda.synchronize()
    assert rc == 0
    assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), (uplo, n, "static scratch differs from caller workspace")
    xs = x.cpu().numpy()
    ref = oracle.symv("d", uplo, n, alpha, A.cpu().numpy().reshape(-1), xs, beta, y0.cpu().numpy(), lda=lda, incx=incx,
                      mode=oracle.MODE_X)
    g = got.cpu().numpy().astype(ref.dtype)
    err = np.linalg.norm(g - ref) / np.linalg.norm(ref)
    assert np.isfinite(err) and err <= 1e-13, (uplo, n, err)


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    # a large product first (two-kernel path, most of the array in use), then a smaller one that leaves the
    # first call's partial sums behind in the array, then a strided x (packed into the array) and the other triangle
    _pair("L", 6000, 6016, 1, 0.7, 0.3, seed=31)
    _pair("L", 2500, 2500, 1, -1.0, 0.0, seed=32)
    _pair("U", 3001, 3008, 2, 1.5, 1.0, seed=33)
    _pair("U", 700, 700, 1, 1.0, 0.5, seed=34)       # one-launch kernel: the array is not touched


def test_static_scratch_refuses_what_does_not_fit():
    n = 60000                       # needs more than the 16 MiB array; refused before the pointers are used
    dummy = 256
    y = torch.zeros(8, dtype=torch.float64, device=DEV)
    rc = kmv.dsymv_static("L", n, 1.0, dummy, n, dummy, 1, 0.0, y, 1, check=False)
    assert rc == kmv.ERR_WORKSPACE
    assert kmv.dsymv_static("Q", 10, 1.0, dummy, 10, dummy, 1, 0.0, y, 1, check=False) == -1
    torch.cuda.synchronize()
