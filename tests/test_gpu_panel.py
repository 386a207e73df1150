"""Panel step of the symmetric tridiagonal reduction (kmv_{s,d}sytrd_panel) against the numpy oracle:
the reflectors, tau, e, the diagonal and W, on matrices that span several tiles, with ragged sizes, padded
leading dimensions and sub-block pointers; the strict upper triangle is NaN and must stay unread and
unwritten, the trailing columns must stay bit-unchanged."""
import numpy as np
import pytest
import torch

from oracle import panel_oracle as po
from paper_1410_1726_amd import workloads as wl

import panel_checks as pc
from gpu_util import DEV, kmv

pytestmark = pytest.mark.gpu

# What a panel result must satisfy is stated per case in panel_checks: the device's deviation from the wide oracle
# against the working-precision oracle's own deviation on the same input (factor panel_checks.K_DEV), and the
# factorisation identities at the tolerance of a single product.
def show(log):
    for entry in log:
        print("   ", entry[0], " ".join(f"{v:.3e}" for v in entry[1:]))


def run_panel(prec, n, nb, lda, ldw, off=0, seed=0):
    k = kmv()
    dt = wl.TORCH_DTYPES[prec]
    parent = wl.matrix(prec, n + off, n + off, lda, seed=seed, device=DEV)
    A = parent[off:, off:] if off else parent
    wl.poison_triangle(A, n, "L")
    before = parent.clone()
    W = torch.full((nb, ldw), float("nan"), dtype=dt, device=DEV)      # column major n x nb, leading dimension ldw
    e = torch.full((nb,), float("nan"), dtype=dt, device=DEV)
    tau = torch.full((nb,), float("nan"), dtype=dt, device=DEV)
    k.SYTRD_PANEL[prec]("L", n, nb, A, lda, e, tau, W, ldw)
    torch.cuda.synchronize()
    return parent, before, W, e, tau


def host_matrix(parent, off, n):
    """n x n numpy array (row index first) of the block that starts at (off, off)"""
    return parent[off:off + n, off:off + n].cpu().numpy().T.copy()


@pytest.mark.parametrize("prec", "sd")
@pytest.mark.parametrize("n,nb,pad,off", [(1, 1, 0, 0), (2, 2, 0, 0), (3, 1, 1, 0), (100, 16, 0, 0), (700, 32, 36, 0),
                                          (1500, 64, 0, 0), (1100, 24, 52, 17), (300, 300, 4, 1)])
def test_panel_against_oracle(prec, n, nb, pad, off):
    check_panel(prec, n, nb, pad, off)


def test_panel_with_many_rows():
    """more than 16384 rows: the panel's own kernels take several passes per workgroup, and the reflector kernel
    more rows than it fetches ahead"""
    check_panel("s", 20000, 3, 0, 0)


def check_panel(prec, n, nb, pad, off):
    lda, ldw = n + off + pad, n + (pad // 2)
    parent, before, W, e, tau = run_panel(prec, n, nb, lda, ldw, off, seed=n + nb)
    A0 = host_matrix(before, off, n)
    want = po.sytrd_panel(A0, nb)
    work = po.sytrd_panel(A0, nb, wide=False)
    A1 = host_matrix(parent, off, n)
    log = []
    low = np.tril(np.ones((n, n), dtype=bool))[:, :nb]
    for i in range(min(nb, n - 1)):
        assert A1[i + 1, i] == 1.0
    Wh = W.cpu().numpy().T[:n]                       # n x nb
    defined = np.zeros((n, nb), dtype=bool)
    for i in range(nb):
        defined[i + 1:, i] = True
    assert np.all(np.isfinite(Wh[defined]))
    what = f"{prec}sytrd_panel L n={n} nb={nb}"
    if nb <= 64:
        # element by element: the first nb columns (diagonal, leading ones, reflector tails), e, tau, W
        pc.against_oracles(prec, what + " columns", A1[:, :nb][low], np.asarray(want["A"])[:, :nb][low],
                           np.asarray(work["A"])[:, :nb][low], log)
        pc.against_oracles(prec, what + " e", e.cpu().numpy(), want["e"], work["e"], log)
        pc.against_oracles(prec, what + " tau", tau.cpu().numpy(), want["tau"], work["tau"], log)
        pc.against_oracles(prec, what + " W", Wh[defined], np.asarray(want["W"])[defined], np.asarray(work["W"])[defined], log)
    else:
        # A long chain of dependent columns: single reflector entries of the late columns are not determined to
        # working accuracy any more (they see a matrix that carries all earlier rounding; the working-precision
        # oracle's own entries are off by orders of magnitude more than a product's tolerance), but the
        # factorisation as a whole is: the identities below, and the diagonal against the oracles.
        pc.against_oracles(prec, what + " d", np.diag(A1)[:nb], np.diag(np.asarray(want["A"]))[:nb],
                           np.diag(np.asarray(work["A"]))[:nb], log)
    pc.check_identities(prec, what, pc.trd_identities(prec, "L", A0, A1, tau.cpu().numpy(), e.cpu().numpy(), Wh, nb), log)
    show(log)
    # untouched: everything of the parent outside the first nb columns of the block's lower triangle
    pb, pa = before.cpu().numpy(), parent.cpu().numpy()          # (cols, lda)
    touched = np.zeros(pb.shape, dtype=bool)
    for i in range(nb):
        touched[off + i, off + i:off + n] = True
    assert np.array_equal(pb[~touched].view(np.uint8), pa[~touched].view(np.uint8)), "wrote outside the panel"
    # rows of W beyond n (the padding of ldw) were not written
    assert np.all(np.isnan(W.cpu().numpy()[:, n:]))


@pytest.mark.parametrize("prec", "sd")
def test_panel_is_deterministic_and_capturable(prec):
    """the whole panel is a sequence of kernel launches with no host round trip: captured in a graph and
    replayed on restored inputs, every replay reproduces the eager result bit for bit"""
    k = kmv()
    n, nb = 900, 32
    dt = wl.TORCH_DTYPES[prec]
    A0 = wl.poison_triangle(wl.matrix(prec, n, n, n, seed=3, device=DEV), n, "L")
    A = A0.clone()
    W = torch.zeros((nb, n), dtype=dt, device=DEV)
    e = torch.zeros(nb, dtype=dt, device=DEV)
    tau = torch.zeros(nb, dtype=dt, device=DEV)
    ws = k.workspace(k.sytrd_panel_workspace_bytes(prec, n, nb))
    k.SYTRD_PANEL[prec]("L", n, nb, A, n, e, tau, W, n, workspace=ws)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (A, W, e, tau)]
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    A.copy_(A0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            k.SYTRD_PANEL[prec]("L", n, nb, A, n, e, tau, W, n, workspace=ws, stream=side)
    for _ in range(3):
        A.copy_(A0)
        for t in (W, e, tau):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip((A, e, tau), (ref[0], ref[2], ref[3])):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
        rows = torch.arange(n, device=DEV).unsqueeze(0)
        cols = torch.arange(nb, device=DEV).unsqueeze(1)
        defined = rows > cols
        assert torch.equal(W[defined], ref[1][defined])


@pytest.mark.parametrize("prec", "cz")
@pytest.mark.parametrize("n,nb,pad,off", [(1, 1, 0, 0), (2, 2, 0, 0), (3, 1, 1, 0), (100, 16, 0, 0), (700, 32, 36, 0),
                                          (1500, 64, 0, 0), (1100, 24, 52, 17)])
def test_hermitian_panel_against_oracle(prec, n, nb, pad, off):
    """kmv_{c,z}hetrd_panel: reflectors, the real e, the complex tau, W and the real diagonal element by element;
    the strict upper triangle and the imaginary parts of the diagonal are NaN on entry"""
    k = kmv()
    dt = wl.TORCH_DTYPES[prec]
    rdt = torch.float32 if prec == "c" else torch.float64
    lda, ldw = n + off + pad, n + (pad // 2)
    parent = wl.matrix(prec, n + off, n + off, lda, seed=n + nb, device=DEV)
    A = parent[off:, off:] if off else parent
    wl.poison_triangle(A, n, "L", real_diag=False)
    host0 = parent.clone()                               # the oracle ignores the diagonal's imaginary part
    dd = torch.arange(n, device=DEV)
    torch.view_as_real(A)[dd, dd, 1] = float("nan")      # ... which is NaN for the device
    before = parent.clone()
    nanv = float("nan")
    W = torch.full((nb, ldw), nanv, dtype=dt, device=DEV)
    e = torch.full((nb,), nanv, dtype=rdt, device=DEV)
    tau = torch.full((nb,), nanv, dtype=dt, device=DEV)
    k.SYTRD_PANEL[prec]("L", n, nb, A, lda, e, tau, W, ldw)
    torch.cuda.synchronize()
    A0 = host_matrix(host0, off, n)
    want = po.hetrd_panel(A0, nb)
    work = po.hetrd_panel(A0, nb, wide=False)
    A1 = host_matrix(parent, off, n)
    log = []
    what = f"{prec}hetrd_panel L n={n} nb={nb}"
    low = np.tril(np.ones((n, n), dtype=bool))[:, :nb]
    got_cols = A1[:, :nb][low]
    assert np.all(np.isfinite(got_cols.view(np.float32 if prec == "c" else np.float64))), "a NaN was read"
    pc.against_oracles(prec, what + " columns", got_cols, np.asarray(want["A"])[:, :nb][low], np.asarray(work["A"])[:, :nb][low], log)
    for i in range(nb):
        assert A1[i, i].imag == 0
        if i < n - 1:
            assert A1[i + 1, i] == 1.0
    pc.against_oracles(prec, what + " e", e.cpu().numpy(), want["e"], work["e"], log)
    pc.against_oracles(prec, what + " tau", tau.cpu().numpy(), want["tau"], work["tau"], log)
    Wh = W.cpu().numpy().T[:n]
    defined = np.zeros((n, nb), dtype=bool)
    for i in range(nb):
        defined[i + 1:, i] = True
    pc.against_oracles(prec, what + " W", Wh[defined], np.asarray(want["W"])[defined], np.asarray(work["W"])[defined], log)
    if pc.affordable(prec, n, nb):
        pc.check_identities(prec, what, pc.trd_identities(prec, "L", A0, A1, tau.cpu().numpy(), e.cpu().numpy(), Wh, nb), log)
    show(log)
    pb, pa = before.cpu().numpy(), parent.cpu().numpy()
    touched = np.zeros(pb.shape, dtype=bool)
    for i in range(nb):
        touched[off + i, off + i:off + n] = True
    keep = ~touched
    assert np.array_equal(pb[keep].view(np.uint8), pa[keep].view(np.uint8)), "wrote outside the panel"
    # the diagonal beyond the panel keeps its real part and its (NaN) imaginary part
    for i in range(nb, n):
        assert A1[i, i].real == A0[i, i].real and np.isnan(A1[i, i].imag)


# ------------------------------------------------------------ bidiagonal panel ----
from oracle import gebrd_panel_oracle as go   # noqa: E402


@pytest.mark.parametrize("prec", "sd")
@pytest.mark.parametrize("m,n,nb,pad,off", [(1, 1, 1, 0, 0), (2, 2, 2, 0, 0), (5, 3, 3, 1, 0), (100, 100, 16, 0, 0),
                                            (700, 500, 32, 36, 0), (1500, 1500, 64, 0, 0), (1300, 900, 24, 52, 17),
                                            (900, 1500 - 700, 8, 3, 1), (900, 700, 260, 4, 0), (700, 520, 200, 4, 0),
                                            (70000, 40, 8, 0, 0)])
def test_gebrd_panel_against_oracle(prec, m, n, nb, pad, off):
    """kmv_{s,d}gebrd_panel on a block at (off, off) of a parent with padded leading dimension: reflector
    vectors, d, e, tauq, taup, X and Y element by element; everything outside the first nb rows and columns
    of the block bit-unchanged"""
    k = kmv()
    dt = wl.TORCH_DTYPES[prec]
    lda, ldx, ldy = m + off + pad, m + pad // 2, n + pad // 3
    parent = wl.matrix(prec, m + off, n + off, lda, seed=m + n + nb, device=DEV)
    before = parent.clone()
    A = parent[off:, off:] if off else parent
    nanv = float("nan")
    X = torch.full((nb, ldx), nanv, dtype=dt, device=DEV)
    Y = torch.full((nb, ldy), nanv, dtype=dt, device=DEV)
    d, e, tauq, taup = (torch.full((nb,), nanv, dtype=dt, device=DEV) for _ in range(4))
    k.GEBRD_PANEL[prec](m, n, nb, A, lda, d, e, tauq, taup, X, ldx, Y, ldy)
    torch.cuda.synchronize()
    A0 = before[off:off + n, off:off + m].cpu().numpy().T.copy()
    A1 = parent[off:off + n, off:off + m].cpu().numpy().T.copy()
    want = go.gebrd_panel(A0, nb)
    work = go.gebrd_panel(A0, nb, wide=False)
    log = []
    what = f"{prec}gebrd_panel {m}x{n} nb={nb}"
    panel = np.zeros((m, n), dtype=bool)       # first nb columns (column reflectors) and first nb rows (row reflectors)
    panel[:, :nb] = True
    panel[:nb, :] = True
    pc.against_oracles(prec, what + " A", A1[panel], np.asarray(want["A"])[panel], np.asarray(work["A"])[panel], log)
    for name, got in (("d", d), ("e", e), ("tauq", tauq), ("taup", taup)):
        pc.against_oracles(prec, what + " " + name, got.cpu().numpy(), want[name], work[name], log)
    Xh, Yh = X.cpu().numpy().T[:m], Y.cpu().numpy().T[:n]
    dx = np.zeros((m, nb), dtype=bool)
    dy = np.zeros((n, nb), dtype=bool)
    for i in range(min(nb, min(m, n) - 1)):
        dx[i + 1:, i] = True
        dy[i + 1:, i] = True
    assert np.all(np.isfinite(np.asarray(Xh[dx], dtype=np.complex128).view(np.float64)))
    assert np.all(np.isfinite(np.asarray(Yh[dy], dtype=np.complex128).view(np.float64)))
    pc.against_oracles(prec, what + " X", Xh[dx], np.asarray(want["X"])[dx], np.asarray(work["X"])[dx], log)
    pc.against_oracles(prec, what + " Y", Yh[dy], np.asarray(want["Y"])[dy], np.asarray(work["Y"])[dy], log)
    if pc.affordable(prec, max(m, n), nb):
        Xz, Yz = np.where(dx, Xh, 0), np.where(dy, Yh, 0)       # undefined entries (scratch) count as zero
        pc.check_identities(prec, what, pc.gebrd_identities(prec, A0, A1, d.cpu().numpy(), e.cpu().numpy(), tauq.cpu().numpy(),
                                                            taup.cpu().numpy(), Xz, Yz, nb), log)
    show(log)
    # untouched: the parent outside the block, the padding, and the block beyond the panel
    pb, pa = before.cpu().numpy(), parent.cpu().numpy()           # (cols, lda)
    touched = np.zeros(pb.shape, dtype=bool)
    touched[off:off + nb, off:off + m] = True                      # first nb columns of the block
    touched[off:off + n, off:off + nb] = True                      # first nb rows of the block
    assert np.array_equal(pb[~touched].view(np.uint8), pa[~touched].view(np.uint8)), "wrote outside the panel"
    assert np.all(np.isnan(X.cpu().numpy()[:, m:])) and np.all(np.isnan(Y.cpu().numpy()[:, n:]))


@pytest.mark.parametrize("prec,m,n", [("d", 900, 700), ("c", 500, 800)])
def test_gebrd_panel_is_deterministic_and_capturable(prec, m, n):
    """the bidiagonal panel (fused kernels plus the two products per column) is launches only: captured in a
    graph and replayed on restored inputs, every replay reproduces the eager result bit for bit"""
    k = kmv()
    nb = 32
    dt = wl.TORCH_DTYPES[prec]
    rdt = {"d": torch.float64, "c": torch.float32}[prec]
    A0 = wl.matrix(prec, m, n, m, seed=5, device=DEV)
    A = A0.clone()
    X = torch.zeros((nb, m), dtype=dt, device=DEV)
    Y = torch.zeros((nb, n), dtype=dt, device=DEV)
    d, e = (torch.zeros(nb, dtype=rdt, device=DEV) for _ in range(2))
    tauq, taup = (torch.zeros(nb, dtype=dt, device=DEV) for _ in range(2))
    ws = k.workspace(k.gebrd_panel_workspace_bytes(prec, m, n, nb))
    k.GEBRD_PANEL[prec](m, n, nb, A, m, d, e, tauq, taup, X, m, Y, n, workspace=ws)
    torch.cuda.synchronize()
    outs = (A, d, e, tauq, taup)
    ref = [t.clone() for t in outs]
    refX, refY = X.clone(), Y.clone()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    A.copy_(A0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            k.GEBRD_PANEL[prec](m, n, nb, A, m, d, e, tauq, taup, X, m, Y, n, workspace=ws, stream=side)
    cols = torch.arange(nb, device=DEV).unsqueeze(1)
    for _ in range(3):
        A.copy_(A0)
        for t in (d, e, tauq, taup, X, Y):
            t.fill_(float("nan"))
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs, ref):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
        for got, want, rows in ((X, refX, m), (Y, refY, n)):
            defined = torch.arange(rows, device=DEV).unsqueeze(0) > cols
            assert torch.equal(torch.view_as_real(got[defined]) if got.is_complex() else got[defined],
                               torch.view_as_real(want[defined]) if want.is_complex() else want[defined])


@pytest.mark.parametrize("prec", "cz")
@pytest.mark.parametrize("m,n,nb,pad,off", [(1, 1, 1, 0, 0), (2, 2, 2, 0, 0), (5, 3, 3, 1, 0), (100, 100, 16, 0, 0),
                                            (700, 500, 32, 36, 0), (1500, 1500, 64, 0, 0), (1300, 900, 24, 52, 17),
                                            (900, 800, 8, 3, 1), (600, 500, 260, 4, 0), (600, 420, 200, 4, 0),
                                            (70000, 40, 8, 0, 0)])
def test_complex_gebrd_panel_against_oracle(prec, m, n, nb, pad, off):
    """kmv_{c,z}gebrd_panel: reflector vectors (rows stored as u^H), the real d and e, the complex tauq and
    taup, X and Y element by element; everything outside the first nb rows and columns bit-unchanged"""
    k = kmv()
    dt = wl.TORCH_DTYPES[prec]
    rdt = torch.float32 if prec == "c" else torch.float64
    lda, ldx, ldy = m + off + pad, m + pad // 2, n + pad // 3
    parent = wl.matrix(prec, m + off, n + off, lda, seed=m + n + nb + 1, device=DEV)
    before = parent.clone()
    A = parent[off:, off:] if off else parent
    nanv = float("nan")
    X = torch.full((nb, ldx), nanv, dtype=dt, device=DEV)
    Y = torch.full((nb, ldy), nanv, dtype=dt, device=DEV)
    d, e = (torch.full((nb,), nanv, dtype=rdt, device=DEV) for _ in range(2))
    tauq, taup = (torch.full((nb,), nanv, dtype=dt, device=DEV) for _ in range(2))
    k.GEBRD_PANEL[prec](m, n, nb, A, lda, d, e, tauq, taup, X, ldx, Y, ldy)
    torch.cuda.synchronize()
    A0 = before[off:off + n, off:off + m].cpu().numpy().T.copy()
    A1 = parent[off:off + n, off:off + m].cpu().numpy().T.copy()
    want = go.gebrd_panel(A0, nb)
    work = go.gebrd_panel(A0, nb, wide=False)
    log = []
    what = f"{prec}gebrd_panel {m}x{n} nb={nb}"
    panel = np.zeros((m, n), dtype=bool)       # first nb columns (column reflectors) and first nb rows (row reflectors)
    panel[:, :nb] = True
    panel[:nb, :] = True
    pc.against_oracles(prec, what + " A", A1[panel], np.asarray(want["A"])[panel], np.asarray(work["A"])[panel], log)
    for name, got in (("d", d), ("e", e), ("tauq", tauq), ("taup", taup)):
        pc.against_oracles(prec, what + " " + name, got.cpu().numpy(), want[name], work[name], log)
    Xh, Yh = X.cpu().numpy().T[:m], Y.cpu().numpy().T[:n]
    dx = np.zeros((m, nb), dtype=bool)
    dy = np.zeros((n, nb), dtype=bool)
    for i in range(min(nb, min(m, n) - 1)):
        dx[i + 1:, i] = True
        dy[i + 1:, i] = True
    assert np.all(np.isfinite(np.asarray(Xh[dx], dtype=np.complex128).view(np.float64)))
    assert np.all(np.isfinite(np.asarray(Yh[dy], dtype=np.complex128).view(np.float64)))
    pc.against_oracles(prec, what + " X", Xh[dx], np.asarray(want["X"])[dx], np.asarray(work["X"])[dx], log)
    pc.against_oracles(prec, what + " Y", Yh[dy], np.asarray(want["Y"])[dy], np.asarray(work["Y"])[dy], log)
    if pc.affordable(prec, max(m, n), nb):
        Xz, Yz = np.where(dx, Xh, 0), np.where(dy, Yh, 0)       # undefined entries (scratch) count as zero
        pc.check_identities(prec, what, pc.gebrd_identities(prec, A0, A1, d.cpu().numpy(), e.cpu().numpy(), tauq.cpu().numpy(),
                                                            taup.cpu().numpy(), Xz, Yz, nb), log)
    show(log)
    pb, pa = before.cpu().numpy(), parent.cpu().numpy()
    touched = np.zeros(pb.shape, dtype=bool)
    touched[off:off + nb, off:off + m] = True
    touched[off:off + n, off:off + nb] = True
    assert np.array_equal(pb[~touched].view(np.uint8), pa[~touched].view(np.uint8)), "wrote outside the panel"
    assert np.all(np.isnan(X.cpu().numpy()[:, m:].real)) and np.all(np.isnan(Y.cpu().numpy()[:, n:].real))


# ------------------------------------------------------------ upper storage ----
@pytest.mark.parametrize("prec", "sdcz")
@pytest.mark.parametrize("n,nb,pad,off", [(1, 1, 0, 0), (2, 2, 0, 0), (3, 1, 1, 0), (100, 16, 0, 0), (700, 32, 36, 0),
                                          (1500, 64, 0, 0), (1100, 24, 52, 17), (60, 60, 4, 1)])
def test_upper_storage_panel_against_oracle(prec, n, nb, pad, off):
    """uplo = 'U': the last nb columns are reduced (SYMV / HEMV 'U' on the leading block, GEMV on the columns to
    the right).  Reflectors, e, tau, W and the diagonal element by element; the strict lower triangle (and the
    imaginary parts of a complex diagonal) are NaN on entry; everything outside the panel's columns bit-unchanged."""
    k = kmv()
    cplx = prec in "cz"
    dt = wl.TORCH_DTYPES[prec]
    rdt = {"s": torch.float32, "d": torch.float64, "c": torch.float32, "z": torch.float64}[prec]
    lda, ldw = n + off + pad, n + (pad // 2)
    parent = wl.matrix(prec, n + off, n + off, lda, seed=n + nb + 2, device=DEV)
    A = parent[off:, off:] if off else parent
    wl.poison_triangle(A, n, "U", real_diag=False)
    host0 = parent.clone()
    if cplx:
        dd = torch.arange(n, device=DEV)
        torch.view_as_real(A)[dd, dd, 1] = float("nan")
    before = parent.clone()
    nanv = float("nan")
    W = torch.full((nb, ldw), nanv, dtype=dt, device=DEV)
    e = torch.full((nb,), nanv, dtype=rdt, device=DEV)
    tau = torch.full((nb,), nanv, dtype=dt, device=DEV)
    k.SYTRD_PANEL[prec]("U", n, nb, A, lda, e, tau, W, ldw)
    torch.cuda.synchronize()
    A0 = host_matrix(host0, off, n)
    want = po.trd_panel_upper(A0, nb)
    work = po.trd_panel_upper(A0, nb, wide=False)
    A1 = host_matrix(parent, off, n)
    log = []
    what = f"{prec} trd_panel U n={n} nb={nb}"
    first = n - nb
    up = np.triu(np.ones((n, n), dtype=bool))
    up[:, :first] = False                                  # upper part of the last nb columns
    got_cols = A1[up]
    assert np.all(np.isfinite(np.asarray(got_cols, dtype=np.complex128).view(np.float64))), "a NaN was read"
    for i in range(first, n):
        assert np.asarray(A1[i, i]).imag == 0
        if i > 0:
            assert A1[i - 1, i] == 1.0
    Wh = W.cpu().numpy().T[:n]
    defined = np.zeros((n, nb), dtype=bool)
    for iw in range(nb):
        defined[:first + iw, iw] = True
    assert np.all(np.isfinite(np.asarray(Wh[defined], dtype=np.complex128).view(np.float64)))
    if nb < n:
        pc.against_oracles(prec, what + " columns", got_cols, np.asarray(want["A"])[up], np.asarray(work["A"])[up], log)
        pc.against_oracles(prec, what + " e", e.cpu().numpy(), want["e"], work["e"], log)
        pc.against_oracles(prec, what + " tau", tau.cpu().numpy(), want["tau"], work["tau"], log)
        pc.against_oracles(prec, what + " W", Wh[defined], np.asarray(want["W"])[defined], np.asarray(work["W"])[defined], log)
    else:
        # a full reduction is a long chain of dependent columns: single reflector entries of the late (small)
        # columns are not determined to working accuracy, the factorisation as a whole is: the identities
        # below, and the diagonal against the oracles
        pc.against_oracles(prec, what + " d", np.real(np.diag(A1)), np.real(np.diag(np.asarray(want["A"]))),
                           np.real(np.diag(np.asarray(work["A"]))), log)
    if pc.affordable(prec, n, nb):
        Wz = np.where(defined, Wh, 0)
        tz, ez = tau.cpu().numpy().copy(), e.cpu().numpy().copy()
        pc.check_identities(prec, what, pc.trd_identities(prec, "U", A0, A1, tz, ez, Wz, nb), log)
    show(log)
    pb, pa = before.cpu().numpy(), parent.cpu().numpy()    # (column, row)
    touched = np.zeros(pb.shape, dtype=bool)
    for i in range(first, n):
        touched[off + i, off:off + i + 1] = True
    assert np.array_equal(pb[~touched].view(np.uint8), pa[~touched].view(np.uint8)), "wrote outside the panel"
    if cplx:       # the diagonal before the panel keeps its real part and its (NaN) imaginary part
        for i in range(first):
            assert A1[i, i].real == A0[i, i].real and np.isnan(A1[i, i].imag)


@pytest.mark.parametrize("prec", "sdcz")
@pytest.mark.parametrize("m,n,nb,pad,off", [(1, 2, 1, 0, 0), (2, 3, 2, 0, 0), (3, 5, 3, 1, 0), (100, 101, 16, 0, 0),
                                            (500, 700, 32, 36, 0), (900, 1300, 24, 52, 17), (800, 900, 8, 3, 1),
                                            (500, 700, 260, 4, 0), (420, 600, 256, 4, 0), (40, 70000, 8, 0, 0)])
def test_wide_gebrd_panel_against_oracle(prec, m, n, nb, pad, off):
    """m < n: lower bidiagonal form (row reflectors first).  Reflector vectors, the real d and e, tauq, taup, X
    and Y element by element; everything outside the first nb rows and columns bit-unchanged"""
    k = kmv()
    cplx = prec in "cz"
    dt = wl.TORCH_DTYPES[prec]
    rdt = {"s": torch.float32, "d": torch.float64, "c": torch.float32, "z": torch.float64}[prec]
    lda, ldx, ldy = m + off + pad, m + pad // 2, n + pad // 3
    parent = wl.matrix(prec, m + off, n + off, lda, seed=m + n + nb + 5, device=DEV)
    before = parent.clone()
    A = parent[off:, off:] if off else parent
    nanv = float("nan")
    X = torch.full((nb, ldx), nanv, dtype=dt, device=DEV)
    Y = torch.full((nb, ldy), nanv, dtype=dt, device=DEV)
    d, e = (torch.full((nb,), nanv, dtype=rdt, device=DEV) for _ in range(2))
    tauq, taup = (torch.full((nb,), nanv, dtype=dt, device=DEV) for _ in range(2))
    k.GEBRD_PANEL[prec](m, n, nb, A, lda, d, e, tauq, taup, X, ldx, Y, ldy)
    torch.cuda.synchronize()
    A0 = before[off:off + n, off:off + m].cpu().numpy().T.copy()
    A1 = parent[off:off + n, off:off + m].cpu().numpy().T.copy()
    want = go.gebrd_panel_wide(A0, nb)
    work = go.gebrd_panel_wide(A0, nb, wide=False)
    log = []
    what = f"{prec}gebrd_panel (wide) {m}x{n} nb={nb}"
    panel = np.zeros((m, n), dtype=bool)
    panel[:, :nb] = True
    panel[:nb, :] = True
    pc.against_oracles(prec, what + " A", A1[panel], np.asarray(want["A"])[panel], np.asarray(work["A"])[panel], log)
    for name, got in (("d", d), ("e", e), ("tauq", tauq), ("taup", taup)):
        pc.against_oracles(prec, what + " " + name, got.cpu().numpy(), want[name], work[name], log)
    Xh, Yh = X.cpu().numpy().T[:m], Y.cpu().numpy().T[:n]
    dx = np.zeros((m, nb), dtype=bool)
    dy = np.zeros((n, nb), dtype=bool)
    for i in range(min(nb, m - 1)):
        dx[i + 1:, i] = True
        dy[i + 1:, i] = True
    assert np.all(np.isfinite(np.asarray(Xh[dx], dtype=np.complex128).view(np.float64)))
    assert np.all(np.isfinite(np.asarray(Yh[dy], dtype=np.complex128).view(np.float64)))
    pc.against_oracles(prec, what + " X", Xh[dx], np.asarray(want["X"])[dx], np.asarray(work["X"])[dx], log)
    pc.against_oracles(prec, what + " Y", Yh[dy], np.asarray(want["Y"])[dy], np.asarray(work["Y"])[dy], log)
    if pc.affordable(prec, max(m, n), nb):
        Xz, Yz = np.where(dx, Xh, 0), np.where(dy, Yh, 0)
        pc.check_identities(prec, what, pc.gebrd_identities(prec, A0, A1, d.cpu().numpy(), e.cpu().numpy(), tauq.cpu().numpy(),
                                                            taup.cpu().numpy(), Xz, Yz, nb), log)
    show(log)
    pb, pa = before.cpu().numpy(), parent.cpu().numpy()
    touched = np.zeros(pb.shape, dtype=bool)
    touched[off:off + nb, off:off + m] = True
    touched[off:off + n, off:off + nb] = True
    assert np.array_equal(pb[~touched].view(np.uint8), pa[~touched].view(np.uint8)), "wrote outside the panel"
