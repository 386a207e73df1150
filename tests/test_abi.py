"""C-ABI checks that need no GPU: the library loads, exports every function the
header declares, rejects illegal arguments with the reference-BLAS argument
numbers before touching the device, and its host-side helpers (work partition,
workspace sizes, tuning keys) behave."""
import os
import re

import pytest

from paper_1410_1726_amd import binding as kmv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DUMMY = 0x1000   # a non-null "device address" that is never dereferenced on error paths
NOWS = (0, 0)


def declared_functions():
    src = open(os.path.join(ROOT, "include", "kmv.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(kmv_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert len(names) >= 16
    for n in names:
        assert hasattr(kmv.lib, n), f"{n} is declared in include/kmv.h but not exported"


@pytest.mark.parametrize("prec", "sdcz")
def test_gemv_argument_errors(prec):
    f = kmv.GEMV[prec]

    def call(trans="N", m=4, n=4, lda=4, incx=1, incy=1, A=DUMMY, x=DUMMY, y=DUMMY):
        return f(trans, m, n, 1.0, A, lda, x, incx, 0.0, y, incy, workspace=NOWS, stream=0, check=False)

    assert call(trans="X") == -1
    assert call(m=-1) == -2
    assert call(n=-1) == -3
    assert call(lda=3) == -6
    assert call(m=0, lda=0) == -6
    assert call(incx=0) == -8
    assert call(incy=0) == -11
    assert call(A=None) == kmv.ERR_NULL
    # quick returns enqueue nothing and need no device
    assert call(m=0, lda=1) == 0
    assert call(n=0) == 0
    assert f("T", 4, 4, 0.0, DUMMY, 4, DUMMY, 1, 1.0, DUMMY, 1, workspace=NOWS, stream=0, check=False) == 0
    # a strided x needs the workspace: missing -> error before any launch
    assert call(incx=2) == kmv.ERR_WORKSPACE
    with pytest.raises(kmv.KmvError):
        f("Q", 4, 4, 1.0, DUMMY, 4, DUMMY, 1, 0.0, DUMMY, 1, workspace=NOWS, stream=0)


@pytest.mark.parametrize("prec", ["s", "d", "c", "z", "c-symmetric", "z-symmetric"])
def test_symv_argument_errors(prec):
    f = kmv.CSYMV[prec[0]] if prec.endswith("symmetric") else kmv.SYMV[prec]

    def call(uplo="L", n=4, lda=4, incx=1, incy=1, A=DUMMY):
        return f(uplo, n, 1.0, A, lda, DUMMY, incx, 0.0, DUMMY, incy, workspace=NOWS, stream=0, check=False)

    assert call(uplo="N") == -1
    assert call(n=-1) == -2
    assert call(lda=3) == -5
    assert call(incx=0) == -7
    assert call(incy=0) == -10
    assert call(A=None) == kmv.ERR_NULL
    assert call(n=0, lda=1) == 0
    # the two-kernel path and a strided x need the workspace (the one-launch kernel with a contiguous x does not)
    assert call(n=5000, lda=5000) == kmv.ERR_WORKSPACE
    assert call(incx=2) == kmv.ERR_WORKSPACE
    assert f("u", 4, 0.0, DUMMY, 4, DUMMY, 1, 1.0, DUMMY, 1, workspace=NOWS, stream=0, check=False) == 0


def test_partition_invariants():
    # Section 6.2: shares are balanced (differ by at most one), contiguous, and
    # tile [0, W); workers beyond W get nothing
    for W in (0, 1, 5, 64, 1000, 4099):
        for Y in (1, 2, 3, 7, 16, 100, 5000):
            pos, sizes = 0, []
            for y in range(Y):
                w, s = kmv.partition(W, Y, y)
                assert s == pos and w >= 0
                pos += w
                sizes.append(w)
            assert pos == W
            assert max(sizes) - min(sizes) <= 1
            assert sizes == sorted(sizes, reverse=True)
    assert kmv.partition(10, 3, 0) == (4, 0)
    assert kmv.partition(10, 3, 1) == (3, 4)
    assert kmv.partition(10, 3, 2) == (3, 7)


def test_workspace_sizes():
    for prec, b in (("s", 4), ("d", 8), ("c", 8), ("z", 16)):
        for trans in "NTC":                           # empty products need no workspace (and no division by zero)
            for m, n in ((0, 0), (0, 7), (7, 0)):
                assert kmv.gemv_workspace_bytes(prec, trans, m, n) == 0
        assert kmv.symv_workspace_bytes(prec, "L", 0) == 0
        small = kmv.gemv_workspace_bytes(prec, "N", 1024, 1024)
        big = kmv.gemv_workspace_bytes(prec, "N", 4096, 4096)
        assert 0 < small <= big
        assert small >= 1024 * b                      # room for a packed x
        n = 8192
        s = kmv.symv_workspace_bytes(prec, "L", n)
        assert s >= n * b and s == kmv.symv_workspace_bytes(prec, "U", n)
        assert s < 0.2 * n * n * b                    # partial sums stay a small share of the matrix
        assert kmv.symv_workspace_bytes(prec, "L", 2048) < 32 << 20   # bounded by the most workgroups x the tallest chunk
    assert kmv.gemv_workspace_bytes("q", "N", 8, 8) == 0
    assert kmv.symv_workspace_bytes("d", "L", -1) == 0


def test_tuning_keys_roundtrip():
    keys = kmv.tuning_keys()
    assert "symv_tiles_per_wave" in keys
    for k in keys:
        old = kmv.get_tuning(k)
        val = {"symv_member_waves": 8, "symv_small_waves": 8, "gemv_tiny_rows": 100, "tuned_table": 1}.get(k, 2)
        kmv.set_tuning(k, val)
        assert kmv.get_tuning(k) == val
        kmv.set_tuning(k, old)
    with pytest.raises(ValueError):
        kmv.set_tuning("no_such_key", 1)
    with pytest.raises(ValueError):
        kmv.set_tuning("gemv_n_splits", 100000)
    with pytest.raises(ValueError):
        kmv.set_tuning("symv_variant", 1)           # the value of a kernel that no longer exists
    with pytest.raises(ValueError):
        kmv.set_tuning("symv_member_waves", 6)
    assert "kmv" in kmv.version()


def test_symv_kernel_variant_query():
    """host-only: names the main kernel without reading or launching anything"""
    assert kmv.symv_kernel_variant("d", "X", 100, DUMMY, 100) == 0
    assert kmv.symv_kernel_variant("q", "L", 100, DUMMY, 100) == 0
    assert kmv.symv_kernel_variant("d", "L", 100, DUMMY, 99) == 0
    for prec in "sdcz":
        for uplo in "LU":
            assert kmv.symv_kernel_variant(prec, uplo, 5000, DUMMY, 5000) == 2
            assert kmv.symv_kernel_variant(prec, uplo, 500, DUMMY, 500) == 3
            edge = {"s": 2176, "d": 2048, "c": 2048, "z": 1664}[prec]   # largest n of the single-launch kernel
            assert kmv.symv_kernel_variant(prec, uplo, edge, DUMMY, edge) == 3
            assert kmv.symv_kernel_variant(prec, uplo, edge + 1, DUMMY, edge + 1) == 2
    try:
        for v in (2, 3):
            kmv.set_tuning("symv_variant", v)
            assert kmv.symv_kernel_variant("s", "L", 5000, DUMMY, 5000) == v
    finally:
        kmv.set_tuning("symv_variant", 0)


def test_table_of_measured_settings():
    """host-only: every row of the compiled-in table is what the query returns inside its size range, holds legal
    tuning values, and the tuned_table key switches the table off"""
    text = open(os.path.join(ROOT, "paper_1410_1726_amd", "csrc", "kmv_tuned_table.inc")).read()
    rows = re.findall(r"\{'(\w)', '(\w)', (\d+), (\d+), ([-\d, ]+)\}", text)
    seen = set()
    for op, prec, lo, hi, vals in rows:
        lo, hi, vals = int(lo), int(hi), [int(v) for v in vals.split(",")]
        assert op in "NTLU" and prec in "sdcz" and 0 < lo < hi and len(vals) == len(kmv.TUNED_FIELDS)
        want = {f: v for f, v in zip(kmv.TUNED_FIELDS, vals) if v}
        assert want, "a row that sets nothing"
        for n in (lo, hi - 1):
            assert kmv.tuned_settings(prec, op, n) == want
        for r in range(lo, hi, max(1, (hi - lo) // 4)):          # ranges of one routine do not overlap
            assert (op, prec, r) not in seen
            seen.add((op, prec, r))
        try:
            for key, v in want.items():
                kmv.set_tuning(key, v)                            # raises on an illegal value
        finally:
            for key in want:
                kmv.set_tuning(key, 0)
    assert kmv.tuned_settings("d", "N", 7) is None                # far below every measured size
    with pytest.raises(ValueError):
        kmv.tuned_settings("q", "N", 4096)
    with pytest.raises(ValueError):
        kmv.tuned_settings("d", "X", 4096)
    if rows:
        op, prec, lo = rows[0][0], rows[0][1], int(rows[0][2])
        kmv.set_tuning("tuned_table", 1)
        try:
            assert kmv.tuned_settings(prec, op, lo) is None
        finally:
            kmv.set_tuning("tuned_table", 0)


def test_tuning_tool_grids_and_apply():
    """host-only parts of the tuning tool: the coarse and fine grids name valid keys and values, and a saved
    setting round-trips through apply()"""
    from paper_1410_1726_amd import tune
    keys = set(kmv.tuning_keys())
    for routine, m, n in (("dgemv_N", 4096, 4096), ("sgemv_T", 512, 9000), ("zhemv_L", 2048, 2048), ("dsymv_U", 20000, 20000)):
        coarse = tune._coarse_grid(routine, m, n)
        assert coarse and set(coarse) <= keys
        first = {key: vals[-1] for key, vals in coarse.items()}
        fine = tune._fine_grid(routine, first)
        assert set(fine) <= keys
        try:
            for grid in (coarse, fine):
                for key, vals in grid.items():
                    for v in vals:
                        kmv.set_tuning(key, v)          # raises on an illegal value
            tune.apply(first)
            assert all(kmv.get_tuning(key) == v for key, v in first.items())
            assert all(kmv.get_tuning(key) == 0 for key in keys - set(first))
        finally:
            for key in keys:
                kmv.set_tuning(key, 0)


def test_tuning_sweep_tool_is_importable():
    from paper_1410_1726_amd import tune
    assert tune.main([]) == 2          # prints its usage, touches no device


@pytest.mark.parametrize("prec", "sdcz")
def test_offset_argument_errors(prec):
    g, f = kmv.GEMV_OFFSET[prec], kmv.SYMV_OFFSET[prec]

    def gemv(trans="N", m=8, n=6, lda=8, offr=0, offc=0, incx=1, A=DUMMY):
        return g(trans, m, n, 1.0, A, lda, DUMMY, incx, 0.0, DUMMY, 1, offr, offc, workspace=NOWS, stream=0, check=False)

    def symv(uplo="L", n=8, lda=8, off=0, A=DUMMY):
        return f(uplo, n, 1.0, A, lda, DUMMY, 1, 0.0, DUMMY, 1, off, workspace=NOWS, stream=0, check=False)

    assert gemv(trans="X") == -1 and gemv(m=-1) == -2 and gemv(n=-1) == -3
    assert gemv(lda=7) == -6                    # the leading dimension is checked against the parent
    assert gemv(lda=7, offr=4) == -6
    assert gemv(offr=-1) == -12 and gemv(offr=9) == -12
    assert gemv(offc=-1) == -13 and gemv(offc=7) == -13
    assert gemv(incx=0) == -8
    assert gemv(offr=8) == 0 and gemv(offc=6) == 0          # empty block: nothing to do
    assert gemv(A=None) == kmv.ERR_NULL
    assert symv(uplo="N") == -1 and symv(n=-1) == -2 and symv(lda=7) == -5
    assert symv(off=-1) == -11 and symv(off=9) == -11
    assert symv(off=8) == 0
    assert symv(A=None) == kmv.ERR_NULL
    assert symv(n=5008, lda=5008, off=8) == kmv.ERR_WORKSPACE      # the two-kernel path needs its workspace


@pytest.mark.parametrize("prec", "sdcz")
def test_devscalars_argument_errors(prec):
    """argument checks come before anything is read or enqueued; the scalars are device addresses here and
    are never dereferenced on the host"""
    g, f = kmv.GEMV_DEVSCALARS[prec], kmv.SYMV_DEVSCALARS[prec]

    def gemv(trans="N", m=8, n=6, lda=8, incx=1, incy=1, alpha=DUMMY, beta=DUMMY, A=DUMMY):
        return g(trans, m, n, alpha, A, lda, DUMMY, incx, beta, DUMMY, incy, workspace=NOWS, stream=0, check=False)

    def symv(uplo="L", n=8, lda=8, incx=1, alpha=DUMMY, beta=DUMMY, A=DUMMY):
        return f(uplo, n, alpha, A, lda, DUMMY, incx, beta, DUMMY, 1, workspace=NOWS, stream=0, check=False)

    assert gemv(trans="X") == -1 and gemv(m=-1) == -2 and gemv(n=-1) == -3 and gemv(lda=7) == -6
    assert gemv(incx=0) == -8 and gemv(incy=0) == -11
    assert gemv(alpha=None) == kmv.ERR_NULL and gemv(beta=None) == kmv.ERR_NULL and gemv(A=None) == kmv.ERR_NULL
    assert gemv(m=0) == 0 and gemv(n=0) == 0
    assert gemv(incx=2) == kmv.ERR_WORKSPACE
    assert symv(uplo="N") == -1 and symv(n=-1) == -2 and symv(lda=7) == -5 and symv(incx=0) == -7
    assert symv(alpha=None) == kmv.ERR_NULL and symv(A=None) == kmv.ERR_NULL
    assert symv(n=0, lda=1) == 0
    assert symv(n=5000, lda=5000) == kmv.ERR_WORKSPACE


@pytest.mark.parametrize("prec", "sdcz")
def test_sytrd_panel_argument_errors(prec):
    f = kmv.SYTRD_PANEL[prec]

    def call(uplo="L", n=8, nb=4, lda=8, ldw=8, A=DUMMY, W=DUMMY):
        return f(uplo, n, nb, A, lda, DUMMY, DUMMY, W, ldw, workspace=NOWS, stream=0, check=False)

    assert call(uplo="X") == -1 and call(uplo="U") == kmv.ERR_WORKSPACE
    assert call(n=-1) == -2
    assert call(nb=-1) == -3 and call(nb=9) == -3
    assert call(lda=7) == -5 and call(ldw=7) == -9
    assert call(n=0, nb=0, lda=1, ldw=1) == 0 and call(nb=0) == 0
    assert call(A=None) == kmv.ERR_NULL and call(W=None) == kmv.ERR_NULL
    assert call() == kmv.ERR_WORKSPACE
    need = kmv.sytrd_panel_workspace_bytes(prec, 4096, 64)
    assert need >= kmv.symv_workspace_bytes(prec, "L", 4095)
    b = {"s": 4, "d": 8, "c": 8, "z": 16}[prec]
    assert need >= kmv.symv_workspace_bytes(prec, "L", 4095) + 64 * 2 * 64 * b      # plus the panel's own partial sums
    assert kmv.sytrd_panel_workspace_bytes("q", 64, 8) == 0 and kmv.sytrd_panel_workspace_bytes(prec, 0, 0) == 0


@pytest.mark.parametrize("prec", "sdcz")
def test_strided_batched_argument_errors(prec):
    g, f = kmv.GEMV_STRIDED_BATCHED[prec], kmv.SYMV_STRIDED_BATCHED[prec]

    def gemv(trans="N", m=8, n=6, lda=8, sA=48, incx=1, sx=6, incy=1, sy=8, batch=3, A=DUMMY):
        return g(trans, m, n, 1.0, A, lda, sA, DUMMY, incx, sx, 0.0, DUMMY, incy, sy, batch, stream=0, check=False)

    def symv(uplo="L", n=8, lda=8, sA=64, incx=1, sx=8, incy=1, sy=8, batch=3, A=DUMMY):
        return f(uplo, n, 1.0, A, lda, sA, DUMMY, incx, sx, 0.0, DUMMY, incy, sy, batch, stream=0, check=False)

    assert gemv(trans="Q") == -1 and gemv(m=-1) == -2 and gemv(n=-1) == -3 and gemv(lda=7) == -6
    assert gemv(sA=-1) == -7 and gemv(incx=2) == -9 and gemv(sx=-1) == -10 and gemv(incy=0) == -13
    assert gemv(sy=7) == -14 and gemv(incy=2, sy=14) == -14 and gemv(sy=-8) == -14
    assert gemv(sy=0, batch=1, A=None) == kmv.ERR_NULL       # a single member may have any stride
    assert gemv(batch=-1) == -15 and gemv(batch=0) == 0 and gemv(m=0) == 0
    assert gemv(A=None) == kmv.ERR_NULL
    assert symv(uplo="X") == -1 and symv(n=-1) == -2 and symv(lda=7) == -5 and symv(sA=-1) == -6
    assert symv(incx=-1) == -8 and symv(sx=-1) == -9 and symv(incy=0) == -12 and symv(sy=7) == -13
    assert symv(batch=-1) == -14 and symv(batch=0) == 0 and symv(n=0, lda=1) == 0
    assert symv(A=None) == kmv.ERR_NULL


@pytest.mark.parametrize("prec", "sdcz")
def test_gebrd_panel_argument_errors(prec):
    f = kmv.GEBRD_PANEL[prec]

    def call(m=8, n=6, nb=4, lda=8, ldx=8, ldy=6, A=DUMMY, X=DUMMY):
        return f(m, n, nb, A, lda, DUMMY, DUMMY, DUMMY, DUMMY, X, ldx, DUMMY, ldy, workspace=NOWS, stream=0, check=False)

    assert call(m=-1) == -1
    assert call(n=-1) == -2
    assert call(nb=-1) == -3 and call(nb=7) == -3 and call(m=5, n=9, lda=8, ldx=8, ldy=9, nb=6) == -3   # nb <= min(m, n)
    assert call(m=5, n=9, ldy=9, nb=5) == kmv.ERR_WORKSPACE    # more columns than rows: lower bidiagonal form
    assert call(lda=7) == -5 and call(ldx=7) == -11 and call(ldy=5) == -13
    assert call(nb=0) == 0 and call(m=0, n=0, nb=0, lda=1, ldx=1, ldy=1) == 0
    assert call(A=None) == kmv.ERR_NULL and call(X=None) == kmv.ERR_NULL
    assert call() == kmv.ERR_WORKSPACE
    need = kmv.gebrd_panel_workspace_bytes(prec, 4096, 4096, 64)
    assert need >= kmv.gemv_workspace_bytes(prec, "T", 4096, 4095)
    assert kmv.gebrd_panel_workspace_bytes("q", 64, 64, 8) == 0 and kmv.gebrd_panel_workspace_bytes(prec, 8, 9, 2) > 0
    if prec in "cz":      # room for the row copy and the three conjugated short rows besides the products' workspace
        esz = {"c": 8, "z": 16}[prec]
        assert need >= kmv.gemv_workspace_bytes(prec, "C", 4096, 4095) + (4096 + 3 * 64) * esz


def test_plain_c_program_links_and_calls_the_library(tmp_path):
    """the header is C99 and the symbols have C linkage: a C program built with gcc runs the host-only calls"""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.join(root, "paper_1410_1726_amd")
    exe = str(tmp_path / "abi_check")
    build = subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-I", os.path.join(root, "include"),
                            os.path.join(root, "tests", "c", "abi_check.c"), "-o", exe, "-L", libdir, "-lkmv",
                            f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), run.stdout + run.stderr


@pytest.mark.parametrize("prec", "sdcz")
def test_pointer_array_batched_argument_errors(prec):
    g, sv = kmv.GEMV_BATCHED[prec], kmv.SYMV_BATCHED[prec]

    def gemv(trans="N", m=8, n=6, lda=8, incx=1, incy=1, batch=2, A=DUMMY, y=DUMMY):
        return g(trans, m, n, 1.0, A, lda, DUMMY, incx, 0.0, y, incy, batch, stream=0, check=False)

    def symv(uplo="L", n=8, lda=8, incx=1, incy=1, batch=2, A=DUMMY):
        return sv(uplo, n, 1.0, A, lda, DUMMY, incx, 0.0, DUMMY, incy, batch, stream=0, check=False)

    assert gemv(trans="X") == -1 and gemv(m=-1) == -2 and gemv(n=-1) == -3 and gemv(lda=7) == -6
    assert gemv(incx=2) == -8 and gemv(incy=0) == -11 and gemv(batch=-1) == -12
    assert gemv(batch=0) == 0 and gemv(m=0, lda=1) == 0
    assert gemv(A=None) == kmv.ERR_NULL and gemv(y=None) == kmv.ERR_NULL
    assert symv(uplo="X") == -1 and symv(n=-1) == -2 and symv(lda=7) == -5
    assert symv(incx=-1) == -7 and symv(incy=0) == -10 and symv(batch=-1) == -11
    assert symv(batch=0) == 0 and symv(n=0, lda=1) == 0 and symv(A=None) == kmv.ERR_NULL


def test_tuning_tool_table_rows():
    """host-only: the size classes of the table-saving mode and the text of a saved row"""
    from paper_1410_1726_amd import tune
    assert tune._size_class(16384, 16) == (15360, 17409) and tune._size_class(4096, 64) == (4032, 4161)
    row = tune._row_text("zhemv_U", 8192, 64, {"symv_variant": 2, "symv_tiles_per_wave": 1, "wg_target": 256})
    assert row.strip().startswith("{'U', 'z', 8064, 8321, 0, 0, 0, 2, 1, 0, 256}")
    assert tune._row_text("cgemv_C", 4096, 16, {"gemv_t_splits": 16}).strip().startswith("{'T', 'c', 3840, 4353, 0, 0, 16, 0, 0, 0, 0}")
    assert tune._op("dgemv_N") == "N" and tune._op("sgemv_T") == "T" and tune._op("dsymv_L") == "L"
    assert len(tune.ROW_FIELDS) == len(kmv.TUNED_FIELDS) and tuple(tune.ROW_FIELDS) == tuple(kmv.TUNED_FIELDS)
    assert len(tune.TABLE_ROUTINES) == 16 and len(set(tune.TABLE_ROUTINES)) == 16


def test_tuning_tool_writes_rows(tmp_path):
    from paper_1410_1726_amd import tune
    rows = [tune._row_text("sgemv_N", 4096, 64, {"gemv_n_row_tiles": 2})]
    path = tune.write_rows(rows, str(tmp_path / "table.inc"))
    text = open(path).read()
    assert text.startswith("// Written by") and "{'N', 's', 4032, 4161, 0, 2, 0, 0, 0, 0, 0}" in text


def test_no_kernel_spills_registers():
    """the build collects the compiler's per-kernel resource figures; no kernel of the library may use scratch
    memory (register spills: a spilling kernel still computes correctly, only several times slower), and the
    report must cover the kernels of every source file"""
    from paper_1410_1726_amd import build
    if not os.path.exists(build.RESOURCES) or os.path.getmtime(build.RESOURCES) + 2 < os.path.getmtime(kmv.LIB_PATH):
        pytest.skip("no resource report for this library (built without paper_1410_1726_amd.build)")
    rows = [ln.split() for ln in open(build.RESOURCES)]
    assert len(rows) > 500 and all(len(r) == 4 for r in rows)
    for family in ("gemv_n_kernel", "gemv_t_kernel", "symv_balanced_kernel", "symv_reduce_kernel", "bd_update_kernel",
                   "panel_reflector_kernel", "reduce_kernel"):
        assert any(family in r[0] for r in rows), family
    spilling = [(r[0], int(r[3])) for r in rows if int(r[3]) > 0]
    assert not spilling, spilling
    assert all(int(r[1]) <= 512 and int(r[2]) <= 160 * 1024 for r in rows)
