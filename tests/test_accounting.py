"""Accounting pins (no GPU): the flop / byte / roofline helpers reproduce the
numbers the paper prints in Section 7 (tables stored under tests/golden/)."""
import os

import pytest

from paper_1410_1726_amd import accounting as acc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append(line.split())
    return out


def test_flop_and_byte_counts_match_the_model():
    # Section 7: real 2n^2 + 2n flops, complex 8n^2 + 12n; GEMV bytes (n^2 + 3n) b,
    # SYMV/HEMV bytes (n(n+1)/2 + 3n) b
    for n in (1, 7, 1024, 49152):
        for p, b in acc.ELEM_BYTES.items():
            f = 8 * n * n + 12 * n if p in "cz" else 2 * n * n + 2 * n
            for op in ("gemv_n", "gemv_t", "symv_l", "hemv_u"):
                assert acc.flops(op, p, n, n) == f
            assert acc.algorithmic_bytes("gemv_n", p, n, n) == (n * n + 3 * n) * b
            assert acc.algorithmic_bytes("gemv_t", p, n, n) == (n * n + 3 * n) * b
            assert acc.algorithmic_bytes("symv_l", p, n, n) == (n * (n + 1) // 2 + 3 * n) * b
    # rectangular generalisation keeps the per-element counts
    assert acc.flops("gemv_n", "d", 10, 20) == 10 * (2 * 20 + 2)
    assert acc.flops("gemv_t", "d", 10, 20) == 20 * (2 * 10 + 2)
    assert acc.algorithmic_bytes("gemv_t", "s", 10, 20) == (200 + 10 + 40) * 4
    with pytest.raises(ValueError):
        acc.flops("symv_l", "d", 3, 4)


def test_operational_intensities_table():
    for p, gemv, symv in rows("op_intensity.txt"):
        assert acc.asymptotic_intensity("gemv_n", p) == pytest.approx(float(gemv), abs=5e-3)
        assert acc.asymptotic_intensity("hemv_l" if p in "cz" else "symv_l", p) == pytest.approx(float(symv), abs=5e-3)
        # the exact ratio tends to the printed value for large n
        n = 1 << 16
        assert acc.intensity("gemv_t", p, n, n) == pytest.approx(float(gemv), rel=1e-3)
        assert acc.intensity("symv_u", p, n, n) == pytest.approx(float(symv), rel=1e-3)


def test_sustained_peak_table_k20c():
    table = rows("sustained_perf_k20c.txt")
    bw = float(table[0][1])
    stream = {r[0]: r[1:] for r in rows("stream_k20c.txt")}
    assert max(float(v) for v in stream["off"]) == bw      # the paper's sustained bandwidth
    assert float(stream["theoretical"][0]) == pytest.approx(2.6 * 40 * 2)
    inconsistent = 0
    for p, gemv, symv, ok in table[1:]:
        assert acc.roofline_gflops("gemv_n", p, bw) == pytest.approx(float(gemv), abs=6e-3)
        r = acc.roofline_gflops("symv_l", p, bw)
        if ok == "1":
            assert r == pytest.approx(float(symv), abs=6e-3)
        else:
            inconsistent += 1
            assert r == pytest.approx(2.0 * bw) and abs(r - float(symv)) > 1.0
    assert inconsistent == 1


def test_rates_helper():
    n = 16384
    sec = acc.algorithmic_bytes("gemv_n", "d", n, n) / 6.4e12
    r = acc.rates("gemv_n", "d", n, n, sec)
    assert r["gbs"] == pytest.approx(6400.0)
    assert r["frac_hbm_peak"] == pytest.approx(0.8)
    assert r["gflops"] == pytest.approx(acc.flops("gemv_n", "d", n, n) / sec / 1e9)
