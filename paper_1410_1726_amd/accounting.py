"""Flop, byte and roofline accounting of the paper's performance model.

Everything here restates Section 7 ("Performance Model"):

* flop count of ``y = alpha*A*x + beta*y`` per output element: a length-``k``
  dot product plus the two scalings and the final addition, i.e. ``2k + 2``
  real flops for real data; a complex addition is 2 real flops and a complex
  multiplication 6, which gives ``8k + 12`` per output element;
* ideal byte count: the matrix once, ``x`` once, ``y`` read and written once;
  a symmetric / Hermitian product reads one triangle including the diagonal;
* operational intensity ``I = flops / bytes`` (Table "Operational
  intensities") and the sustained peak ``R = I * B`` (Eq. roofline), where the
  paper takes ``B`` from a STREAM measurement.

The rectangular generalisation (``m != n``) keeps the same per-element counts.
"""
from __future__ import annotations

ELEM_BYTES = {"s": 4, "d": 8, "c": 8, "z": 16}
IS_COMPLEX = {"s": False, "d": False, "c": True, "z": True}

#: published peak HBM bandwidth of one MI355X in GB/s (the roofline ``peak``)
MI355X_HBM_GBS = 8000.0


def _dims(op: str, m: int, n: int):
    """(length of y, length of the dot products, matrix elements read)."""
    op = op.lower()
    if op == "gemv_n":
        return m, n, m * n
    if op in ("gemv_t", "gemv_c"):
        return n, m, m * n
    if op in ("symv_l", "symv_u", "hemv_l", "hemv_u", "symv", "hemv"):
        if m != n:
            raise ValueError("symmetric product needs m == n")
        return n, n, n * (n + 1) // 2
    raise ValueError(op)


def flops(op: str, prec: str, m: int, n: int) -> int:
    """Real floating point operations of one call (Section 7)."""
    leny, k, _ = _dims(op, m, n)
    if IS_COMPLEX[prec]:
        return leny * (8 * k + 12)
    return leny * (2 * k + 2)


def algorithmic_bytes(op: str, prec: str, m: int, n: int) -> int:
    """Ideal memory traffic of one call in bytes (Section 7)."""
    leny, k, nmat = _dims(op, m, n)
    return (nmat + k + 2 * leny) * ELEM_BYTES[prec]


def intensity(op: str, prec: str, m: int, n: int) -> float:
    """Operational intensity in flop/byte (Table "Operational intensities")."""
    return flops(op, prec, m, n) / algorithmic_bytes(op, prec, m, n)


def asymptotic_intensity(op: str, prec: str) -> float:
    """Large-n limit of :func:`intensity` for a square matrix."""
    per_elem = 8.0 if IS_COMPLEX[prec] else 2.0
    share = 0.5 if op.lower().startswith(("symv", "hemv")) else 1.0
    return per_elem / (share * ELEM_BYTES[prec])


def roofline_gflops(op: str, prec: str, bandwidth_gbs: float) -> float:
    """Sustained peak ``R = I * B`` in Gflop/s with the asymptotic intensity
    (Eq. roofline and Table "Estimated sustained peak performances")."""
    return asymptotic_intensity(op, prec) * bandwidth_gbs


def rates(op: str, prec: str, m: int, n: int, seconds: float) -> dict:
    """Gflop/s, GB/s and fraction of the MI355X HBM peak for one timed call."""
    f, b = flops(op, prec, m, n), algorithmic_bytes(op, prec, m, n)
    gbs = b / seconds / 1e9
    return {"gflops": f / seconds / 1e9, "gbs": gbs, "frac_hbm_peak": gbs / MI355X_HBM_GBS}
