"""Seeded synthetic inputs for the GEMV / SYMV / HEMV tests and benchmark.

This module holds NO arithmetic of the method: it only fills buffers with
random numbers and poison values.  It is the one module that both the GPU
tests / benchmark and the CPU-oracle tests may share, so that both sides see
the same bytes.

The workloads follow the paper's experiments (Section 8.2: square dense
matrices swept over n in the four precisions; sub-blocks of a large parent
matrix obtained by skipping leading rows and columns): dense column-major
matrices with i.i.d. entries, uniform on [-1, 1] or standard normal, complex
entries with independent real and imaginary parts.

Storage convention: a column-major ``rows x cols`` matrix with leading
dimension ``lda`` is returned as a torch tensor of shape ``(cols, lda)``
(row-major), i.e. ``buf[j, i]`` is element (i, j).  ``buf.data_ptr()`` is the
BLAS pointer ``A``; ``buf.numpy()`` (flattened) is the flat buffer the oracle
takes together with ``lda``.
"""
from __future__ import annotations

import torch

TORCH_DTYPES = {
    "s": torch.float32,
    "d": torch.float64,
    "c": torch.complex64,
    "z": torch.complex128,
}
ELEM_BYTES = {"s": 4, "d": 8, "c": 8, "z": 16}


def _generator(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def fill_random(t: torch.Tensor, dist: str, gen: torch.Generator) -> torch.Tensor:
    """Fill ``t`` in place: 'uniform' = U[-1,1], 'normal' = N(0,1),
    'smallint' = integers in {-3..3} (exact in every summation order)."""
    r = torch.view_as_real(t) if t.is_complex() else t
    if dist == "uniform":
        r.uniform_(-1.0, 1.0, generator=gen)
    elif dist == "normal":
        r.normal_(0.0, 1.0, generator=gen)
    elif dist == "smallint":
        if not r.is_contiguous():
            raise ValueError("smallint needs a contiguous tensor")
        flat = r.reshape(-1)
        step = 1 << 26   # slabs, so no temporary as large as the tensor is made
        for s in range(0, flat.numel(), step):
            e = min(flat.numel(), s + step)
            flat[s:e] = torch.randint(-3, 4, (e - s,), generator=gen, device=t.device).to(r.dtype)
    else:
        raise ValueError(dist)
    return t


def matrix(prec: str, rows: int, cols: int, lda: int | None = None, *, dist: str = "uniform",
           seed: int = 0, device="cpu", pad_nan: bool = True) -> torch.Tensor:
    """Column-major ``rows x cols`` matrix, returned as a ``(cols, lda)`` tensor.
    Rows ``rows..lda-1`` of every column (the padding) are NaN when ``pad_nan``."""
    lda = max(1, rows) if lda is None else int(lda)
    if lda < max(1, rows):
        raise ValueError("lda < rows")
    buf = torch.empty((cols, lda), dtype=TORCH_DTYPES[prec], device=device)
    fill_random(buf, dist, _generator(seed * 1000 + 0, device))
    if pad_nan and lda > rows and cols:
        buf[:, rows:] = float("nan")
    return buf


def vector(prec: str, length: int, inc: int = 1, *, dist: str = "uniform", seed: int = 0,
           which: int = 1, device="cpu", gap_value: float | None = None) -> torch.Tensor:
    """Strided vector buffer of ``1 + (length-1)*|inc|`` elements.  ``which``
    picks the random stream (1 = x, 2 = y).  ``gap_value`` (if given) fills the
    skipped positions of a strided vector, e.g. NaN as a canary."""
    ext = 0 if length == 0 else 1 + (length - 1) * abs(inc)
    buf = torch.empty((ext,), dtype=TORCH_DTYPES[prec], device=device)
    fill_random(buf, dist, _generator(seed * 1000 + which, device))
    if gap_value is not None and abs(inc) > 1 and ext:
        keep = buf[:: abs(inc)].clone()
        buf.fill_(gap_value)
        buf[:: abs(inc)] = keep
    return buf


def poison_triangle(buf: torch.Tensor, n: int, uplo: str, *, real_diag: bool = True) -> torch.Tensor:
    """Overwrite the triangle that ``uplo`` does NOT reference with NaN (strictly
    above the diagonal for 'L', strictly below for 'U'), in place, and make the
    diagonal real for complex matrices when ``real_diag``.  ``buf`` is the
    ``(cols, lda)`` storage of an ``n x n`` column-major matrix."""
    lower = uplo.upper() == "L"
    step = 2048
    nan = float("nan")
    for j0 in range(0, n, step):
        j1 = min(n, j0 + step)
        jj = torch.arange(j0, j1, device=buf.device).unsqueeze(1)        # column index
        # rows overlapping the diagonal band of these columns
        ii = torch.arange(j0, j1, device=buf.device).unsqueeze(0)        # row index
        blk = buf[j0:j1, j0:j1]
        bad = (ii < jj) if lower else (ii > jj)
        blk[bad] = nan
        if lower:
            if j0 > 0:
                buf[j0:j1, :j0] = nan      # rows above the band, i < j
        else:
            if j1 < n:
                buf[j0:j1, j1:n] = nan     # rows below the band, i > j
    if real_diag and buf.is_complex() and n:
        d = torch.arange(n, device=buf.device)
        buf[d, d] = buf[d, d].real.to(buf.dtype)
    return buf


def sample_indices(length: int, count: int, seed: int = 0) -> torch.Tensor:
    """``count`` distinct output indices in [0, length): both ends, the
    neighbourhoods of tile boundaries, and seeded random picks in between."""
    if length <= count:
        return torch.arange(length, dtype=torch.int64)
    g = _generator(seed * 1000 + 7, "cpu")
    fixed = [0, 1, length - 1, length - 2, length // 2, 63, 64, 65, 127, 128, 129, 255, 256, 257]
    fixed = [i for i in fixed if 0 <= i < length]
    rnd = torch.randint(0, length, (count,), generator=g).tolist()
    out, seen = [], set()
    for i in fixed + rnd:
        if i not in seen:
            seen.add(i)
            out.append(i)
        if len(out) == count:
            break
    return torch.tensor(sorted(out), dtype=torch.int64)


def vec_extent(length: int, inc: int) -> int:
    return 0 if length == 0 else 1 + (length - 1) * abs(inc)


def ceil_div(a: int, b: int) -> int:
    return -(-a // b)


__all__ = [
    "TORCH_DTYPES", "ELEM_BYTES", "matrix", "vector", "poison_triangle", "fill_random",
    "sample_indices", "vec_extent", "ceil_div",
]
