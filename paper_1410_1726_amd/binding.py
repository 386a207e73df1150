"""Thin ctypes binding of ``libkmv.so`` (argument marshalling only).

Every function has the name and argument order of its C entry point in
``include/kmv.h`` minus the ``kmv_`` prefix.  Matrices and vectors are torch
tensors on the GPU (only ``data_ptr()`` is used, so views that point into the
middle of a larger matrix work as sub-block pointers) or raw integer device
addresses; the workspace and the stream come from torch as well.  No step of
a product runs in Python or in torch: if the HIP library is missing the import
of this module fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkmv.so")

ERR_WORKSPACE = 1001
ERR_NULL = 1002
ERR_HIP = 2000


class KmvError(RuntimeError):
    def __init__(self, name, code):
        super().__init__(f"kmv_{name} returned {code}")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1410_1726_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ch, ci, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_char, ctypes.c_int, ctypes.c_size_t
    gemv_args = [ch, i64, i64, vp, vp, i64, vp, i64, vp, vp, i64, vp, sz, vp]
    symv_args = [ch, i64, vp, vp, i64, vp, i64, vp, vp, i64, vp, sz, vp]
    for p in "sdcz":
        f = getattr(lib, f"kmv_{p}gemv")
        f.argtypes, f.restype = gemv_args, ci
    for name in ("ssymv", "dsymv", "chemv", "zhemv", "csymv", "zsymv"):
        f = getattr(lib, f"kmv_{name}")
        f.argtypes, f.restype = symv_args, ci
    gemv_off_args = gemv_args[:11] + [i64, i64] + gemv_args[11:]
    symv_off_args = symv_args[:10] + [i64] + symv_args[10:]
    for p_ in "sdcz":
        f = getattr(lib, f"kmv_{p_}gemv_offset")
        f.argtypes, f.restype = gemv_off_args, ci
        f = getattr(lib, f"kmv_{p_}{'hemv' if p_ in 'cz' else 'symv'}_offset")
        f.argtypes, f.restype = symv_off_args, ci
    for p_ in "cz":                      # complex symmetric forms
        getattr(lib, f"kmv_{p_}symv_offset").argtypes = symv_off_args
        getattr(lib, f"kmv_{p_}symv_devscalars").argtypes = symv_args
        for suffix in ("offset", "devscalars", "strided_batched"):
            getattr(lib, f"kmv_{p_}symv_{suffix}").restype = ci
    for p_ in "sdcz":
        f = getattr(lib, f"kmv_{p_}gemv_devscalars")
        f.argtypes, f.restype = gemv_args, ci
        f = getattr(lib, f"kmv_{p_}{'hemv' if p_ in 'cz' else 'symv'}_devscalars")
        f.argtypes, f.restype = symv_args, ci
    for name in ("ssytrd_panel", "dsytrd_panel", "chetrd_panel", "zhetrd_panel"):
        f = getattr(lib, f"kmv_{name}")
        f.argtypes, f.restype = [ch, i64, i64, vp, i64, vp, vp, vp, i64, vp, sz, vp], ci
    for p_ in "sdcz":
        f = getattr(lib, f"kmv_{p_}gebrd_panel")
        f.argtypes, f.restype = [i64, i64, i64, vp, i64, vp, vp, vp, vp, vp, i64, vp, i64, vp, sz, vp], ci
    lib.kmv_gebrd_panel_workspace_bytes.argtypes, lib.kmv_gebrd_panel_workspace_bytes.restype = [ch, i64, i64, i64], sz
    lib.kmv_sytrd_panel_workspace_bytes.argtypes, lib.kmv_sytrd_panel_workspace_bytes.restype = [ch, i64, i64], sz
    gemv_b_args = [ch, i64, i64, vp, vp, i64, i64, vp, i64, i64, vp, vp, i64, i64, i64, vp]
    symv_b_args = [ch, i64, vp, vp, i64, i64, vp, i64, i64, vp, vp, i64, i64, i64, vp]
    for p_ in "sdcz":
        f = getattr(lib, f"kmv_{p_}gemv_strided_batched")
        f.argtypes, f.restype = gemv_b_args, ci
        f = getattr(lib, f"kmv_{p_}{'hemv' if p_ in 'cz' else 'symv'}_strided_batched")
        f.argtypes, f.restype = symv_b_args, ci
    for p_ in "cz":
        getattr(lib, f"kmv_{p_}symv_strided_batched").argtypes = symv_b_args
    gemv_p_args = [ch, i64, i64, vp, vp, i64, vp, i64, vp, vp, i64, i64, vp]
    symv_p_args = [ch, i64, vp, vp, i64, vp, i64, vp, vp, i64, i64, vp]
    for p_ in "sdcz":
        f = getattr(lib, f"kmv_{p_}gemv_batched")
        f.argtypes, f.restype = gemv_p_args, ci
    for name in ("ssymv", "dsymv", "chemv", "zhemv", "csymv", "zsymv"):
        f = getattr(lib, f"kmv_{name}_batched")
        f.argtypes, f.restype = symv_p_args, ci
    lib.kmv_gemv_workspace_bytes.argtypes, lib.kmv_gemv_workspace_bytes.restype = [ch, ch, i64, i64], sz
    lib.kmv_symv_workspace_bytes.argtypes, lib.kmv_symv_workspace_bytes.restype = [ch, ch, i64], sz
    lib.kmv_partition.argtypes = [i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.kmv_partition.restype = None
    lib.kmv_stream_probe.argtypes, lib.kmv_stream_probe.restype = [ci, i64, vp, vp, vp, vp, vp], ci
    lib.kmv_set_tuning.argtypes, lib.kmv_set_tuning.restype = [ctypes.c_char_p, i64], ci
    lib.kmv_get_tuning.argtypes, lib.kmv_get_tuning.restype = [ctypes.c_char_p], i64
    lib.kmv_tuning_keys.restype = ctypes.c_char_p
    lib.kmv_tuned_settings.argtypes = [ctypes.c_char, ctypes.c_char, i64, ctypes.POINTER(ctypes.c_int64)]
    lib.kmv_tuned_settings.restype = ctypes.c_int
    lib.kmv_symv_kernel_variant.argtypes = [ctypes.c_char, ctypes.c_char, i64, ctypes.c_void_p, i64]
    lib.kmv_symv_kernel_variant.restype = ctypes.c_int
    lib.kmv_symv_shares.argtypes = [ctypes.c_char, ctypes.c_char, i64, ci, ci, ci, i64, ci, ci, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(i64)]
    lib.kmv_symv_shares.restype = ci
    lib.kmv_dsymv_static.argtypes = [ctypes.c_char, i64, ctypes.c_void_p, ctypes.c_void_p, i64, ctypes.c_void_p, i64,
                                     ctypes.c_void_p, ctypes.c_void_p, i64, ctypes.c_void_p]
    lib.kmv_dsymv_static.restype = ci
    lib.kmv_version.restype = ctypes.c_char_p
    return lib


lib = _load()

_CT = {"s": ctypes.c_float, "d": ctypes.c_double}
_TORCH = {"s": torch.float32, "d": torch.float64, "c": torch.complex64, "z": torch.complex128}


def _scalar(prec, v):
    """Host storage of alpha / beta in the element type of the routine."""
    if prec in "sd":
        return (_CT[prec] * 1)(float(v))
    v = complex(v)
    return ((ctypes.c_float if prec == "c" else ctypes.c_double) * 2)(v.real, v.imag)


def _ptr(t, prec=None):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if prec is not None and t.dtype != _TORCH[prec]:
        raise TypeError(f"expected {_TORCH[prec]}, got {t.dtype}")
    if not t.is_cuda:
        raise ValueError("kmv works on device memory only")
    return ctypes.c_void_p(t.data_ptr())


_ws_cache: dict = {}


def _stream_handle(stream, device=None) -> int:
    if stream is None:
        stream = torch.cuda.current_stream(device)
    return int(stream if isinstance(stream, int) else stream.cuda_stream)


def workspace(nbytes: int, device=None, stream=None) -> torch.Tensor:
    """Grow-only byte buffer per (device, stream) (torch owns the memory).  Products enqueued on different
    streams run concurrently and must not share partial sums, so each stream gets a buffer of its own; a
    buffer that has to grow is replaced only after the device has finished the work that may still use it.
    A caller that passes its own workspace must keep to the same rule: one workspace per stream."""
    dev = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
    key = (dev, _stream_handle(stream, dev))
    buf = _ws_cache.get(key)
    if buf is None or buf.numel() < nbytes:
        if buf is not None:
            torch.cuda.synchronize(dev)
        buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=dev)
        _ws_cache[key] = buf
    return buf


_cached_workspace = workspace   # the wrappers below take a parameter called `workspace`


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)


_ws_bytes_cache: dict = {}


def gemv_workspace_bytes(prec, trans, m, n) -> int:
    key = ("g", prec, trans, m, n)
    v = _ws_bytes_cache.get(key)
    if v is None:
        v = _ws_bytes_cache[key] = int(lib.kmv_gemv_workspace_bytes(prec.encode(), trans.encode(), m, n))
    return v


def symv_workspace_bytes(prec, uplo, n) -> int:
    key = ("s", prec, uplo, n)
    v = _ws_bytes_cache.get(key)
    if v is None:
        v = _ws_bytes_cache[key] = int(lib.kmv_symv_workspace_bytes(prec.encode(), uplo.encode(), n))
    return v


def _ws_args(workspace_, need, y, stream=None):
    """(pointer, bytes) of the workspace: None -> the stream's cached torch buffer of `need()`
    bytes, a tensor -> its storage, a (pointer, bytes) tuple -> as given."""
    if workspace_ is None:
        workspace_ = workspace(need(), None if isinstance(y, int) else y.device, stream)
    if isinstance(workspace_, tuple):
        return workspace_
    return workspace_.data_ptr(), workspace_.numel() * workspace_.element_size()


def _gemv(prec, trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace_=None, stream=None, check=True):
    wsp, wsb = _ws_args(workspace_, lambda: gemv_workspace_bytes(
        prec, trans if trans in tuple("NnTtCc") else "N", max(m, 0), max(n, 0)), y, stream)
    al, be = _scalar(prec, alpha), _scalar(prec, beta)
    rc = getattr(lib, f"kmv_{prec}gemv")(trans.encode(), m, n, al, _ptr(A, prec), lda, _ptr(x, prec), incx, be,
                                         _ptr(y, prec), incy, ctypes.c_void_p(wsp), wsb, _stream(stream))
    if check and rc != 0:
        raise KmvError(f"{prec}gemv", rc)
    return rc


def _symv(name, prec, uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace_=None, stream=None, check=True):
    wsp, wsb = _ws_args(workspace_, lambda: symv_workspace_bytes(
        prec, uplo if uplo in tuple("LlUu") else "L", max(n, 0)), y, stream)
    al, be = _scalar(prec, alpha), _scalar(prec, beta)
    rc = getattr(lib, f"kmv_{name}")(uplo.encode(), n, al, _ptr(A, prec), lda, _ptr(x, prec), incx, be,
                                     _ptr(y, prec), incy, ctypes.c_void_p(wsp), wsb, _stream(stream))
    if check and rc != 0:
        raise KmvError(name, rc)
    return rc


def sgemv(trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _gemv("s", trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


def dgemv(trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _gemv("d", trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


def cgemv(trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _gemv("c", trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


def zgemv(trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _gemv("z", trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


def ssymv(uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _symv("ssymv", "s", uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


def dsymv(uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _symv("dsymv", "d", uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


def dsymv_static(uplo, n, alpha, A, lda, x, incx, beta, y, incy, stream=None, check=True):
    """kmv_dsymv_static: DSYMV with the library's own static device array as workspace (no allocation anywhere, not
    even in this wrapper); products that need more than the array holds are refused with ERR_WORKSPACE."""
    rc = lib.kmv_dsymv_static(uplo.encode(), n, _scalar("d", alpha), _ptr(A, "d"), lda, _ptr(x, "d"), incx,
                              _scalar("d", beta), _ptr(y, "d"), incy, _stream(stream))
    if check and rc != 0:
        raise KmvError("dsymv_static", rc)
    return rc


def chemv(uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _symv("chemv", "c", uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


def zhemv(uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _symv("zhemv", "z", uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


class Prepared:
    """One routine call with every argument already marshalled: calling the object
    only makes the foreign call (for loops that repeat a product, where the
    per-call Python work of the plain wrappers would exceed the kernel time).
    Holds references to the tensors (and the workspace) so that the addresses stay
    valid; the stream is fixed at preparation time."""

    __slots__ = ("_fn", "_args", "_keep", "name")

    def __init__(self, name, fn, args, keep):
        self.name, self._fn, self._args, self._keep = name, fn, args, keep

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != 0:
            raise KmvError(self.name, rc)


def prepare_gemv(prec, trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None) -> Prepared:
    if workspace is None:
        workspace = _cached_workspace(gemv_workspace_bytes(prec, trans, max(m, 0), max(n, 0)),
                                      None if isinstance(y, int) else y.device, stream)
    wsp, wsb = _ws_args(workspace, None, y, stream)
    al, be = _scalar(prec, alpha), _scalar(prec, beta)
    args = (trans.encode(), m, n, al, _ptr(A, prec), lda, _ptr(x, prec), incx, be, _ptr(y, prec), incy,
            ctypes.c_void_p(wsp), wsb, _stream(stream))
    return Prepared(f"{prec}gemv", getattr(lib, f"kmv_{prec}gemv"), args, (A, x, y, workspace))


def prepare_symv(prec, uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None,
                 complex_symmetric=False) -> Prepared:
    """`complex_symmetric` (prec c,z) prepares csymv / zsymv instead of chemv / zhemv."""
    if complex_symmetric and prec not in "cz":
        raise ValueError("complex_symmetric needs prec 'c' or 'z'")
    name = f"{prec}{'hemv' if prec in 'cz' and not complex_symmetric else 'symv'}"
    if workspace is None:
        workspace = _cached_workspace(symv_workspace_bytes(prec, uplo, max(n, 0)),
                                      None if isinstance(y, int) else y.device, stream)
    wsp, wsb = _ws_args(workspace, None, y, stream)
    al, be = _scalar(prec, alpha), _scalar(prec, beta)
    args = (uplo.encode(), n, al, _ptr(A, prec), lda, _ptr(x, prec), incx, be, _ptr(y, prec), incy,
            ctypes.c_void_p(wsp), wsb, _stream(stream))
    return Prepared(name, getattr(lib, f"kmv_{name}"), args, (A, x, y, workspace))


def csymv(uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _symv("csymv", "c", uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


def zsymv(uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
    return _symv("zsymv", "z", uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace, stream, check)


def _gemv_offset(prec):
    def call(trans, m, n, alpha, A, lda, x, incx, beta, y, incy, offset_r, offset_c, workspace=None, stream=None,
             check=True):
        wsp, wsb = _ws_args(workspace, lambda: gemv_workspace_bytes(
            prec, trans if trans in tuple("NnTtCc") else "N", max(m - offset_r, 0), max(n - offset_c, 0)), y, stream)
        rc = getattr(lib, f"kmv_{prec}gemv_offset")(
            trans.encode(), m, n, _scalar(prec, alpha), _ptr(A, prec), lda, _ptr(x, prec), incx, _scalar(prec, beta),
            _ptr(y, prec), incy, offset_r, offset_c, ctypes.c_void_p(wsp), wsb, _stream(stream))
        if check and rc != 0:
            raise KmvError(f"{prec}gemv_offset", rc)
        return rc
    call.__name__ = f"{prec}gemv_offset"
    call.__doc__ = "GEMV with the block of the parent A (m x n) from row offset_r and column offset_c on."
    return call


def _symv_offset(prec, complex_symmetric=False):
    name = f"{prec}{'hemv' if prec in 'cz' and not complex_symmetric else 'symv'}_offset"

    def call(uplo, n, alpha, A, lda, x, incx, beta, y, incy, offset, workspace=None, stream=None, check=True):
        wsp, wsb = _ws_args(workspace, lambda: symv_workspace_bytes(
            prec, uplo if uplo in tuple("LlUu") else "L", max(n - offset, 0)), y, stream)
        rc = getattr(lib, f"kmv_{name}")(
            uplo.encode(), n, _scalar(prec, alpha), _ptr(A, prec), lda, _ptr(x, prec), incx, _scalar(prec, beta),
            _ptr(y, prec), incy, offset, ctypes.c_void_p(wsp), wsb, _stream(stream))
        if check and rc != 0:
            raise KmvError(name, rc)
        return rc
    call.__name__ = name
    call.__doc__ = "SYMV / HEMV with the trailing diagonal block of the parent A (n x n) from `offset` on."
    return call


def _gemv_devscalars(prec):
    def call(trans, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
        wsp, wsb = _ws_args(workspace, lambda: gemv_workspace_bytes(
            prec, trans if trans in tuple("NnTtCc") else "N", max(m, 0), max(n, 0)), y, stream)
        rc = getattr(lib, f"kmv_{prec}gemv_devscalars")(
            trans.encode(), m, n, _ptr(alpha, prec), _ptr(A, prec), lda, _ptr(x, prec), incx, _ptr(beta, prec),
            _ptr(y, prec), incy, ctypes.c_void_p(wsp), wsb, _stream(stream))
        if check and rc != 0:
            raise KmvError(f"{prec}gemv_devscalars", rc)
        return rc
    call.__name__ = f"{prec}gemv_devscalars"
    call.__doc__ = "GEMV with alpha and beta given as one-element device tensors (or device addresses)."
    return call


def _symv_devscalars(prec, complex_symmetric=False):
    name = f"{prec}{'hemv' if prec in 'cz' and not complex_symmetric else 'symv'}_devscalars"

    def call(uplo, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None, check=True):
        wsp, wsb = _ws_args(workspace, lambda: symv_workspace_bytes(
            prec, uplo if uplo in tuple("LlUu") else "L", max(n, 0)), y, stream)
        rc = getattr(lib, f"kmv_{name}")(
            uplo.encode(), n, _ptr(alpha, prec), _ptr(A, prec), lda, _ptr(x, prec), incx, _ptr(beta, prec),
            _ptr(y, prec), incy, ctypes.c_void_p(wsp), wsb, _stream(stream))
        if check and rc != 0:
            raise KmvError(name, rc)
        return rc
    call.__name__ = name
    call.__doc__ = "SYMV / HEMV with alpha and beta given as one-element device tensors (or device addresses)."
    return call


def _gemv_strided_batched(prec):
    def call(trans, m, n, alpha, A, lda, strideA, x, incx, stridex, beta, y, incy, stridey, batch, stream=None,
             check=True):
        rc = getattr(lib, f"kmv_{prec}gemv_strided_batched")(
            trans.encode(), m, n, _scalar(prec, alpha), _ptr(A, prec), lda, strideA, _ptr(x, prec), incx, stridex,
            _scalar(prec, beta), _ptr(y, prec), incy, stridey, batch, _stream(stream))
        if check and rc != 0:
            raise KmvError(f"{prec}gemv_strided_batched", rc)
        return rc
    call.__name__ = f"{prec}gemv_strided_batched"
    call.__doc__ = "`batch` GEMVs of one shape; member b uses A + b*strideA, x + b*stridex, y + b*stridey."
    return call


def _symv_strided_batched(prec, complex_symmetric=False):
    name = f"{prec}{'hemv' if prec in 'cz' and not complex_symmetric else 'symv'}_strided_batched"

    def call(uplo, n, alpha, A, lda, strideA, x, incx, stridex, beta, y, incy, stridey, batch, stream=None,
             check=True):
        rc = getattr(lib, f"kmv_{name}")(
            uplo.encode(), n, _scalar(prec, alpha), _ptr(A, prec), lda, strideA, _ptr(x, prec), incx, stridex,
            _scalar(prec, beta), _ptr(y, prec), incy, stridey, batch, _stream(stream))
        if check and rc != 0:
            raise KmvError(name, rc)
        return rc
    call.__name__ = name
    call.__doc__ = "`batch` SYMV / HEMV products of one shape; member b uses A + b*strideA, x + b*stridex, y + b*stridey."
    return call


def pointer_array(tensors_or_addresses, device=None) -> torch.Tensor:
    """Device array of device addresses (int64) for the `_batched` calls: one entry per member, taken from
    tensors (their `data_ptr()`) or given as integers."""
    addrs = [t if isinstance(t, int) else t.data_ptr() for t in tensors_or_addresses]
    if device is None:
        device = next((t.device for t in tensors_or_addresses if not isinstance(t, int)), "cuda")
    return torch.tensor(addrs, dtype=torch.int64, device=device)


def _ptr_array(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if t.dtype != torch.int64:
        raise TypeError(f"expected an int64 tensor of device addresses, got {t.dtype}")
    if not t.is_cuda:
        raise ValueError("the pointer arrays live in device memory")
    return ctypes.c_void_p(t.data_ptr())


def _gemv_batched(prec):
    def call(trans, m, n, alpha, A, lda, x, incx, beta, y, incy, batch, stream=None, check=True):
        rc = getattr(lib, f"kmv_{prec}gemv_batched")(
            trans.encode(), m, n, _scalar(prec, alpha), _ptr_array(A), lda, _ptr_array(x), incx, _scalar(prec, beta),
            _ptr_array(y), incy, batch, _stream(stream))
        if check and rc != 0:
            raise KmvError(f"{prec}gemv_batched", rc)
        return rc
    call.__name__ = f"{prec}gemv_batched"
    call.__doc__ = "`batch` GEMVs of one shape; A, x, y are int64 device tensors of device addresses (see pointer_array)."
    return call


def _symv_batched(prec, complex_symmetric=False):
    name = f"{prec}{'hemv' if prec in 'cz' and not complex_symmetric else 'symv'}_batched"

    def call(uplo, n, alpha, A, lda, x, incx, beta, y, incy, batch, stream=None, check=True):
        rc = getattr(lib, f"kmv_{name}")(
            uplo.encode(), n, _scalar(prec, alpha), _ptr_array(A), lda, _ptr_array(x), incx, _scalar(prec, beta),
            _ptr_array(y), incy, batch, _stream(stream))
        if check and rc != 0:
            raise KmvError(name, rc)
        return rc
    call.__name__ = name
    call.__doc__ = "`batch` SYMV / HEMV products of one shape; A, x, y are int64 device tensors of device addresses."
    return call


GEMV_BATCHED = {p_: _gemv_batched(p_) for p_ in "sdcz"}
SYMV_BATCHED = {p_: _symv_batched(p_) for p_ in "sdcz"}          # HEMV for the complex precisions
CSYMV_BATCHED = {p_: _symv_batched(p_, True) for p_ in "cz"}
sgemv_batched, dgemv_batched, cgemv_batched, zgemv_batched = (GEMV_BATCHED[p_] for p_ in "sdcz")
ssymv_batched, dsymv_batched, chemv_batched, zhemv_batched = (SYMV_BATCHED[p_] for p_ in "sdcz")
csymv_batched, zsymv_batched = (CSYMV_BATCHED[p_] for p_ in "cz")
GEMV_STRIDED_BATCHED = {p_: _gemv_strided_batched(p_) for p_ in "sdcz"}
SYMV_STRIDED_BATCHED = {p_: _symv_strided_batched(p_) for p_ in "sdcz"}
sgemv_strided_batched, dgemv_strided_batched, cgemv_strided_batched, zgemv_strided_batched = (
    GEMV_STRIDED_BATCHED[p_] for p_ in "sdcz")
ssymv_strided_batched, dsymv_strided_batched, chemv_strided_batched, zhemv_strided_batched = (
    SYMV_STRIDED_BATCHED[p_] for p_ in "sdcz")


def sytrd_panel_workspace_bytes(prec, n, nb) -> int:
    return int(lib.kmv_sytrd_panel_workspace_bytes(prec.encode(), n, nb))


def _sytrd_panel(prec):
    name = f"{prec}{'hetrd' if prec in 'cz' else 'sytrd'}_panel"
    eprec = {"s": "s", "d": "d", "c": "s", "z": "d"}[prec]      # e is real

    def call(uplo, n, nb, A, lda, e, tau, W, ldw, workspace=None, stream=None, check=True):
        wsp, wsb = _ws_args(workspace, lambda: sytrd_panel_workspace_bytes(prec, max(n, 0), max(min(nb, n), 0)), A, stream)
        rc = getattr(lib, f"kmv_{name}")(
            uplo.encode(), n, nb, _ptr(A, prec), lda, _ptr(e, eprec), _ptr(tau, prec), _ptr(W, prec), ldw,
            ctypes.c_void_p(wsp), wsb, _stream(stream))
        if check and rc != 0:
            raise KmvError(name, rc)
        return rc
    call.__name__ = name
    call.__doc__ = "Panel step of the symmetric tridiagonal reduction on device tensors (see include/kmv.h)."
    return call


def gebrd_panel_workspace_bytes(prec, m, n, nb) -> int:
    return int(lib.kmv_gebrd_panel_workspace_bytes(prec.encode(), m, n, nb))


def _gebrd_panel(prec):
    rprec = {"s": "s", "d": "d", "c": "s", "z": "d"}[prec]      # d and e are real

    def call(m, n, nb, A, lda, d, e, tauq, taup, X, ldx, Y, ldy, workspace=None, stream=None, check=True):
        wsp, wsb = _ws_args(workspace, lambda: gebrd_panel_workspace_bytes(prec, max(m, 0), max(n, 0), max(nb, 0)), A, stream)
        rc = getattr(lib, f"kmv_{prec}gebrd_panel")(
            m, n, nb, _ptr(A, prec), lda, _ptr(d, rprec), _ptr(e, rprec), _ptr(tauq, prec), _ptr(taup, prec),
            _ptr(X, prec), ldx, _ptr(Y, prec), ldy, ctypes.c_void_p(wsp), wsb, _stream(stream))
        if check and rc != 0:
            raise KmvError(f"{prec}gebrd_panel", rc)
        return rc
    call.__name__ = f"{prec}gebrd_panel"
    call.__doc__ = "Panel step of the bidiagonal reduction on device tensors (see include/kmv.h)."
    return call


GEBRD_PANEL = {p_: _gebrd_panel(p_) for p_ in "sdcz"}
sgebrd_panel, dgebrd_panel, cgebrd_panel, zgebrd_panel = (GEBRD_PANEL[p_] for p_ in "sdcz")
SYTRD_PANEL = {p_: _sytrd_panel(p_) for p_ in "sdcz"}      # HETRD for the complex precisions
ssytrd_panel, dsytrd_panel, chetrd_panel, zhetrd_panel = (SYTRD_PANEL[p_] for p_ in "sdcz")
GEMV_DEVSCALARS = {p_: _gemv_devscalars(p_) for p_ in "sdcz"}
SYMV_DEVSCALARS = {p_: _symv_devscalars(p_) for p_ in "sdcz"}
sgemv_devscalars, dgemv_devscalars, cgemv_devscalars, zgemv_devscalars = (GEMV_DEVSCALARS[p_] for p_ in "sdcz")
ssymv_devscalars, dsymv_devscalars, chemv_devscalars, zhemv_devscalars = (SYMV_DEVSCALARS[p_] for p_ in "sdcz")
sgemv_offset, dgemv_offset, cgemv_offset, zgemv_offset = (_gemv_offset(p_) for p_ in "sdcz")
ssymv_offset, dsymv_offset, chemv_offset, zhemv_offset = (_symv_offset(p_) for p_ in "sdcz")
GEMV_OFFSET = {"s": sgemv_offset, "d": dgemv_offset, "c": cgemv_offset, "z": zgemv_offset}
SYMV_OFFSET = {"s": ssymv_offset, "d": dsymv_offset, "c": chemv_offset, "z": zhemv_offset}

GEMV = {"s": sgemv, "d": dgemv, "c": cgemv, "z": zgemv}
SYMV = {"s": ssymv, "d": dsymv, "c": chemv, "z": zhemv}   # HEMV for the complex precisions
CSYMV = {"c": csymv, "z": zsymv}                          # complex symmetric
CSYMV_OFFSET = {p_: _symv_offset(p_, True) for p_ in "cz"}
CSYMV_DEVSCALARS = {p_: _symv_devscalars(p_, True) for p_ in "cz"}
CSYMV_STRIDED_BATCHED = {p_: _symv_strided_batched(p_, True) for p_ in "cz"}
csymv_offset, zsymv_offset = (CSYMV_OFFSET[p_] for p_ in "cz")
csymv_devscalars, zsymv_devscalars = (CSYMV_DEVSCALARS[p_] for p_ in "cz")
csymv_strided_batched, zsymv_strided_batched = (CSYMV_STRIDED_BATCHED[p_] for p_ in "cz")


def partition(W, Y, y):
    w, s = ctypes.c_int64(), ctypes.c_int64()
    lib.kmv_partition(W, Y, y, ctypes.byref(w), ctypes.byref(s))
    return w.value, s.value


def stream_probe(kind, n, a, b=None, c=None, sink=None, stream=None):
    rc = lib.kmv_stream_probe(kind, n, _ptr(a), _ptr(b), _ptr(c), _ptr(sink), _stream(stream))
    if rc != 0:
        raise KmvError("stream_probe", rc)


def set_tuning(key, value):
    if lib.kmv_set_tuning(key.encode(), int(value)) != 0:
        raise ValueError(f"bad tuning {key}={value}")


def get_tuning(key):
    return int(lib.kmv_get_tuning(key.encode()))


def tuning_keys():
    return lib.kmv_tuning_keys().decode().split(",")


TUNED_FIELDS = ("gemv_n_splits", "gemv_n_row_tiles", "gemv_t_splits", "symv_variant", "symv_tiles_per_wave",
                "symv_unit_tiles", "wg_target")


def tuned_settings(prec, op, n):
    """Row of the compiled-in table of measured settings that the planners apply to a square product of
    routine op ('N', 'T', 'L', 'U') at size n, as {key: value} without the zero fields; None if no row applies."""
    vals = (ctypes.c_int64 * 7)()
    rc = int(lib.kmv_tuned_settings(prec.encode(), op.encode(), n, vals))
    if rc < 0:
        raise ValueError(f"bad arguments ({prec!r}, {op!r}, {n})")
    return {f: int(v) for f, v in zip(TUNED_FIELDS, vals) if v} if rc == 1 else None


def symv_kernel_variant(prec, uplo, n, A, lda):
    """2 (balanced shares) or 3 (one launch): the main kernel a symv/hemv call with these
    arguments launches; A may be a tensor or an integer address"""
    addr = A if isinstance(A, int) else A.data_ptr()
    return int(lib.kmv_symv_kernel_variant(prec.encode(), uplo.encode(), n, ctypes.c_void_p(addr), lda))


def symv_shares(prec, uplo, n, shift, chunk_tiles, unit_tiles, slots, fixed, edge=0):
    """Table of shares of the balanced SYMV/HEMV kernel for these settings: (workers, work,
    [(chunk, piece)] * (workers + 1), first[272], last[272]); None for arguments out of range."""
    start = (ctypes.c_uint32 * 801)()
    first, last = (ctypes.c_uint16 * 272)(), (ctypes.c_uint16 * 272)()
    work = ctypes.c_int64(0)
    y = int(lib.kmv_symv_shares(prec.encode(), uplo.encode(), n, shift, chunk_tiles, unit_tiles, slots, fixed, edge, start, first,
                                last, ctypes.byref(work)))
    if y < 0:
        return None
    return y, work.value, [(e >> 20, e & 0xFFFFF) for e in start[: y + 1]], list(first), list(last)


def version():
    return lib.kmv_version().decode()
