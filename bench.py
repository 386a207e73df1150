#!/usr/bin/env python3
"""Benchmark of the kmv hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--table FILE]

One "step" is one pass of the whole hot path over one batch of synthetic
inputs.  The default workload `all` runs four groups per step, one after the
other, each bracketed by device synchronisations:

  sweep      the size sweep the headline metric is quoted on: SGEMV / DGEMV (N
             and T) and DSYMV / ZHEMV (L and U) on square matrices, n = 1024 ..
             32768 in steps of 1024 plus n = 1000, 4099, 17001 for GEMV, lda = n,
             entries U[-1,1], seed 0 (268 products)
  target16k  all 16 routine x precision products at n = 16384 and 32768
  large      all 16 at n = 49152 (s, c) / 40960 (d, z), lda = n + 32, N(0,1)
             entries, incx 1 and 2
  subblock   DGEMV N, T and DSYMV L on blocks of a 20000 x 20000 parent at
             offsets 1, 17, 63, 1000

`value` is the sweep group's throughput (the configurations the metric is
quoted on); every group reports its own throughput and per-routine fractions
of the HBM peak.  All inputs are resident in HBM before the timed region
starts; every product whose matrix is smaller than 512 MB works on a region
of its own, so no product finds its matrix in a cache because another product
read it (the same small products timed back to back on one region are
reported separately as `cache_resident`).

The metric follows the paper's performance model (Section 7): algorithmic
bytes (matrix once, x once, y read and written once; one triangle for the
symmetric products) divided by time, in GB/s, as a fraction of the HBM peak;
Gflop/s with the paper's flop counts are reported alongside.

Prints ONE JSON line on stdout.  `--table FILE` additionally writes one JSON
line per (routine, n) with GB/s, % of peak and Gflop/s (the "vs n" curves).
Only the `cpu_baseline` leg touches the CPU oracle.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

COLD_BYTES = 512e6      # products with a smaller matrix get a region of their own (and a cache-resident timing)
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "default_step_hbm_traffic.txt")


def measured_traffic(kernel):
    """HBM bytes (read + written) per launch of `kernel` in the default benchmark, from the rocprofv3 --pmc
    summary under profiles/ (lines `traffic kernel=<name> ... bytes_per_launch=<n> library=<version>`), or
    None when the summary is missing, does not list the kernel or was made with another library version."""
    from paper_1410_1726_amd import binding as k
    try:
        with open(TRAFFIC_PROFILE) as f:
            for line in f:
                if not line.startswith("traffic "):
                    continue
                kv = dict(item.split("=", 1) for item in line.split()[1:] if "=" in item)
                if kv.get("kernel") == kernel.replace(" ", "") and kv.get("library") == k.version().replace(" ", "_"):
                    return int(kv["bytes_per_launch"])
    except (OSError, ValueError, KeyError):
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="all", choices=["all", "sweep", "target16k", "large", "subblock", "panel", "sytrd", "gebrd", "batched", "csymv", "rect", "tiny"])
    ap.add_argument("--prec", default="d", choices=list("sdcz"), help="precision of the sytrd / gebrd / batched workloads")
    ap.add_argument("--uplo", default="L", choices=["L", "U"], help="stored triangle of the sytrd workload")
    ap.add_argument("--table", default=None, help="write per-(routine, n) JSON lines to this file")
    ap.add_argument("--only", default=None, help="regular expression on 'routine:n' (e.g. 'dsymv_L:16384|dgemv_N:'): time only "
                                                 "the matching products of the workload (for profiles)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cache-resident", action="store_true",
                    help="skip the back-to-back calls of the cache-sized products after the timed steps (for profiles: every "
                         "launch of the run then belongs to a step)")
    ap.add_argument("--tuning", action="append", default=[], help="key=value for kmv_set_tuning")
    return ap.parse_args()


# --------------------------------------------------------------- workloads ----
def products(workload):
    """List of dicts describing the products of one step."""
    out = []
    if workload == "all":
        for group in ("sweep", "target16k", "large", "subblock"):
            for p in products(group):
                p["group"] = group
                out.append(p)
        return out
    if workload == "sweep":
        sizes = [1024 * k for k in range(1, 33)]
        for prec in "sd":
            for trans in "NT":
                for n in sizes + [1000, 4099, 17001]:
                    out.append(dict(kind="gemv", prec=prec, mode=trans, n=n, lda=n, alpha=1.0, beta=1.0))
        for prec in "dz":
            for uplo in "LU":
                for n in sizes:
                    out.append(dict(kind="symv", prec=prec, mode=uplo, n=n, lda=n, alpha=1.0, beta=0.0))
    elif workload == "target16k":
        for prec in "sdcz":
            for n in (16384, 32768):
                for trans in "NT":
                    out.append(dict(kind="gemv", prec=prec, mode=trans, n=n, lda=n, alpha=1.0, beta=1.0))
                for uplo in "LU":
                    out.append(dict(kind="symv", prec=prec, mode=uplo, n=n, lda=n, alpha=1.0, beta=0.0))
    elif workload == "large":      # lda = n + 32, normal entries, alpha 0.7, beta 0.3, incx 1 and 2
        for prec in "sdcz":
            n = 49152 if prec in "sc" else 40960
            for incx in (1, 2):
                for trans in "NT":
                    out.append(dict(kind="gemv", prec=prec, mode=trans, n=n, lda=n + 32, alpha=0.7, beta=0.3,
                                    incx=incx, dist="normal"))
                for uplo in "LU":
                    out.append(dict(kind="symv", prec=prec, mode=uplo, n=n, lda=n + 32, alpha=0.7, beta=0.3,
                                    incx=incx, dist="normal"))
    elif workload == "subblock":   # blocks of a 20000 x 20000 fp64 parent at (o, o)
        for o in (1, 17, 63, 1000):
            for n in (2048, 8192, 19000 - o):
                for trans in "NT":
                    out.append(dict(kind="gemv", prec="d", mode=trans, n=n, lda=20000, off=o, parent=20000,
                                    alpha=-1.0, beta=1.0))
                out.append(dict(kind="symv", prec="d", mode="L", n=n, lda=20000, off=o, parent=20000,
                                alpha=-1.0, beta=1.0))
    elif workload == "panel":      # the products of one 64-column panel of the two-sided reductions (Section 10):
        # column j of the panel multiplies by the trailing block that starts at j or j+1 of a 16384 x 16384 parent
        for j in range(64):
            out.append(dict(kind="symv", prec="d", mode="L", n=16384 - (j + 1), lda=16384, off=j + 1, parent=16384,
                            alpha=1.0, beta=0.0))
            out.append(dict(kind="gemv", prec="d", mode="T", n=16384 - j, lda=16384, off=j, parent=16384,
                            alpha=1.0, beta=0.0))
            out.append(dict(kind="gemv", prec="d", mode="N", n=16384 - (j + 1), lda=16384, off=j + 1, parent=16384,
                            alpha=1.0, beta=0.0))
    elif workload == "csymv":      # complex symmetric SYMV beside HEMV, same shapes
        for prec in "cz":
            for n in (16384, 32768):
                for uplo in "LU":
                    out.append(dict(kind="symv", prec=prec, mode=uplo, n=n, lda=n, alpha=1.0, beta=0.0, csym=True))
                    out.append(dict(kind="symv", prec=prec, mode=uplo, n=n, lda=n, alpha=1.0, beta=0.0))
    elif workload == "rect":       # panels as in blocked reductions: tall-skinny and short-wide, d and s, N and T
        shapes = [(65536, 32), (65536, 128), (65536, 512), (16384, 64), (16384, 256), (16384, 1024), (16384, 4096),
                  (32, 65536), (128, 65536), (512, 65536), (64, 16384), (256, 16384), (1024, 16384), (4096, 16384)]
        for prec in "ds":
            for m, n in shapes:
                for trans in "NT":
                    out.append(dict(kind="gemv", prec=prec, mode=trans, m=m, n=n, lda=m, alpha=1.0, beta=1.0))
    elif workload == "tiny":       # DGEMV N, m = n = lda = 1024, alpha 1.5, beta 0.5
        out.append(dict(kind="gemv", prec="d", mode="N", n=1024, lda=1024, alpha=1.5, beta=0.5))
    return out


def op_name(p):
    if p["kind"] == "gemv":
        return "gemv_" + p["mode"].lower()
    return ("hemv_" if p["prec"] in "cz" else "symv_") + p["mode"].lower()


def routine_name(p):
    if p["kind"] == "gemv":
        return f"{p['prec']}gemv_{p['mode']}"
    return f"{p['prec']}{'hemv' if p['prec'] in 'cz' and not p.get('csym') else 'symv'}_{p['mode']}"


def kernel_name(p):
    """main device kernel of a product (what rocprofv3 lists)"""
    t = {"s": "float", "d": "double", "c": "kmv::cf32", "z": "kmv::cf64"}[p["prec"]]
    if p["kind"] == "gemv":
        return f"gemv_{'n' if p['mode'] == 'N' else 't'}_kernel<{t}>"
    from paper_1410_1726_amd import binding as k
    esize = {"s": 4, "d": 8, "c": 8, "z": 16}[p["prec"]]
    # only the alignment of A matters to the choice: the bench buffers are 256-byte aligned
    variant = k.symv_kernel_variant(p["prec"], p["mode"], p["n"], 256 + (p.get("off", 0) * (p["lda"] + 1)) * esize, p["lda"])
    return f"{ {1: 'symv_kernel', 2: 'symv_balanced_kernel', 3: 'symv_small_kernel'}[variant] }<{t}>"


def matrix_span(p):
    """elements of the flat buffer that the product's matrix (or its parent) spans"""
    cols = p.get("parent", 0) or p["n"]
    return p["lda"] * cols


class Inputs:
    """Device buffers: per (precision, distribution) one flat matrix buffer and one x / y pair.  A product views
    the buffer with its own lda; a product whose matrix is smaller than COLD_BYTES views a region of its own (the
    regions of one buffer are laid end to end), so that its matrix is not in a cache because another product
    just read the same addresses; the large ones all start at the front, each of them alone replaces whatever
    the caches held.  Filled once, before anything is timed.  The unreferenced triangle of the symmetric
    products holds ordinary random numbers here (one buffer serves all sizes, so there is no one triangle to
    poison): it is never loaded, so its content cannot change the timing; the parity tests run the same shapes
    with that triangle set to NaN, and check_poisoned() below runs one poisoned product per routine."""

    def __init__(self, prods, torch, wl, acc):
        need, vlen, small = {}, {}, {}
        esize = {"s": 4, "d": 8, "c": 8, "z": 16}
        self.offset = {}
        for i, p in enumerate(prods):
            key = (p["prec"], p.get("dist", "uniform"))
            span = matrix_span(p)
            need[key] = max(need.get(key, 0), span)
            vlen[key] = max(vlen.get(key, 0), 1 + (max(p["n"], p.get("m", 0)) - 1) * abs(p.get("incx", 1)))
            if span * esize[p["prec"]] < COLD_BYTES and not p.get("parent"):
                self.offset[i] = small.get(key, 0)
                small[key] = self.offset[i] + (span + 63) // 64 * 64
        self.mat, self.vec = {}, {}
        for key, elems in need.items():
            prec, dist = key
            elems = max(elems, small.get(key, 0))
            flat = torch.empty(elems, dtype=wl.TORCH_DTYPES[prec], device="cuda")
            g = torch.Generator(device="cuda")
            g.manual_seed(0)
            wl.fill_random(flat, dist, g)
            self.mat[key] = flat
            self.vec[key] = (wl.vector(prec, vlen[key], 1, dist=dist, seed=0, which=1, device="cuda"),
                             wl.vector(prec, vlen[key], 1, dist=dist, seed=0, which=2, device="cuda"))

    def views(self, i, p, own_region=True):
        key = (p["prec"], p.get("dist", "uniform"))
        n, lda, off = p["n"], p["lda"], p.get("off", 0)
        cols = p.get("parent", 0) or n
        start = self.offset.get(i, 0) if own_region else 0
        A2 = self.mat[key][start: start + lda * cols].view(cols, lda)
        A = A2[off:, off:] if off else A2
        x, y = self.vec[key]
        return A, x, y


def check_poisoned(k, torch, wl):
    """One product per symmetric routine on a matrix whose unreferenced triangle is NaN (and y NaN, beta = 0):
    the result must be finite.  Not timed; the element-wise comparison with the oracle is the parity tests'."""
    n = 4100
    for prec in "sdcz":
        for uplo in "LU":
            A = wl.poison_triangle(wl.matrix(prec, n, n, n + 12, seed=3, device="cuda"), n, uplo)
            x = wl.vector(prec, n, 1, seed=3, which=1, device="cuda")
            y = torch.full_like(x, float("nan"))
            k.SYMV[prec](uplo, n, 1.0, A, n + 12, x, 1, 0.0, y, 1)
            torch.cuda.synchronize()
            if not bool(torch.isfinite(torch.view_as_real(y) if y.is_complex() else y).all()):
                raise RuntimeError(f"bench.py: {prec} symv/hemv {uplo} read the unreferenced triangle or y with beta = 0")
    return "ok"


def make_call(p, k, A, x, y):
    n, lda, incx = p["n"], p["lda"], p.get("incx", 1)
    # arguments are marshalled once, outside the timed region; a call is then one foreign call
    if p["kind"] == "gemv":
        return k.prepare_gemv(p["prec"], p["mode"], p.get("m", n), n, p["alpha"], A, lda, x, incx, p["beta"], y, 1)
    return k.prepare_symv(p["prec"], p["mode"], n, p["alpha"], A, lda, x, incx, p["beta"], y, 1,
                          complex_symmetric=bool(p.get("csym")))


def tiny_latency(k, torch, wl):
    """DGEMV N 1024 x 1024: microseconds per call with the matrix resident in cache (the
    same buffers every call) and cold (96 distinct matrices in rotation, 768 MiB, more
    than the last-level cache), both as a back-to-back series between two events."""
    n, copies = 1024, 96
    As = [wl.matrix("d", n, n, n, seed=s, device="cuda") for s in range(copies)]
    x = wl.vector("d", n, seed=0, which=1, device="cuda")
    y = wl.vector("d", n, seed=0, which=2, device="cuda")
    calls = [k.prepare_gemv("d", "N", n, n, 1.5, A, n, x, 1, 0.5, y, 1) for A in As]

    def series(seq, reps):
        for c in seq[:4]:
            c()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            for c in seq:
                c()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * len(seq))

    return {"warm": round(series(calls[:1] * copies, 5), 2), "cold": round(series(calls, 5), 2)}


# ------------------------------------------------------------ CPU baseline ----
DTYPE_NAMES = {"s": "f32", "d": "f64", "c": "c64", "z": "c128"}


def sytrd_panel_bench(args, k, torch, wl, acc):
    """One step = the panel step of the tridiagonal reduction (kmv_dsytrd_panel) on the first 64 columns of a
    16384 x 16384 fp64 matrix: per column one DSYMV on the trailing block and the products with the two
    reflector panels (two N products with a row of the other panel, two T and two N products with v) plus the
    reflector and the scaling of w, which the library runs as three kernels of its own, all enqueued without a
    host round trip.  The bytes counted are those of the algorithm's products, each panel product as a GEMV of
    its own (what the step costs when built from BLAS calls), so that the figure compares across
    implementations.  The matrix is restored from a copy before every step, outside the timed brackets."""
    n, nb, prec, uplo = 16384, 64, args.prec, args.uplo
    A0 = wl.matrix(prec, n, n, n, seed=0, device="cuda")
    A = A0.clone()
    dt = wl.TORCH_DTYPES[prec]
    rdt = wl.TORCH_DTYPES[{"c": "s", "z": "d"}.get(prec, prec)]      # e is real
    esz = A0.element_size()
    W = torch.zeros((nb, n), dtype=dt, device="cuda")
    e = torch.zeros(nb, dtype=rdt, device="cuda")
    tau = torch.zeros(nb, dtype=dt, device="cuda")
    ws = k.workspace(k.sytrd_panel_workspace_bytes(prec, n, nb))
    stream = torch.cuda.current_stream()
    nbytes = nflops = 0
    for i in range(nb):
        ops = [("gemv_n", n - i, i)] * 2 if i else []
        m = n - i - 1
        ops += [("symv_l", m, m)] + ([("gemv_t", m, i), ("gemv_n", m, i)] * 2 if i else [])
        for op, mm, nn in ops:
            nbytes += acc.algorithmic_bytes(op, prec, mm, nn)
            nflops += acc.flops(op, prec, mm, nn)
        nbytes += 6 * m * esz          # the two vector kernels: v read and written, then w and v read, w written
    times = []
    for step in range(args.warmup + args.steps):
        A.copy_(A0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        k.SYTRD_PANEL[prec](uplo, n, nb, A, n, e, tau, W, n, workspace=ws)
        e1.record(stream)
        host_ms = (time.perf_counter() - t0) * 1e3
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        if step >= args.warmup:
            times.append((wall_ms, e0.elapsed_time(e1), host_ms))
    step_ms = sum(t[0] for t in times) / len(times)
    value = nbytes / (step_ms * 1e-3) / 1e9
    symv_bytes = sum(acc.algorithmic_bytes("symv_l", prec, n - i - 1, n - i - 1) for i in range(nb))
    return {
        "metric": "achieved HBM GB/s (algorithmic bytes / time) for xGEMV/xSYMV vs n, 1 GPU",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_NAMES[prec], "data": "synthetic",
        "config": {"workload": f"panel step of the tridiagonal reduction (kmv_{prec}{'hetrd' if prec in 'cz' else 'sytrd'}_panel, "
                               f"uplo {uplo}), n=16384, nb=64, lda=n, U[-1,1]: 64 SYMV/HEMV on trailing blocks + 378 products "
                               "with the reflector panels + 128 vector steps (three fused kernels per column)",
                   "products_per_step": nb + 6 * (nb - 1)},
        "frac_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "gflops": round(nflops / (step_ms * 1e-3) / 1e9, 1),
        "device_ms_per_step": round(sum(t[1] for t in times) / len(times), 3),
        "host_enqueue_ms_per_step": round(sum(t[2] for t in times) / len(times), 3),
        "symv_share_of_bytes": round(symv_bytes / nbytes, 4),
        "roofline": None,
    }


def gebrd_panel_bench(args, k, torch, wl, acc):
    """One step = the panel step of the bidiagonal reduction (kmv_dgebrd_panel) on the first 64 columns and rows of
    a 16384 x 16384 matrix: per column GEMV-T and GEMV-N on the whole trailing block and eleven products with the
    accumulated panels, two reflectors, two scalings (the panel products and vector steps run in four fused
    launches per column; the bytes counted are those of the algorithm's products, each as a GEMV of its own)."""
    m = n = 16384
    nb, prec = 64, args.prec
    A0 = wl.matrix(prec, m, n, m, seed=0, device="cuda")
    A = A0.clone()
    dt = wl.TORCH_DTYPES[prec]
    rdt = wl.TORCH_DTYPES[{"c": "s", "z": "d"}.get(prec, prec)]      # d and e are real
    X = torch.zeros((nb, m), dtype=dt, device="cuda")
    Y = torch.zeros((nb, n), dtype=dt, device="cuda")
    d, e = (torch.zeros(nb, dtype=rdt, device="cuda") for _ in range(2))
    tauq, taup = (torch.zeros(nb, dtype=dt, device="cuda") for _ in range(2))
    ws = k.workspace(k.gebrd_panel_workspace_bytes(prec, m, n, nb))
    stream = torch.cuda.current_stream()
    nbytes = nflops = big = 0
    for i in range(nb):
        mi, ni = m - i, n - i - 1
        ops = [("gemv_n", mi, i)] * 2 if i else []
        ops += [("gemv_t", mi, ni), ("gemv_n", ni, i + 1), ("gemv_n", mi - 1, ni), ("gemv_t", ni, i + 1), ("gemv_n", mi - 1, i + 1)]
        if i:
            ops += [("gemv_t", mi, i), ("gemv_n", ni, i), ("gemv_t", mi, i), ("gemv_t", i, ni), ("gemv_t", i, ni),
                    ("gemv_n", i, ni), ("gemv_n", mi - 1, i)]
        for op, mm, nn in ops:
            nbytes += acc.algorithmic_bytes(op, prec, mm, nn)
            nflops += acc.flops(op, prec, mm, nn)
        big += acc.algorithmic_bytes("gemv_t", prec, mi, ni) + acc.algorithmic_bytes("gemv_n", prec, mi - 1, ni)
    times = []
    for step in range(args.warmup + args.steps):
        A.copy_(A0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        k.GEBRD_PANEL[prec](m, n, nb, A, m, d, e, tauq, taup, X, m, Y, n, workspace=ws)
        e1.record(stream)
        host_ms = (time.perf_counter() - t0) * 1e3
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        if step >= args.warmup:
            times.append((wall_ms, e0.elapsed_time(e1), host_ms))
    step_ms = sum(t[0] for t in times) / len(times)
    value = nbytes / (step_ms * 1e-3) / 1e9
    return {
        "metric": "achieved HBM GB/s (algorithmic bytes / time) for xGEMV/xSYMV vs n, 1 GPU",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_NAMES[prec], "data": "synthetic",
        "config": {"workload": f"panel step of the bidiagonal reduction (kmv_{prec}gebrd_panel), m=n=16384, nb=64, lda=m, "
                               "U[-1,1]: 128 GEMV on trailing blocks + about 690 products with the panels (four fused kernels per column)",
                   "products_per_step": 2 * nb + 11 * (nb - 1)},
        "frac_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "gflops": round(nflops / (step_ms * 1e-3) / 1e9, 1),
        "device_ms_per_step": round(sum(t[1] for t in times) / len(times), 3),
        "host_enqueue_ms_per_step": round(sum(t[2] for t in times) / len(times), 3),
        "trailing_block_share_of_bytes": round(big / nbytes, 4),
        "roofline": None,
    }


def batched_bench(args, k, torch, wl, acc):
    """One step = strided batches of small products (--prec, default fp64), 1 GiB of matrices per batch: GEMV N and
    T and SYMV/HEMV L at n = 64 .. 1024, one call (one launch) per batch.  For comparison the same products as a
    loop of single calls (prepared, so a call is one foreign call) are timed on the first 256 members."""
    prec = args.prec
    dt = wl.TORCH_DTYPES[prec]
    esz = torch.empty(0, dtype=dt).element_size()
    total = (1 << 30) // esz             # elements of matrix storage per batch (1 GiB)
    flat = torch.empty(total, dtype=dt, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    wl.fill_random(flat, "uniform", g)
    stream = torch.cuda.current_stream()
    rows, tot_bytes, tot_ms = [], 0, 0.0
    sizes = (64, 128, 256, 512, 1024)
    cases = [(kind, n) for n in sizes for kind in ("gemv_n", "gemv_t", "symv_l")]
    xs = wl.vector(prec, total // min(sizes), 1, seed=0, which=1, device="cuda")     # batch * n elements at most
    ys = wl.vector(prec, total // min(sizes), 1, seed=0, which=2, device="cuda")
    symv_name = prec + ("hemv" if prec in "cz" else "symv")

    def run(kind, n, batch):
        if kind == "symv_l":
            k.SYMV_STRIDED_BATCHED[prec]("L", n, 1.0, flat, n, n * n, xs, 1, n, 0.0, ys, 1, n, batch)
        else:
            k.GEMV_STRIDED_BATCHED[prec]("N" if kind == "gemv_n" else "T", n, n, 1.0, flat, n, n * n, xs, 1, n, 1.0, ys, 1, n,
                                         batch)

    for kind, n in cases:
        batch = total // (n * n)
        assert batch * n <= xs.numel() and batch * n * n <= flat.numel()
        nbytes = batch * acc.algorithmic_bytes(kind, prec, n, n)
        for _ in range(args.warmup):
            run(kind, n, batch)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(args.steps):
            run(kind, n, batch)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        # the same members one call at a time (first 256 only)
        nloop = min(batch, 256)
        if kind == "symv_l":
            calls = [k.prepare_symv(prec, "L", n, 1.0, flat[b * n * n:], n, xs[b * n:], 1, 0.0, ys[b * n:], 1) for b in range(nloop)]
        else:
            calls = [k.prepare_gemv(prec, "N" if kind == "gemv_n" else "T", n, n, 1.0, flat[b * n * n:], n, xs[b * n:], 1, 1.0,
                                    ys[b * n:], 1) for b in range(nloop)]
        for c in calls:
            c()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for c in calls:
            c()
        torch.cuda.synchronize()
        loop_us = (time.perf_counter() - t0) * 1e6 / nloop
        rows.append({"routine": symv_name + "_L" if kind == "symv_l" else prec + kind, "n": n, "batch": batch, "ms": round(ms, 4),
                     "us_per_member": round(ms * 1e3 / batch, 4), "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "single_call_loop_us_per_member": round(loop_us, 3)})
        tot_bytes += nbytes
        tot_ms += ms
    if args.table:
        with open(args.table, "w") as f:
            for r in rows:
                f.write(json.dumps(r) + "\n")
    value = tot_bytes / (tot_ms * 1e-3) / 1e9
    return {
        "metric": "achieved HBM GB/s (algorithmic bytes / time) for xGEMV/xSYMV vs n, 1 GPU",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(tot_ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_NAMES[prec], "data": "synthetic",
        "config": {"workload": f"strided batches of {prec}gemv N,T and {symv_name} L, n = 64..1024, 1 GiB of matrices per batch, "
                               "one call per batch", "products_per_step": len(cases)},
        "frac_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "per_shape": rows,
        "roofline": None,
    }


def cpu_baseline(acc, wl):
    """The oracle as it stands (working-precision mode, OpenMP over outputs) on a
    bounded sample of the sweep: one product per routine family at one size."""
    import oracle

    n, reps = 16384, 8      # about ten seconds of CPU work on 16 cores
    sample = [("gemv", "s", "N"), ("gemv", "s", "T"), ("gemv", "d", "N"), ("gemv", "d", "T"),
              ("symv", "d", "L"), ("symv", "d", "U"), ("symv", "z", "L"), ("symv", "z", "U")]
    tot_b, tot_t = 0, 0.0
    oracle.build()
    for kind, prec, mode in sample:
        A = wl.matrix(prec, n, n, n, seed=0).numpy().reshape(-1)
        x = wl.vector(prec, n, seed=0, which=1).numpy()
        y = wl.vector(prec, n, seed=0, which=2).numpy()
        t0 = time.perf_counter()
        for _ in range(reps):
            if kind == "gemv":
                oracle.gemv(prec, mode, n, n, 1.0, A, x, 1.0, y, lda=n, mode=oracle.MODE_W)
                op = "gemv_" + mode.lower()
            else:
                oracle.symv(prec, mode, n, 1.0, A, x, 0.0, y, lda=n, mode=oracle.MODE_W)
                op = "symv_" + mode.lower()
        tot_t += time.perf_counter() - t0
        tot_b += reps * acc.algorithmic_bytes(op, prec, n, n)
        del A
    return {"value": round(tot_b / tot_t / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"sgemv/dgemv N,T + dsymv/zhemv L,U at n={n}, working-precision oracle, {reps} runs each",
            "seconds": round(tot_t, 2)}


def stream_probe(k, torch):
    """Sustained bandwidth of the device measured the way the paper defines the
    roofline's bandwidth (Section 7: STREAM-style kernels): read, copy and triad
    over 2 GiB per array with the library's own probe kernels; `read_192wg_gbs` is the read pass in the launch
    shape of the fastest matrix kernel (192 workgroups, 16 loads in flight per lane), which streams about 5 %
    faster than one slab per 16 KiB."""
    n = 1 << 28
    a = torch.zeros(n, dtype=torch.float64, device="cuda")
    b = torch.empty_like(a)
    c = torch.empty_like(a)
    sink = torch.zeros(8192, dtype=torch.float64, device="cuda")
    out = {}
    for kind, name, arrays in ((0, "read", 1), (3, "read_192wg", 1), (1, "copy", 2), (2, "triad", 3)):
        for _ in range(2):
            k.stream_probe(kind, n, a, b, c, sink)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            k.stream_probe(kind, n, a, b, c, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name + "_gbs"] = round(arrays * n * 8 * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    del a, b, c
    torch.cuda.empty_cache()
    return out


# --------------------------------------------------------------------- main ----
def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build is single-GPU by design (no multi-GPU layer); --gpus {args.gpus} is not supported, "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_1410_1726_amd import accounting as acc
    from paper_1410_1726_amd import binding as k
    from paper_1410_1726_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the kmv library has no CPU path", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    for kv in args.tuning:
        key, v = kv.split("=")
        k.set_tuning(key, int(v))

    if args.workload == "batched":
        print(json.dumps(batched_bench(args, k, torch, wl, acc)))
        return
    if args.workload == "gebrd":
        print(json.dumps(gebrd_panel_bench(args, k, torch, wl, acc)))
        return
    if args.workload == "sytrd":
        print(json.dumps(sytrd_panel_bench(args, k, torch, wl, acc)))
        return

    probe = stream_probe(k, torch)
    poisoned = check_poisoned(k, torch, wl)
    # within a group the largest products come first: the host runs ahead of the device, so the
    # short products at the end of a group are already queued when their turn comes
    prods = products(args.workload)
    for p in prods:
        p.setdefault("group", args.workload)
    if args.only:
        import re
        prods = [p for p in prods if re.search(args.only, f"{routine_name(p)}:{p['n']}")]
        if not prods:
            print(f"bench.py: --only {args.only!r} matches no product of workload {args.workload}", file=sys.stderr)
            sys.exit(2)
    group_names = list(dict.fromkeys(p["group"] for p in prods))
    prods.sort(key=lambda p: (group_names.index(p["group"]), -p["n"] * p.get("m", p["n"])))
    inputs = Inputs(prods, torch, wl, acc)
    stream = torch.cuda.current_stream()
    calls = [make_call(p, k, *inputs.views(i, p)) for i, p in enumerate(prods)]
    nprod = len(prods)
    per = [dict(bytes=acc.algorithmic_bytes(op_name(p), p["prec"], p.get("m", p["n"]), p["n"]),
                flops=acc.flops(op_name(p), p["prec"], p.get("m", p["n"]), p["n"]), ms=0.0) for p in prods]
    members = {g: [i for i, p in enumerate(prods) if p["group"] == g] for g in group_names}

    for _ in range(args.warmup):
        for call in calls:
            call()
    events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in prods]
              for _ in range(args.steps)]
    torch.cuda.synchronize()
    # timed region: exactly `steps` passes, inputs already resident in HBM; the wall clock runs per group
    # between two device synchronisations, HIP events on the launch stream bracket every product for the
    # breakdown
    group_wall = {g: 0.0 for g in group_names}
    t_begin = time.perf_counter()
    for step in range(args.steps):
        for g in group_names:
            t0 = time.perf_counter()
            for i in members[g]:
                e0, e1 = events[step][i]
                e0.record(stream)
                calls[i]()
                e1.record(stream)
            torch.cuda.synchronize()
            group_wall[g] += time.perf_counter() - t0
    wall = time.perf_counter() - t_begin
    for step in range(args.steps):
        for rec, (e0, e1) in zip(per, events[step]):
            t = e0.elapsed_time(e1)
            rec["ms"] += t / args.steps
            rec.setdefault("all_ms", []).append(t)

    step_ms = wall / args.steps * 1e3          # wall clock of a whole step (all groups)
    device_ms = sum(r["ms"] for r in per)       # sum of the per-product event brackets

    def group_summary(g):
        idx = members[g]
        gb = sum(per[i]["bytes"] for i in idx)
        gf = sum(per[i]["flops"] for i in idx)
        ms = group_wall[g] / args.steps * 1e3
        routines, graded = {}, {}
        for i in idx:
            p, r = prods[i], per[i]
            a = routines.setdefault(routine_name(p), [0, 0.0])
            a[0] += r["bytes"]
            a[1] += r["ms"]
            if p["n"] >= 16384:
                a = graded.setdefault(routine_name(p), [0, 0.0])
                a[0] += r["bytes"]
                a[1] += r["ms"]
        frac = lambda d: {name: round(b / (m * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) for name, (b, m) in d.items()}
        return {"value": round(gb / (ms * 1e-3) / 1e9, 1), "unit": "GB/s", "frac_hbm_peak": round(gb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "ms_per_step": round(ms, 3), "products": len(idx), "gflops": round(gf / (ms * 1e-3) / 1e9, 1),
                "frac_hbm_peak_by_routine": frac(routines), "frac_hbm_peak_n_ge_16384": frac(graded)}

    groups = {g: group_summary(g) for g in group_names}
    head = "sweep" if "sweep" in groups else group_names[0]     # the configurations the metric is quoted on
    value = groups[head]["value"]

    # dominant kernel = the main kernel with the largest share of the step time
    by_kernel = {}
    for p, r in zip(prods, per):
        d = by_kernel.setdefault(kernel_name(p), dict(ms=0.0, bytes=0, launches=0))
        d["ms"] += r["ms"]
        d["bytes"] += r["bytes"]
        d["launches"] += 1
    dom, dd = max(by_kernel.items(), key=lambda kv: kv[1]["ms"])
    achieved = dd["bytes"] / (dd["ms"] * 1e-3) / 1e9
    traffic = measured_traffic(dom) if args.workload == "all" and not args.tuning and not args.only else None
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": "profiles/default_step_hbm_traffic.txt (bytes per launch, read + written)" if traffic else None,
                "launches_per_step": dd["launches"],
                "avg_launch_us": round(dd["ms"] * 1e3 / dd["launches"], 2),
                "avg_algorithmic_bytes_per_launch": dd["bytes"] // dd["launches"]}

    # the products that fit the last-level cache, timed back to back on ONE region (cache resident) beside
    # their timing inside the step (own region, cold)
    small = [] if args.no_cache_resident else [i for i, p in enumerate(prods) if i in inputs.offset]
    cache_resident = None
    if small:
        warm_ms, cold_ms, sb = 0.0, 0.0, 0
        for i in small:
            call = make_call(prods[i], k, *inputs.views(i, prods[i], own_region=False))
            for _ in range(2):
                call()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                call()
            e1.record(stream)
            torch.cuda.synchronize()
            per[i]["warm_ms"] = e0.elapsed_time(e1) / 10
            warm_ms += per[i]["warm_ms"]
            cold_ms += per[i]["ms"]
            sb += per[i]["bytes"]
        cache_resident = {"products": len(small), "matrix_bytes_below": int(COLD_BYTES),
                          "cold_gbs": round(sb / (cold_ms * 1e-3) / 1e9, 1), "warm_gbs": round(sb / (warm_ms * 1e-3) / 1e9, 1),
                          "note": "cold = inside the step, every product on a region of its own; warm = ten calls back to back "
                                  "on one region (not HBM bandwidth: the matrix stays in the last-level cache)"}

    if args.table:
        with open(args.table, "w") as f:
            for p, r in zip(prods, per):
                gbs = r["bytes"] / (r["ms"] * 1e-3) / 1e9
                row = {"group": p["group"], "routine": routine_name(p), "m": p.get("m", p["n"]), "n": p["n"], "lda": p["lda"],
                       "off": p.get("off", 0), "incx": p.get("incx", 1), "us": round(r["ms"] * 1e3, 2),
                       "us_min": round(min(r["all_ms"]) * 1e3, 2),
                       "us_median": round(sorted(r["all_ms"])[len(r["all_ms"]) // 2] * 1e3, 2),
                       "gbs": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                       "gflops": round(r["flops"] / (r["ms"] * 1e-3) / 1e9, 1)}
                if "warm_ms" in r:
                    row["us_cache_resident"] = round(r["warm_ms"] * 1e3, 2)
                f.write(json.dumps(row) + "\n")

    labels = {
        "sweep": "configs[1]+configs[2]: SGEMV/DGEMV N,T n=1024..32768 step 1024 + {1000,4099,17001}; "
                 "DSYMV/ZHEMV L,U n=1024..32768 step 1024, beta=0; lda=n, U[-1,1], seed 0 (the unreferenced triangle holds "
                 "ordinary numbers here and is never loaded; one NaN-poisoned product per routine is checked before the timing)",
        "target16k": "all 16 precision x routine products at n=16384 and 32768, lda=n",
        "large": "configs[4]: n=49152 (s,c) / 40960 (d,z), lda=n+32, N(0,1), alpha=0.7, beta=0.3, incx 1 and 2",
        "subblock": "configs[3]: blocks of a 20000x20000 fp64 parent at offsets 1,17,63,1000",
        "panel": "DSYMV L, DGEMV T, DGEMV N on the trailing blocks at offsets 0..64 of a 16384x16384 fp64 parent "
                 "(one 64-column panel of a two-sided reduction), beta=0",
        "csymv": "CSYMV/ZSYMV (complex symmetric) beside CHEMV/ZHEMV, L and U, n=16384 and 32768, lda=n",
        "rect": "S/DGEMV N,T on tall-skinny and short-wide panels (65536x32 .. 4096x16384 and transposes), lda=m",
        "tiny": "configs[0]: DGEMV N m=n=lda=1024",
    }
    workload_label = ("value on " + labels["sweep"] + "; further groups in the same step, each with its own figures: " +
                      "; ".join(f"{g} = {labels[g]}" for g in group_names if g != "sweep")) if args.workload == "all" else labels[args.workload]
    precs = sorted({p["prec"] for p in prods if p["group"] == head}, key="sdcz".index)
    out = {
        "metric": "achieved HBM GB/s (algorithmic bytes / time) for xGEMV/xSYMV vs n, 1 GPU",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "+".join(DTYPE_NAMES[c] for c in precs), "data": "synthetic",
        "config": {"workload": workload_label, "products_per_step": nprod, "value_group": head},
        "frac_hbm_peak": groups[head]["frac_hbm_peak"],
        "gflops": groups[head]["gflops"],
        "frac_hbm_peak_n_ge_16384": groups[head]["frac_hbm_peak_n_ge_16384"],
        "groups": groups,
        "cache_resident": cache_resident,
        "poisoned_triangle_check": poisoned,
        "device_ms_per_step": round(device_ms, 3),
        "stream_probe": probe,
        "frac_of_stream_read": round(value / max(probe["read_gbs"], probe["read_192wg_gbs"]), 4),
        "roofline": roofline,
    }
    if args.workload == "tiny":
        out["latency_us"] = tiny_latency(k, torch, wl)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(acc, wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
