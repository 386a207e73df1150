"""Tuning sweeps: time one routine under several settings of the library's tuning
keys, with the settings ALTERNATING inside one process.

The paper keeps tuning parameters apart from the kernel templates and sweeps them
coarse to fine (Section 9).  Here the template instances are compiled in and the
keys of kmv_set_tuning pick among them at run time, so a sweep is a loop over
settings.  Alternating matters on this hardware: the device slows by a few per cent
over a minute-long run, so two back-to-back series are not comparable, while
interleaved rounds are (the defaults in the planners were chosen this way).

  python -m paper_1410_1726_amd.tune dsymv_L 16384 symv_unit_tiles=1,2 wg_target=512,768
  python -m paper_1410_1726_amd.tune sgemv_N 8192x65536 gemv_n_splits=0,32,64,128
  python -m paper_1410_1726_amd.tune zhemv_L 40960 lda_pad=32 symv_tiles_per_wave=2,3     (lda = n + 32)
  python -m paper_1410_1726_amd.tune dsymv_L 18999 off=1 lda_pad=1000                     (block at (1, 1), lda = 20000)

A value 0 means "let the library choose".  Prints the median time of every
combination (microseconds, GB/s of algorithmic bytes) and marks the fastest.

  python -m paper_1410_1726_amd.tune auto dgemv_N 16384 [--save best.json]

runs the paper's two stages for one routine and shape without a hand-written
grid: a coarse stage over the routine's kernel-shape keys, then a fine stage
around the best coarse point over its split / workgroup counts, and reports
the best setting next to the library's own choice (optionally as JSON that
`apply(json.load(...))` turns back into tuning values).

  python -m paper_1410_1726_amd.tune table [routine,routine,...] [n,n,...]

runs the automatic mode over routines x square sizes and prints one line per case:
the library's choice, the best setting found and what it would gain (the per-size
table that says where the planners' defaults leave time on the floor).

  python -m paper_1410_1726_amd.tune table --save [routine,...] [n,...]

does the same with the saved table switched off, measures every gain of 3% or more a
second time against the planners' rule, and writes the settings that held up as rows
of csrc/kmv_tuned_table.inc.  The rows are compiled into the library (build again
afterwards): the planners look a square product's size up there before they
fall back on their rules.
"""
from __future__ import annotations

import itertools
import statistics
import sys

import torch

from . import accounting as acc
from . import binding as k
from . import workloads as wl


def _time(call, reps, warm=2):
    for _ in range(warm):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        call()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e3


def sweep(routine: str, m: int, n: int, grid: dict, rounds: int = 5, reps: int = 10, lda_pad: int = 0, off: int = 0):
    """routine like 'dgemv_T', 'zhemv_U', 'ssymv_L'; grid: {key: [values]}; lda = m + off + lda_pad, the matrix is
    the block at (off, off) of its parent.  Returns
    [(settings dict, median microseconds)], in grid order."""
    keys = list(grid)
    combos = [dict(zip(keys, vals)) for vals in itertools.product(*(grid[key] for key in keys))] or [{}]
    return sweep_settings(routine, m, n, combos, rounds, reps, lda_pad, off)


def sweep_settings(routine: str, m: int, n: int, combos: list, rounds: int = 5, reps: int = 10, lda_pad: int = 0,
                   off: int = 0):
    """The same over an explicit list of settings dicts ({} = the library's own choice, saved table included)."""
    prec, name, mode = routine[0], routine[1:5], routine[-1]
    sym = name in ("symv", "hemv")
    lda = m + off + lda_pad
    A = wl.matrix(prec, m + off, n + off, lda, device="cuda")
    if off:
        A = A[off:, off:]        # a sub-block pointer: same leading dimension, any alignment
    lenx, leny = (n, n) if sym else ((n, m) if mode == "N" else (m, n))
    x = wl.vector(prec, lenx, device="cuda")
    y = wl.vector(prec, leny, which=2, device="cuda")
    times = [[] for _ in combos]
    saved = {key: k.get_tuning(key) for key in k.tuning_keys()}
    try:
        for _ in range(rounds):
            for i, combo in enumerate(combos):
                for key in k.tuning_keys():
                    k.set_tuning(key, 0)
                for key, v in combo.items():
                    k.set_tuning(key, v)
                if combo:       # an explicit setting is measured against the planners' rules, not the saved table
                    k.set_tuning("tuned_table", 1)
                # the plan (kernel, splits, workspace layout) is fixed when the call is prepared
                call = (k.prepare_symv(prec, mode, n, 1.0, A, lda, x, 1, 0.0, y, 1) if sym
                        else k.prepare_gemv(prec, mode, m, n, 1.0, A, lda, x, 1, 1.0, y, 1))
                times[i].append(_time(call, reps))
    finally:
        for key, v in saved.items():
            k.set_tuning(key, v)
    return [(combo, statistics.median(t)) for combo, t in zip(combos, times)]


def apply(settings: dict) -> None:
    """Set the tuning keys of a saved result (all other keys back to automatic)."""
    for key in k.tuning_keys():
        k.set_tuning(key, 0)
    for key, v in settings.items():
        k.set_tuning(key, int(v))


def _coarse_grid(routine: str, m: int, n: int) -> dict:
    name, mode = routine[1:5], routine[-1]
    if name == "gemv" and mode == "N":
        return {"gemv_n_row_tiles": [1, 2, 4], "gemv_n_splits": [0, 8, 32, 128]}
    if name == "gemv":
        return {"gemv_t_splits": [0, 1, 2, 4, 8, 16]}
    variants = [2] + ([3] if n <= 4096 else [])
    return {"symv_variant": variants, "symv_tiles_per_wave": [1, 2, 3, 4], "symv_unit_tiles": [1, 2]}


def _fine_grid(routine: str, best: dict) -> dict:
    name, mode = routine[1:5], routine[-1]
    fixed = {key: [v] for key, v in best.items()}
    if name == "gemv" and mode == "N":
        s0 = best.get("gemv_n_splits", 0)
        if s0 <= 0:
            return {}
        around = sorted({max(1, min(256, int(round(s0 * f)))) for f in (0.5, 0.75, 0.875, 1.0, 1.125, 1.25, 1.5, 2.0)})
        fixed["gemv_n_splits"] = around
        return fixed
    if name == "gemv":
        return {}
    if best.get("symv_variant") == 2:
        fixed["wg_target"] = [0, 256, 512, 768]
        return fixed
    return {}


def auto(routine: str, m: int, n: int, rounds: int = 3, reps: int = 8):
    """Coarse stage, then a fine stage around its best point.  Returns (best settings, microseconds,
    microseconds of the library's own choice)."""
    default_us = sweep(routine, m, n, {}, rounds, reps)[0][1]
    coarse = sweep(routine, m, n, _coarse_grid(routine, m, n), rounds, reps)
    best, best_us = min(coarse, key=lambda r: r[1])
    stages = [("coarse", coarse)]
    fine_grid = _fine_grid(routine, best)
    if fine_grid:
        fine = sweep(routine, m, n, fine_grid, rounds, reps)
        stages.append(("fine", fine))
        fb, fus = min(fine, key=lambda r: r[1])
        if fus < best_us:
            best, best_us = fb, fus
    return best, best_us, default_us, stages


TABLE_ROUTINES = tuple(f"{p}gemv_{t}" for p in "sdcz" for t in ("N", "C" if p in "cz" else "T")) + \
    tuple(f"{p}{'hemv' if p in 'cz' else 'symv'}_{u}" for p in "sdcz" for u in "LU")
TABLE_SIZES = (2048, 4096, 8192, 12288, 16384, 24576, 32768)
SAVE_GAIN = 0.03           # a setting enters the saved table when it beats the planner's rule by this much, twice
TABLE_FILE = "csrc/kmv_tuned_table.inc"
ROW_FIELDS = ("gemv_n_splits", "gemv_n_row_tiles", "gemv_t_splits", "symv_variant", "symv_tiles_per_wave", "symv_unit_tiles",
              "wg_target")


CLASS_WIDTHS = (16, 64)    # a row serves n -+ n/16 if it holds up at both ends, else n -+ n/64, else n alone


def _size_class(n, width):
    """[lo, hi) around the measured size n."""
    return n - n // width, n + n // width + 1


def _op(routine):
    return routine[-1] if routine[1:5] in ("symv", "hemv") else ("N" if routine[-1] == "N" else "T")


def _row_text(routine, n, width, settings):
    op = _op(routine)
    lo, hi = _size_class(n, width)
    vals = ", ".join(str(int(settings.get(f, 0))) for f in ROW_FIELDS)
    return f"    {{'{op}', '{routine[0]}', {lo}, {hi}, {vals}}},   // {routine} n = {n}"


def table(routines=TABLE_ROUTINES, sizes=TABLE_SIZES, out=sys.stdout, save=False):
    """One line per (routine, n): library's choice vs the best setting the automatic mode finds.  With `save` the
    library's choice is taken with the saved table off, and the settings that beat it twice become table rows."""
    op_of = {"gemv": lambda r: "gemv_" + ("n" if r[-1] == "N" else "t"), "symv": lambda r: "symv_l", "hemv": lambda r: "hemv_l"}
    print(f"{'routine':9s} {'n':>6s} {'library us':>11s} {'GB/s':>8s} {'best us':>9s} {'gain':>6s}  best settings", file=out)
    rows = []
    rule = {"tuned_table": 1}
    for routine in routines:
        for n in sizes:
            if routine[0] == "z" and n > 24576:      # 32768^2 complex doubles are 17 GB: skipped to keep the run short
                continue
            best, best_us, default_us, _ = auto(routine, n, n)
            if save:
                default_us = sweep_settings(routine, n, n, [rule], 3, 8)[0][1]
            note = ""
            if save and best and default_us / best_us - 1 >= SAVE_GAIN:
                # second measurement, rule and candidate alternating
                (_, r_us), (_, b_us) = sweep_settings(routine, n, n, [{"tuned_table": 1}, best], 5, 8)
                if r_us / b_us - 1 >= SAVE_GAIN:
                    # the row will serve a class of sizes: it must not lose at the ends of the class
                    note = ""
                    for width in CLASS_WIDTHS:
                        lo, hi = _size_class(n, width)
                        ends = []
                        for ne in (lo, hi - 1):
                            (_, re_us), (_, be_us) = sweep_settings(routine, ne, ne, [{"tuned_table": 1}, best], 3, 8)
                            ends.append(100 * (re_us / be_us - 1))
                        note += f" ends {lo}: {ends[0]:+.1f}% {hi - 1}: {ends[1]:+.1f}%"
                        if min(ends) >= -1.0:
                            rows.append(_row_text(routine, n, width, best))
                            note = f"  saved for [{lo}, {hi}) (second measurement {100 * (r_us / b_us - 1):+.1f}%,{note})"
                            break
                    else:
                        # the split and tile counts that win depend on how the size divides into tiles
                        rows.append(f"    {{'{_op(routine)}', '{routine[0]}', {n}, {n + 1}, "
                                    + ", ".join(str(int(best.get(f, 0))) for f in ROW_FIELDS) + f"}},   // {routine} n = {n}")
                        note = f"  saved for n = {n} alone (second measurement {100 * (r_us / b_us - 1):+.1f}%,{note})"
                else:
                    note = f"  not saved (second measurement {100 * (r_us / b_us - 1):+.1f}%)"
            nbytes = acc.algorithmic_bytes(op_of[routine[1:5]](routine), routine[0], n, n)
            text = " ".join(f"{key}={v}" for key, v in best.items()) or "(defaults)"
            print(f"{routine:9s} {n:6d} {default_us:11.1f} {nbytes / default_us / 1e3:8.1f} {best_us:9.1f} "
                  f"{100 * (default_us / best_us - 1):+5.1f}%  {text}{note}", file=out, flush=True)
    return rows


def write_rows(rows, path=None):
    import os
    path = path or os.path.join(os.path.dirname(os.path.abspath(__file__)), TABLE_FILE)
    with open(path, "w") as f:
        f.write("// Written by: python -m paper_1410_1726_amd.tune table --save\n")
        f.write("// {routine, precision, n_lo, n_hi, " + ", ".join(ROW_FIELDS) + "}; 0 = the planner's rule\n")
        for r in rows:
            f.write(r + "\n")
    return path


def main(argv):
    if argv and argv[0] == "table":
        save = "--save" in argv
        out_path = None
        if save:
            i = argv.index("--save")
            del argv[i]
        if "--out" in argv:
            i = argv.index("--out")
            out_path = argv[i + 1]
            del argv[i:i + 2]
        routines = tuple(argv[1].split(",")) if len(argv) > 1 and argv[1] else TABLE_ROUTINES
        sizes = tuple(int(v) for v in argv[2].split(",")) if len(argv) > 2 else TABLE_SIZES
        rows = table(routines, sizes, save=save)
        if save:
            print(f"{len(rows)} rows written to {write_rows(rows, out_path)}; build the library again to compile them in")
        return 0
    if len(argv) < 2:
        print(__doc__)
        return 2
    if argv[0] == "auto":
        save = None
        if "--save" in argv:
            i = argv.index("--save")
            save = argv[i + 1]
            del argv[i:i + 2]
        routine, shape = argv[1], argv[2]
        m, n = (int(v) for v in shape.split("x")) if "x" in shape else (int(shape), int(shape))
        best, best_us, default_us, stages = auto(routine, m, n)
        for label, res in stages:
            print(f"{label} stage:")
            for combo, us in res:
                print("  " + " ".join(f"{key}={v}" for key, v in combo.items()) + f"   {us:.1f} us")
        gain = 100 * (default_us / best_us - 1)
        print(f"{routine} {m}x{n}: library's choice {default_us:.1f} us; best found {best_us:.1f} us ({gain:+.1f}%) with {best}")
        if save:
            import json
            with open(save, "w") as f:
                json.dump({"routine": routine, "m": m, "n": n, "settings": best, "us": best_us, "default_us": default_us}, f)
        return 0
    routine, shape = argv[0], argv[1]
    m, n = (int(v) for v in shape.split("x")) if "x" in shape else (int(shape), int(shape))
    grid, lda_pad, off = {}, 0, 0
    for spec in argv[2:]:
        key, vals = spec.split("=")
        if key == "lda_pad":          # not a tuning key: the matrix gets the leading dimension m + off + lda_pad
            lda_pad = int(vals)
            continue
        if key == "off":              # not a tuning key: the matrix is the block at (off, off) of its parent
            off = int(vals)
            continue
        grid[key] = [int(v) for v in vals.split(",")]
    res = sweep(routine, m, n, grid, lda_pad=lda_pad, off=off)
    op = {"gemv": "gemv_" + routine[-1].lower(), "symv": "symv_l", "hemv": "hemv_l"}[routine[1:5]]
    nbytes = acc.algorithmic_bytes(op, routine[0], m, n)
    best = min(us for _, us in res)
    print(f"{routine} {m}x{n} on {torch.cuda.get_device_name(0)}")
    for combo, us in res:
        text = " ".join(f"{key}={v}" for key, v in combo.items()) or "(defaults)"
        print(f"  {text:50s} {us:10.1f} us {nbytes / us / 1e3:9.1f} GB/s{'  <- fastest' if us == best else ''}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
