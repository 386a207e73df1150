"""The tuning tool's automatic mode and the compiled-in table of measured settings
(Section 9: coarse and fine sweeps over tuning parameters kept apart from the kernels):
whatever setting the sweep picks, and whatever row the planners take from the table,
the product still agrees with the oracle."""
import os
import re

import pytest
import torch

from paper_1410_1726_amd import binding as kmv
from paper_1410_1726_amd import tune
from paper_1410_1726_amd import workloads as wl

from gpu_util import check, gemv_case, symv_case

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def reset():
    for key in kmv.tuning_keys():
        kmv.set_tuning(key, 0)


def run_case(routine, n, sample=None, seed=3):
    prec, name, mode = routine[0], routine[1:5], routine[-1]
    if name == "gemv":
        _, err, _ = gemv_case(prec, mode, n, n, 0.75, -0.5, lda=n, seed=seed, sample=sample)
    else:
        _, err, _ = symv_case(prec, mode, n, 0.75, -0.5, lda=n, seed=seed, sample=sample)
    return err


@pytest.mark.parametrize("routine,n", [("dgemv_N", 3072), ("zhemv_L", 2560)])
def test_automatic_mode_picks_a_setting_that_agrees_with_the_oracle(routine, n):
    try:
        best, best_us, default_us, stages = tune.auto(routine, n, n, rounds=2, reps=3)
        assert [label for label, _ in stages][0] == "coarse" and best_us > 0 and default_us > 0
        # the best point is the fastest of the stage it came from
        assert best_us == min(us for _, res in stages for _, us in res)
        assert all(kmv.get_tuning(key) == 0 for key in kmv.tuning_keys()), "the sweep must restore the caller's values"
        tune.apply(best)
        check(routine[0], run_case(routine, n), f"{routine} n={n} under {best}")
    finally:
        reset()


def table_rows():
    text = open(os.path.join(ROOT, "paper_1410_1726_amd", "csrc", "kmv_tuned_table.inc")).read()
    return [(m.group(1), m.group(2), int(m.group(3)), int(m.group(4)))
            for m in re.finditer(r"\{'(\w)', '(\w)', (\d+), (\d+),", text)]


def test_products_planned_from_the_table_agree_with_the_oracle():
    """every row of the compiled-in table: the product at the row's smallest and largest size, planned by the
    library itself (the row applies: square, lda = n), against the oracle on sampled outputs"""
    rows = table_rows()
    names = {("N", False): "gemv_N", ("N", True): "gemv_N", ("T", False): "gemv_T", ("T", True): "gemv_C"}
    try:
        reset()
        for op, prec, lo, hi in rows:
            cplx = prec in "cz"
            routine = prec + (names[(op, cplx)] if op in "NT" else ("hemv_" if cplx else "symv_") + op)
            for n in sorted({lo, hi - 1}):
                assert kmv.tuned_settings(prec, op, n) is not None
                sample = wl.sample_indices(n, 32, 5).numpy()
                check(prec, run_case(routine, n, sample=sample), f"{routine} n={n} planned from the table")
                torch.cuda.empty_cache()
        # and one size with the table switched off: the planners' rules alone
        if rows:
            op, prec, lo, hi = rows[0]
            kmv.set_tuning("tuned_table", 1)
            assert kmv.tuned_settings(prec, op, lo) is None
    finally:
        reset()
