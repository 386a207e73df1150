"""Build ``libkmv.so`` (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_1410_1726_amd.build

hipcc cross-compiles without a GPU, so this runs anywhere the ROCm toolchain is
installed.  The library is written next to this file.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libkmv.so")
SOURCES = ["kmv_symv_real.hip", "kmv_symv_herm.hip", "kmv_symv_csym.hip", "kmv_gemv.hip", "kmv_api.hip",
           "kmv_aux.hip", "kmv_panel.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instructions are unreliable on the target boxes: keep the
    # compiler from forming them
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the kmv library needs the ROCm toolchain")


def build_library(verbose: bool = False, extra_flags=(), out: str | None = None) -> str:
    """Compile every source (always, even when a library exists) and link.
    `extra_flags` / `out` build a variant next to the default library."""
    out = out or LIB
    os.makedirs(BUILD, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(BUILD, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        if verbose and r.stderr.strip():
            print(r.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = out + ".tmp"
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    # python -m paper_1410_1726_amd.build [-DFLAG ...] [-o variant.so]
    args = sys.argv[1:]
    target = None
    if "-o" in args:
        i = args.index("-o")
        target = os.path.abspath(args[i + 1])
        del args[i:i + 2]
    print(build_library(verbose=True, extra_flags=tuple(args), out=target))
