"""Build ``libkmv.so`` (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_1410_1726_amd.build

hipcc cross-compiles without a GPU, so this runs anywhere the ROCm toolchain is
installed.  The library is written next to this file.
"""
from __future__ import annotations

import os
import re
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
    # per-kernel register, LDS and scratch figures as compiler remarks: collected into RESOURCES below
    "-Rpass-analysis=kernel-resource-usage",
]
RESOURCES = os.path.join(BUILD, "resource_usage.txt")     # one line per kernel: name vgprs lds_bytes scratch_bytes_per_lane


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the kmv library needs the ROCm toolchain")


def _kernel_resources(remarks: str) -> dict:
    """{mangled kernel name: (VGPRs, LDS bytes per workgroup, scratch bytes per lane)} from the compiler's
    kernel-resource-usage remarks.  Scratch above zero means the kernel spills registers to memory: none of the
    library's kernels does, and tests/test_abi.py keeps it that way."""
    out, name, cur = {}, None, {}
    for ln in remarks.splitlines():
        m = re.search(r"remark: (?:.*: )?Function Name: (\S+)", ln)
        if m:
            name, cur = m.group(1), {}
            continue
        m = re.search(r"remark: (?:.*: )?\s*(VGPRs|LDS Size \[bytes/block\]|ScratchSize \[bytes/lane\]): (\d+)", ln)
        if m and name:
            cur[m.group(1)] = int(m.group(2))
            if len(cur) == 3:
                out[name] = (cur["VGPRs"], cur["LDS Size [bytes/block]"], cur["ScratchSize [bytes/lane]"])
                name = None
    return out


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
        other = [ln for ln in r.stderr.splitlines() if "remark:" not in ln and "-Rpass-analysis" not in ln]
        if verbose and any(ln.strip() for ln in other):
            print("\n".join(other), file=sys.stderr)
        return obj, _kernel_resources(r.stderr)

    with ThreadPoolExecutor(max_workers=6) as ex:
        done = list(ex.map(compile_one, SOURCES))
    objs = [d[0] for d in done]
    tmp = out + ".tmp"
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    os.replace(tmp, out)
    if out == LIB:      # the report describes the default library
        with open(RESOURCES + ".tmp", "w") as f:
            for _, kernels in done:
                for name, (vgprs, lds, scratch) in sorted(kernels.items()):
                    f.write(f"{name} {vgprs} {lds} {scratch}\n")
        os.replace(RESOURCES + ".tmp", RESOURCES)
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
