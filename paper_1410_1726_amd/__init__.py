"""MI355X-native dense matrix-vector products (GEMV / SYMV / HEMV, s/d/c/z).

``paper_1410_1726_amd.binding`` is the ctypes front end of the HIP library
``libkmv.so`` (C ABI in ``include/kmv.h``); ``accounting`` holds the flop /
byte / roofline formulas of the paper's performance model; ``workloads`` the
seeded synthetic inputs; ``build`` compiles the library with hipcc.
Importing the package does not load the library; importing ``binding`` does
and fails loudly when it has not been built.
"""
__all__ = ["accounting", "binding", "build", "workloads"]
