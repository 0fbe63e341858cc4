"""MI355X-native parallel prefix-verification (PPV) and fused constrained sampling.

``binding``    ctypes front of the C-ABI library libppv_hip.so (hand-written HIP, gfx950)
``workloads``  seeded synthetic inputs (no arithmetic of the method)
``build``      compiles the library in-tree with hipcc
"""
__all__ = ["binding", "workloads", "build"]
