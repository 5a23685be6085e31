"""MI355X-native budgeted MoE-layer forward (MoE-Spec expert budgeting) behind a C ABI.

``binding``   ctypes marshalling of libmoespec.so (HIP kernels, gfx950)
``build``     compiles the library in-tree with hipcc
``workloads`` seeded synthetic inputs (no method arithmetic)
"""
__all__ = ["binding", "build", "workloads"]
