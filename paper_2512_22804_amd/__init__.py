"""MI355X-native MoR (Mixture of Representations) analyse-select-quantize path.

``binding``   ctypes front end of the C-ABI library ``libmor.so`` (HIP kernels for gfx950);
``build``     compiles that library in-tree with hipcc;
``workloads`` seeded synthetic BF16 operands (no method arithmetic).
"""
__all__ = ["binding", "build", "workloads"]
