"""FP64 GEMM emulated on the gfx950 INT8 matrix cores (Ozaki scheme, ozIMMU_H form).

`ozimmu` (the binding to the C-ABI HIP library) is imported lazily so that the
input generators can be used on machines without the built library.
"""

__all__ = ["inputs", "ozimmu"]


def __getattr__(name):
    if name in ("ozimmu", "inputs"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
