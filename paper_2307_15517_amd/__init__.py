"""MXInt block quantizer and MXInt x MXInt GEMM/GEMV for MI355X (gfx950).

The compute lives in a C-ABI shared library built from ``csrc/``; ``mx`` is a thin
binding with the same entry-point names.  ``inputs`` draws the synthetic workloads.
The binding is imported lazily so that ``inputs`` can be used without the library.
"""


def __getattr__(name):
    if name == "mx":
        import importlib
        return importlib.import_module(__name__ + ".mx")
    raise AttributeError(name)
