"""MI355X-native LoCoCo segment step (hand-written HIP behind a C ABI).

`inputs` holds the seeded synthetic workloads; `binding` is the thin ctypes
layer over the shared library and is imported lazily so that the input
generators can be used where the library has not been built.
"""

__all__ = ["inputs", "binding"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
