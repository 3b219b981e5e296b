"""MI355X-native SpMM / sparse 3x3 convolution for pruned-weight inference.

`synth` (seeded input generators) imports nothing else.  `sparsert` is the thin
binding over the C-ABI library `libsparsert.so`; it is imported lazily so the
generators stay usable where the HIP library has not been built.
"""

__all__ = ["synth", "sparsert"]


def __getattr__(name):
    if name in ("sparsert", "synth"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
