"""Decode attention with asynchronized softmax (FlashDecoding++, arXiv
2311.01282, Section 3) for MI355X: hand-written gfx950 HIP kernels behind the
C-ABI library ``libfdattn`` plus a thin ctypes binding.

``fdattn`` (the binding) is imported lazily so that ``synth`` (seeded input
generation, no GPU code) can be used without the compiled library.
"""


def __getattr__(name):
    if name == "fdattn":
        import importlib
        return importlib.import_module(__name__ + ".fdattn")
    raise AttributeError(name)
