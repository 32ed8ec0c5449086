"""SinkRouter decode attention for MI355X (gfx950).

``binding`` is the thin ctypes layer over the C-ABI library built from
``csrc/``; ``synth`` builds seeded synthetic inputs.  The binding is loaded on
first use and raises if the HIP library has not been built: there is no CPU
fallback.
"""
__all__ = ["binding", "synth", "build"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
