"""MI355X-native verification step for FlexSpec-style edge-cloud speculative decoding.

`flexverify` (the ctypes binding of libflexverify.so) is imported on first use so that the
seeded input generators in `synth` stay importable on machines without the built library.
"""

__all__ = ["synth", "flexverify"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
