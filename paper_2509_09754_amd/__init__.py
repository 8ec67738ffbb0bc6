"""MI355X-native LAVa prefill-end KV-cache eviction path.

`lava` (the ctypes binding over the HIP library) is imported on first attribute access so
that `synth` (input generators, no GPU needed) can be used on its own.
"""
import importlib

__all__ = ["lava", "synth"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
