"""MI355X-native paged decode attention and KV-block migration (gfx950).

The compute lives in the C-ABI shared library built from ``csrc/``; ``binding``
marshals arguments for it and ``workloads`` makes seeded synthetic inputs.
Importing the package does not load the library; the first call through
``binding`` does, and raises if it has not been built.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding", "build"]


def __getattr__(name):
    if name in ("binding", "build"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
