"""Elastic Cache hot path for AMD MI355X (gfx950): Python binding over the C-ABI library.

The compute lives in ``csrc/`` (hand-written HIP) and is reached through
``libelastic_cache.so``; this package only marshals arguments.  PyTorch is used
for device memory and streams.  Importing the package does not load the library;
the first call does, and fails loudly if it has not been built.
"""
from . import synthetic  # noqa: F401  (numpy-only input recipes)

__all__ = ["synthetic", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
