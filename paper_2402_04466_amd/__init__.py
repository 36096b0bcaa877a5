"""MI355X-native per-frame hot path of concurrent tool-tracking application streams.

The product is ``libhs.so`` (C ABI declared in ``include/hs.h``, HIP kernels for gfx950).
This package is the thin ctypes binding over it (``api``: same names, argument marshalling
only) plus a small harness (``harness``) that uses PyTorch for device memory.

Importing the package does not load the library; the first API call does, and fails
loudly if ``libhs.so`` has not been built (``python -m paper_2402_04466_amd.build``).
"""
from .api import *  # noqa: F401,F403
from . import api

__all__ = list(api.__all__)
