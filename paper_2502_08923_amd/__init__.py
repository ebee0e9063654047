"""CopySpec copy-and-verify step for MI355X (gfx950): HIP kernels behind a C ABI
(`include/copyspec.h`, built into `libcopyspec.so`) and a thin ctypes binding.

    from paper_2502_08923_amd import binding as cs
    cs.load_library()          # raises if the shared library has not been built
"""
from . import binding  # noqa: F401

__all__ = ["binding"]
