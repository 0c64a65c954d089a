"""MI355X-native quantised-expert MoE forward with low-rank compensation (TileQ hot path).

The product is ``libtileq.so`` (hand-written gfx950 HIP kernels behind the C ABI of
``include/tileq.h``).  This package is a thin ctypes binding over it: argument marshalling only;
torch supplies device memory and the stream.  There is no CPU fallback: importing
``paper_2605_09281_amd.binding`` fails loudly if the library has not been built.
"""
from .build import build_library, library_path  # noqa: F401

__all__ = ["build_library", "library_path"]
