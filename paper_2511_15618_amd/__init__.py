"""MI355X-native predict / verify / commit decode path for hourglass mesh transformers.

Thin ctypes binding over libflashmesh.so (hand-written HIP kernels for gfx950).  PyTorch is
used only to own device memory and the stream; every step of the path runs in the library.
"""
from .binding import FlashMesh, FmConfig, FmStats, load_library, LibraryMissing  # noqa: F401
