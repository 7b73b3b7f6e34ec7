"""MI355X-native selective KV recomputation for reused RAG chunk-caches (Cache-Craft hot path).

Thin ctypes binding over libcachecraft.so (HIP, gfx950): argument marshalling only -- every step
of the path runs in the library's kernels.  PyTorch supplies device memory and streams.
"""
from .binding import (CC_BF16, CC_F32, CC_IMPL_AUTO, CC_IMPL_MFMA_NARROW, CC_IMPL_MFMA_WIDE, CC_IMPL_SCALAR,
                      CacheCraftError, Context, FocusTracker, Preloader, chunk_ab, chunk_cci, chunk_reuse, preload_depth,
                      library_path, load_library)

__all__ = ["CC_BF16", "CC_F32", "CC_IMPL_AUTO", "CC_IMPL_MFMA_NARROW", "CC_IMPL_MFMA_WIDE", "CC_IMPL_SCALAR", "CacheCraftError", "Context", "FocusTracker", "Preloader", "chunk_ab", "chunk_cci", "chunk_reuse", "preload_depth",
           "library_path", "load_library"]
