"""MI355X-native (gfx950, hand-written HIP) implementation of DART's drafting step.

Thin ctypes binding over libdart.so (see include/dart.h).  Every step of the path --
draft forward, top-k, N-gram lookup, tree pruning -- runs in the library's HIP kernels;
this package only marshals arguments.  PyTorch supplies device memory and streams.
There is no CPU fallback: if the library has not been built, loading raises.
"""
from .binding import (DartError, DraftContext, NgramTable, PruneParams, library_path,
                      load_library, bf16_bits_to_tensor, tree_verify_greedy, topk_static, debug_stream_read,
                      EXPORTED_SYMBOLS, DEBUG_SYMBOLS)

__all__ = ["DartError", "DraftContext", "NgramTable", "PruneParams", "library_path",
           "load_library", "bf16_bits_to_tensor", "tree_verify_greedy", "topk_static", "debug_stream_read", "EXPORTED_SYMBOLS", "DEBUG_SYMBOLS"]
