"""MI355X-native MetaSD hot path: thin Python binding over the C-ABI library (libmetasd.so).

Everything the method computes runs in the HIP kernels of ``csrc/``; this package only marshals
arguments and uses PyTorch to own device memory and the stream.  There is no CPU fallback: if the
library is missing or no GPU is present the calls raise.
"""
from .binding import (MetaSD, MetaSDError, accept_logits, accept_logits_noalloc, ACCEPT_NOALLOC_MAX_ITEMS, lib_path, load_library, pack_weight, philox_words,
                      sample_logits, stream_read, STREAM_READ_SINK_WORDS, EXPORTS)

__all__ = ["MetaSD", "MetaSDError", "accept_logits", "accept_logits_noalloc", "ACCEPT_NOALLOC_MAX_ITEMS", "sample_logits", "philox_words", "stream_read", "STREAM_READ_SINK_WORDS", "pack_weight", "load_library",
           "lib_path", "EXPORTS"]
