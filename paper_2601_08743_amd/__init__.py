"""MI355X-native TableCache hot path: table-KV stitch + suffix prefill attention.

``paper_2601_08743_amd.binding`` is the ctypes layer over the C-ABI library
(``libtablecache.so``, built from ``csrc/``); importing it fails loudly when the
library has not been built.  ``paper_2601_08743_amd.workloads`` only generates
seeded synthetic inputs and needs neither the library nor a GPU.
"""
__all__ = ["workloads", "binding"]
