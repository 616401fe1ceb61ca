"""MI355X-native RS-DGC local gradient compressor (hand-written HIP for gfx950).

``paper_2312_17530_amd.binding`` is the ctypes layer over the C-ABI library
``librsdgc.so`` (argument marshalling only); ``paper_2312_17530_amd.synth`` makes the
seeded synthetic workloads.  Importing the package does not load the library; the
binding raises if the library has not been built.
"""
__all__ = ["binding", "synth"]
