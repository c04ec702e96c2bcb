"""MI355X-native hot path of Metis (spectral split + NVFP4 quantize + FP4 GEMMs).

The compute lives in csrc/ (hand-written HIP for gfx950 behind a C ABI declared
in include/metis.h); `metis` is the thin ctypes binding.  Importing this package
does not load the shared library; the first call does, and fails loudly if it
has not been built (python -c "import __graft_entry__ as g; g.build()").
"""
__all__ = ["metis", "workloads"]
