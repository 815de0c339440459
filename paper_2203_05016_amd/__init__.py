"""MI355X-native Shfl-BW sparse-weight x dense-activation product (linear
layers and implicit-GEMM convolution) behind a C-ABI library.

``paper_2203_05016_amd.binding`` is the thin ctypes layer over the library;
``paper_2203_05016_amd.synth`` draws seeded synthetic inputs and holds no
arithmetic of the method.  The library is loaded on first use and its
absence is an error: there is no CPU fallback.
"""
__all__ = ["binding", "synth"]
