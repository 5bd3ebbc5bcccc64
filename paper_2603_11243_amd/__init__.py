"""MI355X-native gate -> verify -> accept path of CTC-draft self-speculative decoding.

Thin ctypes binding over libssd.so (hand-written HIP for gfx950).  There is no CPU fallback:
importing `paper_2603_11243_amd.binding` raises if the library has not been built.
"""
__all__ = ["binding", "build"]
