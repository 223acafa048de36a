"""MI355X-native hot path of LPC-SVRG / ALPC-SVRG (arXiv 1901.08924).

`paper_1901_08924_amd.lpc` binds the C ABI of include/lpc.h (liblpc_hip.so, hand-written HIP for
gfx950).  Importing it loads the library and fails loudly if that is impossible.
"""
__all__ = ["build", "lpc"]
