"""MI355X-native TokenCarve compression path (arXiv 2503.10501, Section 3.3).

The package is a thin ctypes binding over libtokencarve.so (hand-written HIP for
gfx950, C ABI in include/tokencarve.h).  PyTorch is used only to own device
memory and streams.  There is no CPU fallback: importing `binding` without a
built library raises.
"""
__all__ = ["binding", "build"]
