"""MI355X-native binary HDC hot path (arXiv 2206.04746): thin Python binding over libhdc.so.

Every step of the path runs in the HIP kernels of ``csrc/``; this package only marshals
arguments (PyTorch tensors supply device memory and the stream).  There is no CPU fallback:
importing :mod:`paper_2206_04746_amd.binding` fails loudly if the library has not been built.
"""
__all__ = ["binding", "build"]
