"""Entropy Adaptive Decoding on AMD MI355X: thin Python binding of the C-ABI library.

Everything the method computes runs in the HIP kernels of `libead.so`; this package
only marshals arguments (ctypes) and borrows PyTorch for device memory and streams.
There is no CPU fallback: loading fails loudly if the library has not been built.
"""
from .binding import (EAD, BITS, NATS, SMALL, LARGE, EadError, Gate, entropy_argmax, lib,  # noqa: F401
                      exported_symbols)
