"""MI355X-native surrogate-gradient BPTT for layered LIF spiking networks.

The package is a thin ctypes binding over the C ABI declared in include/snn.h
(libsnn_hip.so, built from csrc/ by build.py).  Every step of the training path
runs in the library's HIP kernels; Python only marshals arguments.
"""
from .binding import (SNN, SnnError, load_library, library_path, SURROGATES, PRECISIONS,  # noqa: F401
                      TENSORS, STEPS, KERNELS, OPTIONS, weight_grad_static)
