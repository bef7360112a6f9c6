"""MI355X-native forward pass of one MoE++ layer (arXiv 2410.07348).

Thin Python binding over the C ABI of libmoepp.so (include/moepp.h): argument
marshalling only.  PyTorch provides device memory and streams; every step of
the layer runs in the library's HIP kernels.  There is no CPU fallback: if the
library cannot be loaded, importing the binding's functions raises.
"""
from .binding import (Layer, Desc, MoeppError, load_library, lib_path, F32, BF16,
                      KERNEL_NAMES, EXPORTS, mfma_ceiling, stream_ceiling, layer_forward_static,
                      STATIC_SCRATCH_BYTES)

__all__ = ["Layer", "Desc", "MoeppError", "load_library", "lib_path", "F32", "BF16",
           "KERNEL_NAMES", "EXPORTS", "mfma_ceiling", "stream_ceiling", "layer_forward_static",
           "STATIC_SCRATCH_BYTES"]
