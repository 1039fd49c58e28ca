"""MI355X-native binary (+-1 x +-1) convolution hot path of BCNN.

``binding`` is the Python face of the C ABI in include/bcnn.h (libbcnn.so, HIP
kernels for gfx950); ``workloads`` draws the seeded synthetic tensors;
``build`` compiles the library.
"""
from . import workloads  # noqa: F401

__all__ = ["binding", "build", "workloads"]
