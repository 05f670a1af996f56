"""MI355X-native binarized convolution / GEMM (sign-encode, packed im2col,
XOR-popcount GEMM) behind a plain C ABI.

Importing the package does not load the HIP library; ``binding.lib()`` does, and
raises if it has not been built.  ``inputs`` only draws seeded synthetic tensors.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs"]
