"""MI355X-native homomorphic convolution layer over RNS-CKKS ciphertexts.

The product is the C-ABI library built from csrc/ (see include/he_mi355x.h); `binding`
exposes the same entry points on torch device tensors.  Importing this package does not load
the library; `binding.load()` does, and fails loudly if it has not been built.
"""
__all__ = ["binding", "build"]
