"""Seeded synthetic input generators shared by the CPU oracle's tests and the HIP path's
tests and benchmark.

This package holds no arithmetic of the encrypted-convolution method itself (no NTT, no
modular polynomial products, no key switching, no encoding): it only searches for the
NTT-friendly primes that parameterise a workload and draws the random numbers both sides
consume (uniform residues, ternary secrets, rounded Gaussian errors, float messages and
filter weights).  Neither the oracle nor the HIP library is imported from here.
"""
from .params import HEParams, config_params, ntt_primes, is_prime  # noqa: F401
from .sampling import (  # noqa: F401
    make_rng,
    uniform_limbs,
    ternary_secret,
    gaussian_error,
    conv_tensors,
)
