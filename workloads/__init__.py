"""Seeded synthetic inputs shared by the oracle tests and the GPU tests.

This package only *draws* inputs (sparsity patterns, values, dense operands)
and rounds them to the storage type.  It contains none of the method's
arithmetic: no SpMM, no SDDMM, no format conversion.
"""
from .generators import (  # noqa: F401
    Csr,
    Dense,
    CONFIG_NAMES,
    make_config,
    stream,
    round_to_bits,
    bits_to_f64,
    csr_from_coo,
    uniform_fixed_degree,
    rmat,
    stencil5,
    lognormal_degree,
    dense,
    random_csr,
)
