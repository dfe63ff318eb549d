"""CPU oracle for the GDWS forward pass and its construction -- TEST INFRASTRUCTURE ONLY.

A slow, plain, double-precision implementation written from the paper's
definitions.  It shares no code with the HIP library and must never be imported
by the product package: only the tests, the smoke check and the bench's
cpu_baseline leg use it.
"""
from .gdws import (                                                      # noqa: F401
    build, offsets, chan_of, slices, svd_slices, numerical_rank, truncated_factors,
    expand_weight, weight_error, error_from_sigmas, mego, lego, gamma_from_budget, sparse_g, compact_factors,
    macs_dense, macs_gdws, conv_dense, gdw, pw, duplicate_channels, gdws_forward, gdws_backward,
    add_relu, maxpool, network_forward, round_to, max_threads,
)
