"""Seeded synthetic inputs (CSR A, dense B) shared by the tests, the bench and the oracle checks.

This package holds no arithmetic of the SpMM method itself: it only draws
random sparsity patterns and values, rounds them to their storage type and hands
the same bits to whoever asks.
"""
from .configs import (  # noqa: F401
    Workload,
    CONFIG_NAMES,
    make_config,
    random_csr,
    band_csr,
    band_full_csr,
    occupancy_csr,
    column_entries_csr,
    OCCUPANCY_SPEC,
    dense_from_bits,
    to_bits,
    from_bits,
    recast,
    storage_dtype,
    DTYPES_8BIT,
)
