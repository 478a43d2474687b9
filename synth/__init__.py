"""Seeded synthetic inputs for the SpMM hot path.

This package only draws random matrices (positions, values, dense operands) and
rounds them to a storage type.  It contains none of the method's arithmetic: no
format conversion, no group-size rule, no SpMM.  Both the CPU oracle's tests and
the HIP path's tests/bench take their inputs from here.
"""
from .workloads import (  # noqa: F401
    CONFIG_NAMES,
    bounded_zipf_kmax,
    bounded_zipf_sample,
    make_config,
    random_block_coo,
    random_coo,
    round_to_dtype,
    storage_array,
    surface_kernel_map,
    voxel_kernel_map,
    zipf_rows_coo,
)
