"""MI355X-native SpMM over the Insum fixed-length sparse formats (GroupCOO, BlockGroupCOO),
and point-cloud sparse convolution over a kernel map grouped the same way.

Thin Python binding of ``libinsum.so``: the functions below only marshal arguments
(device pointers of torch tensors, sizes, the current HIP stream) into the C ABI declared
in ``include/insum.h``.  Every step of the computation runs in the library's HIP kernels;
there is no CPU or PyTorch fallback, and importing this package fails if the library can
neither be loaded nor built.
"""
from . import api  # noqa: F401
from .api import (  # noqa: F401
    BlockGroupCOO,
    GroupCOO,
    InsumError,
    MapGroupCOO,
    insum_coo_to_blockgroupcoo,
    insum_coo_to_groupcoo,
    insum_choose_group_size,
    insum_default_group_size,
    insum_groupcoo_transpose,
    insum_group_size_candidates,
    insum_indirect_access_cost,
    insum_map_count_groups,
    insum_map_to_groupcoo,
    insum_spconv_groupcoo,
    insum_spconv_groupcoo_workspace_bytes,
    insum_spmm_blockgroupcoo,
    insum_spmm_blockgroupcoo_plan,
    insum_spmm_blockgroupcoo_workspace_bytes,
    insum_spmm_groupcoo,
    insum_spmm_groupcoo_noalloc,
    insum_spmm_groupcoo_transposed,
    insum_spmm_groupcoo_workspace_bytes,
    insum_status_string,
    insum_version,
    library_path,
)
