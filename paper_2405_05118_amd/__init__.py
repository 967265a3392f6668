"""MI355X-native tiled evaluation of multi-dimensional homomorphisms (md_hom).

The product is the C-ABI library ``libmdh.so`` (HIP kernels for gfx950, declared in
``include/mdh.h``); this package is a thin binding with the same entry-point names
(``mdh_matmul``, ``mdh_stencil``, ``mdh_mcc``, ``mdh_custom_reduce`` ...) that only
marshals arguments.  PyTorch is used for device memory and streams, nothing else.
There is no CPU fallback: if the library is missing, loading fails loudly.
"""
from .binding import (  # noqa: F401
    MDH_CUSTOM_REDUCE,
    MDH_BMATMUL,
    MDH_DOT,
    MDH_MATVEC,
    MDH_SCAN,
    MDH_MATMUL,
    MDH_MCC,
    MDH_STENCIL,
    MdhError,
    TileParams,
    lib,
    mdh_calib_copy,
    mdh_calib_mfma,
    mdh_calib_read,
    mdh_calib_valu,
    mdh_candidate,
    CustomDesc,
    CustomOp,
    custom_desc,
    mdh_custom_candidate,
    mdh_custom_create,
    mdh_custom_default_params,
    mdh_custom_destroy,
    mdh_custom_num_candidates,
    mdh_custom_run,
    mdh_custom_source,
    mdh_custom_validate_params,
    mdh_custom_workspace_size,
    mdh_custom_reduce,
    mdh_default_params,
    mdh_dot,
    mdh_matvec,
    mdh_matmul,
    mdh_matmul_ex,
    mdh_mcc,
    mdh_num_candidates,
    mdh_part_offset,
    mdh_scan,
    mdh_stencil,
    mdh_strerror,
    mdh_tune,
    mdh_validate_params,
    mdh_version,
    mdh_workspace_size,
)
