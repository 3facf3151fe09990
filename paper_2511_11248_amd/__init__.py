"""MI355X-native table-lookup mixed-precision matmul (the hot path of T-MAN, arxiv 2511.11248).

Thin binding over the C-ABI library ``libtman.so`` (see ``include/tman.h``): the functions here have
the same names as the C entry points and only marshal arguments; every step runs in HIP kernels.
"""
from .api import (  # noqa: F401
    Shape,
    TmanError,
    library_path,
    tman_packed_bytes,
    tman_lut_bytes,
    tman_mpgemv_workspace_bytes,
    tman_mpgemm_workspace_bytes,
    tman_pack_weights,
    tman_unpack_weights,
    tman_build_lut,
    tman_build_lut_batch,
    tman_mpgemv,
    tman_mpgemm,
    tman_noalloc_init,
    tman_check_packed,
    tman_device_status,
    tman_mpgemv_noalloc,
    tman_mpgemm_tile_rows,
    tman_mpgemm_batch_prepare,
    tman_mpgemm_batch_run,
    bound_mpgemm_batch_run,
    tman_mpgemv_batch_desc_bytes,
    tman_mpgemv_batch_prepare,
    tman_mpgemv_batch_run,
    tman_mpgemv_x,
    tman_mpgemv_x_batch_prepare,
    tman_mpgemv_x_batch_run,
    bound_build_lut_batch,
    bound_mpgemv_x_batch_run,
    bound_mpgemv_batch_run,
    tman_status_string,
    tman_layout_version,
)
