"""Padded, strided 2-D convolution as one CSR sparse matrix T, built and
applied (SpMV / SpMM) by hand-written HIP kernels for gfx950.

The compute lives in ``libconvspmv.so`` (C ABI declared in
``include/convspmv.h``); ``binding`` marshals torch device pointers into it.
"""
from .binding import (  # noqa: F401
    ConvError,
    ConvMulti,
    ConvPlan,
    conv_csc_build,
    conv_compact_build,
    conv_csr_build,
    conv_dispatch_info,
    conv_csr_build_channels,
    conv_nnz,
    conv_out_shape,
    conv_plan_set_march_min_jobs,
    conv_csr_fill_noalloc,
    conv_spmv,
    conv_spmv_from_csc,
    conv_strerror,
    conv_update_kernel,
    library_path,
)
