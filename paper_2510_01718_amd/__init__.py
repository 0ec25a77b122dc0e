"""BD Attention K/V up-projection for AMD MI355X: thin Python binding over the C-ABI library.

Every step of the path runs in the HIP kernels of libbda.so; this package only marshals
arguments (see `binding`).  Importing it never builds anything; `load()` raises if the library
has not been built (`python -m paper_2510_01718_amd.build`).
"""
from .binding import (  # noqa: F401
    BDA_F32, BDA_F16, BDA_BF16, BDA_F64,
    BASIS_FIRST, BASIS_LAST, BASIS_RESIDUAL_MIN, BASIS_OFFSET_SEARCH, BASIS_EXPLICIT,
    SIDE_NONE, SIDE_Q, SIDE_O,
    BdaError, load, lib_path, exported_symbols,
    bda_prepare, bda_prepare_lowrank, bda_prepare_device, bda_prepare_device_ex, bda_prepare_device_workspace_bytes, bda_prepare_device_static, bda_packed_weights_bytes, bda_pack_weights, bda_kv_project_packed, bda_kv_project, bda_dense_project, bda_lowrank_linear,
    bda_kv_project_backward, bda_kv_project_plan, bda_dense_project_plan, LaunchPlan,
    KERNEL_NONE, KERNEL_GENERAL, KERNEL_MFMA, KERNEL_STREAM, KERNEL_LEAN, KERNEL_DECODE, KERNEL_DUO,
    bda_kv_project_ex, bda_dense_project_ex, bda_kv_project_backward_ex, bda_last_error, bda_version,
)
