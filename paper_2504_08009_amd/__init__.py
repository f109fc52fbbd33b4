"""Ozaki scheme II FP64 GEMM emulation on MI355X: thin Python binding over liboz2.so (C ABI, include/oz2.h).

Every step of the path runs in the HIP kernels of liboz2.so; this package only marshals arguments.
The library is loaded on first use and a missing build is an error (there is no fallback path).
"""
from .binding import (  # noqa: F401
    OZ2_GEMM_AUTO, OZ2_GEMM_CLASSICAL, OZ2_GEMM_STRASSEN, OZ2_PRODUCT_INT32, OZ2_PRODUCT_RESIDUE_U8, OZ2_SHIFT_CAUCHY_SCHWARZ, OZ2_SHIFT_INT8_PRODUCT, OZ2_SHIFT_MAX,
    Oz2Error, get_moduli, host_crt_element, host_crt_element_digits, host_residues, lib, max_moduli, min_moduli, moduli_for_bits, oz2_dgemm, oz2_dgemm_static, OZ2_STATIC_SCRATCH_BYTES, oz2_dgemm_ex, oz2_init, oz2_dsyrk, oz2_dtrmm,
    oz2_set_kblock, oz2_set_round_sync, oz2_set_shift_mode, oz2_set_product_format, oz2_set_bit_split, oz2_set_nonfinite_check, oz2_set_stage_events, oz2_calibrate_mfma,
    oz2_stage1_convert, oz2_stage2_gemm, oz2_stage3_crt, set_workspace, workspace_bytes, workspace_layout,
    oz2_set_gemm_algorithm, oz2_gemm_algorithm_for, workspace_bytes_strassen, workspace_bytes_preferred,
    Workspace, dgemm, Context,
    OZ2_OPT_SHIFT_MODE, OZ2_OPT_PRODUCT_FORMAT, OZ2_OPT_GEMM_ALGORITHM, OZ2_OPT_KBLOCK, OZ2_OPT_BIT_SPLIT, OZ2_OPT_NONFINITE_CHECK,
)
