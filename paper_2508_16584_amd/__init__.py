"""libgg_fp8 for MI355X: padding-free FP8 grouped GEMM with fine-grained block scaling.

Thin Python binding (ctypes) over the C-ABI shared library built from csrc/.
Every step of the computation runs in the library's HIP kernels; this package
only marshals arguments.  There is no CPU fallback: without the built library
`load_library()` raises.
"""
from .binding import (  # noqa: F401
    GGError,
    build_library,
    check_offsets,
    grouped_gemm,
    grouped_gemm_padded,
    grouped_gemm_splitk_noalloc,
    noalloc_max_elements,
    grouped_gemm_swiglu,
    grouped_gemm_wgrad,
    quantize_cols,
    library_path,
    load_library,
    load_probe_library,
    probe_gemm_kstep,
    probe_wgrad_parts,
    probe_hbm,
    probe_issue_mix,
    probe_lds_fetch,
    probe_library_path,
    probe_mfma,
    auto_variant,
    auto_variant_padded,
    num_variants,
    pad,
    padded_rows_cap,
    status_str,
    unpad,
    quantize_rows,
    swiglu_quantize_rows,
    variant_name,
    version,
    workspace_bytes,
)
