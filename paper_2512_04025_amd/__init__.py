"""Pyramid Sparse Attention forward pass for AMD MI355X (gfx950).

Thin Python binding over the C ABI declared in include/psa.h.  Every step runs in the HIP kernels of
libpsa.so; this package only marshals arguments (PyTorch supplies device memory and streams).
"""
from .binding import (  # noqa: F401
    PSA_ALLOC_BUDGET, PSA_CAP_ALL_HEADS, PSA_CAP_PER_HEAD, PSA_ALLOC_QUANTILE, PSA_ALLOC_THRESHOLD, PSA_ALLOC_THRESHOLD_EXCL, PSA_BF16, PSA_EST_MAX, PSA_EST_MEAN,
    PSA_F32, PSA_REP_POOLED, PSA_REP_STRIDED, PsaError, PsaParams, library_path, load_library,
    make_params, psa_allocate_levels, psa_attention_bwd, psa_attention_fwd, psa_attention_fwd_static, psa_query_bwd_sizes, psa_build_pyramid, psa_build_pyramid_cap, psa_dense_ref, psa_hilbert_order, psa_level_cap, psa_permute_tokens,
    psa_probe_copy, psa_probe_mfma, psa_query_sizes, psa_status_str,
)
