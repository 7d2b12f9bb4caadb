"""MI355X-native structured-tensor kernels (StructTensor hot path).

Thin Python binding over the C ABI of ``libstructtensor_hip.so`` (see
``include/structtensor.h``): argument marshalling only.  PyTorch is used for
device memory and streams; every step of the computation runs in the HIP
kernels.  There is no CPU fallback: if the library cannot be loaded, importing
the binding's functions raises.
"""
from .binding import (  # noqa: F401
    Descriptor,
    covar_pr2,
    MTTKRP_FIXED_I,
    MTTKRP_FIXED_IK,
    MTTKRP_FIXED_K,
    STRUCT_DIAG,
    STRUCT_FIXED_I,
    STRUCT_FIXED_J,
    STRUCT_UPPER,
    count_struct,
    expand_band,
    mttkrp_fixed,
    thp_struct,
    ttm_struct,
    StructTensorError,
    count_band,
    count_sym2,
    count_sym3,
    count_sym4,
    expand_sym,
    batax_utri,
    batax_utri_noalloc,
    probe_empty,
    probe_stream,
    lib,
    moment2_sym,
    moment3_sym,
    moment4_sym,
    mttkrp_sym3,
    rank_band,
    rank_sym2,
    rank_sym3,
    rank_sym4,
    ttm_band,
    unrank_band,
    unrank_band_batch,
    unrank_device,
    unrank_sym2,
    unrank_sym2_batch,
    unrank_sym3,
    unrank_sym3_batch,
    unrank_sym4,
    unrank_sym4_batch,
    workspace_bytes,
)
