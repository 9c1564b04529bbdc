"""MI355X-native batched IVF-PQ and flat vector search (HIP kernels behind a C ABI).

The Python layer only marshals arguments: torch tensors supply device memory
and the current HIP stream; every step of the search runs in libvs.so.
"""
from .binding import (  # noqa: F401
    METRIC_IP,
    METRIC_L2,
    VS_MAX_K,
    IVFPQ,
    VSError,
    lib,
    vs_flat_search,
    vs_refine,
    vs_kmeans,
    vs_ivfpq_train,
    vs_ivfpq_add,
    vs_ivfpq_coarse,
    vs_ivfpq_code_size,
    vs_ivfpq_create,
    vs_ivfpq_destroy,
    vs_ivfpq_get_assignments,
    vs_ivfpq_get_codes,
    vs_ivfpq_get_list_sizes,
    vs_ivfpq_ntotal,
    vs_ivfpq_search,
    vs_last_error,
    vs_profile_enable,
    vs_profile_read,
    vs_set_option,
    vs_counters_read,
    vs_version,
)
