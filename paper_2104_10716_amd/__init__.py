"""MI355X-native edge-sampled SpMM (ES-SpMM).

Thin binding over the C-ABI library ``libes_spmm.so`` (see ``include/es_spmm.h``):
argument marshalling only -- every step of the computation runs in the HIP
kernels.  PyTorch supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    ES_BUCKET,
    ES_FASTRAND,
    ES_FULL,
    ES_SPMM_STATIC_WS_MAX_ROWS,
    MODES,
    NORMS,
    EsSpmmError,
    es_spmm,
    es_spmm_backward,
    es_spmm_backward_ex,
    es_spmm_backward_pull,
    es_spmm_ex,
    es_launch_opts_t,
    es_spmm_launch_info,
    es_spmm_materialize,
    es_spmm_materialize_transposed,
    es_spmm_max_W,
    es_spmm_norm,
    es_spmm_sample_edges,
    es_spmm_status_string,
    es_spmm_tile_slots,
    es_spmm_transpose_graph,
    es_spmm_validate_csr,
    es_spmm_static_ws,
    es_spmm_workspace_bytes,
    es_spmm_ws,
    library_path,
    load_library,
)
