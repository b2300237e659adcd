"""MI355X-native Adamas decode path: HIP kernels behind a C ABI (libadamas.so) and a thin
ctypes binding with the same entry-point names (see include/adamas.h)."""

from .binding import (  # noqa: F401
    AdamasError,
    Config,
    EXPORTED_SYMBOLS,
    adamas_decode_step,
    adamas_decode_step_paged,
    adamas_decode_step_stages,
    STAGE_ALL,
    STAGE_SCAN,
    STAGE_SELECT_ATTN,
    VARIANT_L2,
    VARIANT_NO_HADAMARD,
    adamas_encode_keys,
    adamas_full_attn,
    adamas_full_attn_workspace_bytes,
    adamas_encode_query,
    adamas_manhattan_distance,
    adamas_select_topk,
    adamas_sparse_attn,
    adamas_status_string,
    adamas_stream_read,
    adamas_workspace_bytes,
    build_id,
    library,
    library_path,
)
