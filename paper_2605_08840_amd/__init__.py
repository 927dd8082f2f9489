"""ReST-KV eviction hot path for AMD MI355X: Python binding of librestkv.so."""
from .binding import (  # noqa: F401
    LIB_PATH, RESTKV_BF16, RESTKV_F32, RESTKV_GROUP_MAX, RESTKV_IND_ATTENTION, RESTKV_IND_VALUE_NORM,
    RESTKV_POOL_MAX, RESTKV_TEMPORAL_INV_EMA, RESTKV_TEMPORAL_MEAN, LayerBuffers, RestkvError, RestkvParams, alloc_layer_buffers,
    alloc_workspace, evict_layer, lib, make_params, restkv_compact, restkv_prepare_wo, restkv_score, restkv_score_from_attention,
    restkv_score_smooth, restkv_select, restkv_select_b, restkv_select_static, restkv_select_static_capacity, restkv_smooth, restkv_smooth_b, restkv_debug_force_fp32,
    restkv_stream_reference, restkv_timing_enable, restkv_timing_read, restkv_version, restkv_workspace_bytes, strerror,
)
