"""MI355X-native hot path of cross-request KV reuse: paged incremental attention and the
KV pack / unpack / append kernels, behind the C ABI of include/mtserve.h."""
from .binding import (  # noqa: F401
    MTS_BF16, MTS_F32, MTS_OK, BatchMeta, CacheDesc, MtsError,
    mts_attn_incremental, mts_attn_incremental_noalloc, MTS_NOALLOC_SCRATCH_BYTES, mts_attn_incremental_staged, mts_attn_incremental_unappended, mts_attn_pointwise,
    mts_attn_pointwise_unappended, mts_attn_unappended_appends, mts_attn_workspace_bytes, mts_attn_set_tuning, AttnTuning,
    MTS_ATTN_KERNEL_AUTO, MTS_ATTN_KERNEL_STREAMING, MTS_ATTN_KERNEL_PREFILL, MTS_ATTN_KERNEL_PLAIN, mts_elem_offset, mts_kv_append, mts_kv_append_layers, mts_kv_pack,
    mts_kv_pack_layers, mts_kv_unpack, mts_kv_unpack_layers, mts_last_error, mts_page_bytes, mts_pages_for, mts_stage_d2h_async,
    mts_stage_h2d_async, mts_diag_stream_read, mts_version, mts_xfer_create, mts_xfer_destroy, mts_xfer_drain,
    mts_xfer_offload_pending_tokens, mts_xfer_offload_submit, mts_xfer_onload_submit,
    mts_xfer_onload_wait_layer, XferConfig, XferRuns, MTS_ERR_BUSY, CacheManager,
)
