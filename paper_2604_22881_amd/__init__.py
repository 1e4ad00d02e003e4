"""MI355X-native hot path of cross-request KV reuse: paged incremental attention and the
KV pack / unpack / append kernels, behind the C ABI of include/mtserve.h."""
from .binding import (  # noqa: F401
    MTS_BF16, MTS_F32, MTS_OK, BatchMeta, CacheDesc, MtsError,
    mts_attn_incremental, mts_attn_pointwise, mts_attn_workspace_bytes, mts_elem_offset, mts_kv_append, mts_kv_pack,
    mts_kv_unpack, mts_last_error, mts_page_bytes, mts_pages_for, mts_stage_d2h_async,
    mts_stage_h2d_async, mts_version,
)
