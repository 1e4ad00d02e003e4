"""CPU oracle for the cached-prefix incremental-attention path.

TEST INFRASTRUCTURE ONLY.  Nothing under this package is part of the product:
only the test-suite, the smoke check and the benchmark's ``cpu_baseline`` leg
may import it.  It shares no code, tables or helpers with the HIP path and is
written directly from the paper's statement of the method.

Pinned functions (see tests/test_oracle_*.py): page arithmetic, unpack, append,
pack, attn_incremental, full_recompute, attn_pointwise, full_recompute_pointwise.
No function here is "parity unpinned"; attn_pointwise follows a definition this build
states itself (the paper prints none), and its pins hold it to that definition.

oracle/cache_model.py is the plain model of the host-side cache manager (LRU, page counts,
locking, offload trigger); it is pinned by hand-worked traces and the paper's page arithmetic
in tests/test_cache_manager.py and imported from there directly.
"""
from .mts_oracle import (  # noqa: F401
    PagedStore,
    pages_for,
    store_bytes,
    onload_pages,
    kv_bytes_per_token,
    attended_pairs,
    decode_values,
    unpack,
    append,
    pack,
    attn_incremental,
    full_recompute,
    attn_pointwise,
    full_recompute_pointwise,
)
