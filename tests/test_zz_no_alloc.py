"""mts_attn_incremental_noalloc (the entry point for callers that cannot allocate: its split-kv
partials live in a device array the library owns) against mts_attn_incremental on the same
inputs, through the C ABI: two calls in a row on the shared buffer, the second with a smaller
batch, and the refusal of shapes the buffer cannot hold.  Collected last on purpose."""
import numpy as np
import pytest

import mts_workloads as W
from helpers import as_values, draw_step_data

pytestmark = pytest.mark.gpu

# bf16 inputs, fp32 accumulation: max|a - b| <= 2e-2 * max|b| per (user, head) tile
REL_TOL = 2e-2


def _both(w):
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    data = draw_step_data(w, layers=[0])
    step = G.GpuStep(w, fill_byte=0xFF)
    step.unpack_histories(data, 0)
    step.append(data, 0)
    ref = as_values(step.attention(data, 0))                       # caller-provided workspace
    q = G.to_dev(data["q"][0])
    out = torch.full((max(w.total_new, 1), w.heads, w.head_dim), -1, dtype=q.dtype, device=G.DEV)
    mts.mts_attn_incremental_noalloc(step.cache.desc, 0, q, out, step.batch.meta)
    torch.cuda.synchronize()
    got = as_values(G.to_host(out[:w.total_new], w.np_dtype))
    return got, ref


def _compare(w, got, ref):
    assert np.isfinite(got).all()
    for u in range(w.batch):
        lo, hi = int(w.new_indptr[u]), int(w.new_indptr[u + 1])
        for h in range(w.heads):
            g, r = got[lo:hi, h], ref[lo:hi, h]
            if r.size:
                assert np.abs(g - r).max() <= REL_TOL * max(np.abs(r).max(), 1e-30), (u, h)
    # same kernels, same deterministic merge order: the two results are in fact the same bits
    assert np.array_equal(got, ref)


def test_two_calls_in_a_row_second_smaller():
    # many users with ragged histories: most wavefront shares cut a (query tile, head), so the
    # library-owned buffer carries partials in both calls
    rng = np.random.default_rng(4242)
    P1 = rng.integers(100, 3000, size=40).tolist()
    n1 = rng.integers(1, 65, size=40).tolist()
    big = W.custom_workload("noalloc_big", 31, "bf16", 1, 8, 64, 16, P1, n1, chunk_tokens=512)
    got, ref = _both(big)
    _compare(big, got, ref)
    small = W.custom_workload("noalloc_small", 32, "bf16", 1, 4, 128, 16, [700, 0, 333, 64], [17, 40, 1, 9],
                              chunk_tokens=256)
    got, ref = _both(small)
    _compare(small, got, ref)


def test_refuses_shapes_beyond_the_buffer():
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    # 64-query tiles at D = 128 on a launch of 1024 wavefronts need more than the buffer holds
    w = W.custom_workload("noalloc_huge", 33, "bf16", 1, 8, 128, 16, [60000] * 8, [64] * 8, chunk_tokens=1024)
    desc = mts.CacheDesc(0x1000, 0, mts.MTS_BF16, 1, w.num_pages, 16, 8, 128)
    desc.layer_stride_bytes = w.num_pages * mts.mts_page_bytes(desc)
    batch = G.DeviceBatch.from_workload(w, G.DEV)
    assert mts.mts_attn_workspace_bytes(desc, batch.meta) > mts.MTS_NOALLOC_SCRATCH_BYTES
    q = torch.zeros(w.total_new, 8, 128, dtype=torch.int16, device=G.DEV)
    with pytest.raises(mts.MtsError) as e:
        mts.mts_attn_incremental_noalloc(desc, 0, q, q, batch.meta)      # refused before any launch
    assert e.value.code == mts.binding.MTS_ERR_WORKSPACE
    assert "scratch" in str(e.value)
