"""The step bench.py times is replayed from a HIP graph: a captured step (scatter of restored
users, per layer append + attention, gather of the users to offload) must give, on every replay,
exactly what the same calls give eagerly - with the program's own eager work and
synchronisations between the replays, and with inputs that change from replay to replay."""
import numpy as np
import pytest

import mts_workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("deferred", [False, True])
def test_captured_step_replays_equal_the_eager_step(deferred):
    import torch
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd.runtime import DeviceBatch, PagedKVCache, SegmentList
    dev = "cuda:0"
    w = W.custom_workload("graph", 21, "bf16", 3, 4, 64, 16, [700, 90, 300, 0, 1500, 15, 260], [20, 3, 40, 64, 33, 17, 8],
                          miss_users=np.array([1, 4], np.int32), evict_users=np.array([2, 6], np.int32), chunk_tokens=256)
    L, H, D, N = w.layers, w.heads, w.head_dim, w.total_new
    torch.manual_seed(3)
    cache = PagedKVCache(L, w.num_pages, w.page_size, H, D, w.dtype, dev)
    batch = DeviceBatch.from_workload(w, dev)
    ws_bytes = mts.mts_attn_workspace_bytes(cache.desc, batch.meta)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    miss = [int(u) for u in w.miss_users]
    msegs = SegmentList.for_histories(miss, [w.prefix_lens[u] for u in miss], w.chunk_tokens, dev)
    evict = [int(u) for u in w.evict_users]
    esegs = SegmentList.for_histories(evict, [w.total_lens[u] for u in evict], w.chunk_tokens, dev)
    staging = torch.empty(L, msegs.total_tokens * 2 * H * D, device=dev, dtype=torch.bfloat16)
    offload = torch.empty(L, esegs.total_tokens * 2 * H * D, device=dev, dtype=torch.bfloat16)
    q = torch.empty(L, N, H, D, device=dev, dtype=torch.bfloat16)
    k = torch.empty_like(q); v = torch.empty_like(q); out = torch.empty_like(q)
    pool0 = torch.randn(cache.pool.numel() // 2, device=dev, dtype=torch.bfloat16).view(torch.uint8)

    def draw(seed):
        g = torch.Generator(device=dev); g.manual_seed(seed)
        for t in (q, k, v, staging):
            t.copy_(torch.randn(t.shape, device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16))
        cache.pool.view(torch.uint8).copy_(pool0)           # every run starts from the same pool
        out.zero_(); offload.zero_()

    stream = torch.cuda.Stream(device=dev)
    s = stream.cuda_stream
    esize = 2

    def step():
        mts.mts_kv_unpack_layers(cache.desc, 0, L, staging, staging.stride(0) * esize, *msegs.args(), batch.meta, stream=s)
        for l in range(L):
            if deferred:
                mts.mts_attn_incremental_unappended(cache.desc, l, q[l], k[l], v[l], out[l], batch.meta, 0.0, ws, ws_bytes,
                                                    stream=s)
            else:
                mts.mts_kv_append(cache.desc, l, k[l], v[l], batch.meta, stream=s)
                mts.mts_attn_incremental(cache.desc, l, q[l], out[l], batch.meta, 0.0, ws, ws_bytes, stream=s)
        if deferred:
            mts.mts_kv_append_layers(cache.desc, 0, L, k, v, k.stride(0) * esize, batch.meta, stream=s)
        mts.mts_kv_pack_layers(cache.desc, 0, L, offload, offload.stride(0) * esize, *esegs.args(), batch.meta, stream=s)

    def snapshot():
        torch.cuda.synchronize()
        return out.clone(), offload.clone(), cache.pool.clone()

    # eager references for three different inputs
    refs = []
    for seed in (11, 12, 13):
        draw(seed)
        torch.cuda.synchronize()
        step()
        refs.append(snapshot())
    # capture once (the capture itself runs nothing), then replay with fresh inputs each time
    draw(11)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        step()
    for i, seed in enumerate((11, 12, 13, 12)):
        draw(seed)                                           # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        want = refs[(11, 12, 13).index(seed)]
        for name, a, b in zip(("attention output", "packed runs", "pool"), got, want):
            assert torch.equal(a.view(torch.uint8).flatten(), b.view(torch.uint8).flatten()), f"replay {i}: {name} differs"
