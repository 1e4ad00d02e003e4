"""The host_staging workload at its full size with the link in the loop, in the stream structure
bench.py times for it (Alg. 1 steps 7, 8.2-8.4, 9; Sec. 4.2, 4.4): 256 users, 4 layers; the 4
cache-miss users' histories lie in pinned host memory in host-chunk runs and are copied
(hipMemcpyAsync) and scattered layer by layer on a side stream, one event per layer; the compute
stream runs the cached users' append + attention of a layer meanwhile, waits for the layer's
event, then runs the restored users'; afterwards the 4 users chosen for offload are gathered and
copied back to pinned memory.

Checked against the oracle: attention of every restored user, every offloaded user and two more
cached users on all heads and all layers (their K/V/Q are seeded host data; everybody else keeps a
device-side draw), and the offload round trip bit for bit."""
import dataclasses

import numpy as np
import pytest

import mts_workloads as W
import oracle
from helpers import as_values

pytestmark = pytest.mark.gpu


def test_host_staging_full_size_through_pinned_memory():
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd.runtime import DeviceBatch, PagedKVCache, SegmentList

    w = W.make_workload("host_staging")
    L, H, D, S = w.layers, w.heads, w.head_dim, w.page_size
    dev = G.DEV
    rng = np.random.default_rng([w.seed, 8])
    miss = [int(u) for u in w.miss_users]
    evict = [int(u) for u in w.evict_users]
    hit = [u for u in range(w.batch) if u not in set(miss)]
    extra = [u for u in (int(np.argmax(w.total_lens)), int(np.argmin(w.total_lens))) if u not in miss + evict]
    sampled = sorted(set(miss + evict + extra))
    assert len(miss) == 4 and len(evict) == 4 and w.batch == 256 and L == 4

    cache = PagedKVCache(L, w.num_pages, S, H, D, w.dtype, dev)
    torch.manual_seed(w.seed)
    cache.pool.view(torch.bfloat16).normal_()
    # the batch in the order the step runs it: cached users' rows first, then the restored users'
    order = hit + miss
    row_of = {}                                     # user -> first row in q / k_new / v_new / out
    pos = 0
    for u in order:
        row_of[u] = pos
        pos += int(w.new_lens[u])
    N = pos
    hit_b, n_hit = DeviceBatch.from_workload_users(w, hit, dev)
    miss_b, n_miss = DeviceBatch.from_workload_users(w, miss, dev)
    full_b, _ = DeviceBatch.from_workload_users(w, order, dev)
    pos_in_order = {u: i for i, u in enumerate(order)}

    # seeded host data of the sampled users, all layers
    hist = {u: [W.normal_elements(rng, (2, int(w.prefix_lens[u]), H, D), w.dtype) for _ in range(L)] for u in sampled}
    qh = [W.normal_elements(rng, (N, H, D), w.dtype) for _ in range(L)]
    kh = [W.normal_elements(rng, (N, H, D), w.dtype) for _ in range(L)]
    vh = [W.normal_elements(rng, (N, H, D), w.dtype) for _ in range(L)]
    q = [G.to_dev(a) for a in qh]
    kn = [G.to_dev(a) for a in kh]
    vn = [G.to_dev(a) for a in vh]
    out = [torch.zeros_like(x) for x in q]

    # cached sampled users: their histories are in the pool before the step (one scatter per layer)
    cached = [u for u in sampled if u not in miss]
    csegs = SegmentList.for_histories([pos_in_order[u] for u in cached], [w.prefix_lens[u] for u in cached],
                                      w.chunk_tokens, dev)

    def runs_of(users, layer):
        parts = []
        for u in users:
            for start, cnt in W.host_chunks(int(w.prefix_lens[u]), w.chunk_tokens):
                parts.append(np.ascontiguousarray(hist[u][layer][:, start:start + cnt]).reshape(-1))
        return np.concatenate(parts)
    for l in range(L):
        mts.mts_kv_unpack(cache.desc, l, G.to_dev(runs_of(cached, l)), *csegs.args(), full_b.meta)
    torch.cuda.synchronize()

    # restored users: pinned host memory, one block per layer
    msegs = SegmentList.for_histories(list(range(len(miss))), [w.prefix_lens[u] for u in miss], w.chunk_tokens, dev)
    layer_elems = msegs.total_tokens * 2 * H * D
    pinned = torch.empty(L, layer_elems, dtype=torch.int16, pin_memory=True)
    for l in range(L):
        pinned[l].numpy()[:] = runs_of(miss, l).view(np.int16)
    staging = torch.empty(L, layer_elems, dtype=torch.int16, device=dev)
    ws_bytes = max(mts.mts_attn_workspace_bytes(cache.desc, hit_b.meta), mts.mts_attn_workspace_bytes(cache.desc, miss_b.meta))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    compute, side = torch.cuda.Stream(), torch.cuda.Stream()
    ev = [torch.cuda.Event() for _ in range(L)]
    cs, ss = compute.cuda_stream, side.cuda_stream
    torch.cuda.synchronize()

    def layer_work(l, b, lo, hi):
        mts.mts_kv_append(cache.desc, l, kn[l][lo:hi], vn[l][lo:hi], b.meta, stream=cs)
        mts.mts_attn_incremental(cache.desc, l, q[l][lo:hi], out[l][lo:hi], b.meta, 0.0, ws, ws_bytes, stream=cs)

    for l in range(L):
        mts.mts_stage_h2d_async(staging[l], pinned[l], layer_elems * 2, stream=ss)
        mts.mts_kv_unpack(cache.desc, l, staging[l], *msegs.args(), miss_b.meta, stream=ss)
        ev[l].record(side)
    for l in range(L):
        layer_work(l, hit_b, 0, n_hit)
        compute.wait_event(ev[l])                                   # Alg. 1 step 8.3
        layer_work(l, miss_b, n_hit, n_hit + n_miss)
    # offload (step 9): gather the chosen users' whole sequences, all layers in one launch, copy back
    esegs = SegmentList.for_histories([pos_in_order[u] for u in evict], [w.total_lens[u] for u in evict],
                                      w.chunk_tokens, dev)
    e_elems = esegs.total_tokens * 2 * H * D
    off_dev = torch.empty(L, e_elems, dtype=torch.int16, device=dev)
    off_host = torch.empty(L, e_elems, dtype=torch.int16, pin_memory=True)
    mts.mts_kv_pack_layers(cache.desc, 0, L, off_dev, e_elems * 2, *esegs.args(), full_b.meta, stream=cs)
    mts.mts_stage_d2h_async(off_host, off_dev, L * e_elems * 2, stream=cs)
    torch.cuda.synchronize()

    # ---- the oracle on the sampled users ----------------------------------------------------
    sub = W.custom_workload("sampled", w.seed, w.dtype, L, H, D, S, [w.prefix_lens[u] for u in sampled],
                            [w.new_lens[u] for u in sampled], chunk_tokens=w.chunk_tokens)
    store = oracle.PagedStore(L, sub.num_pages, S, H, D, sub.np_dtype)
    rows = np.concatenate([np.arange(row_of[u], row_of[u] + int(w.new_lens[u])) for u in sampled])
    worst = 0.0
    for l in range(L):
        for i, u in enumerate(sampled):
            for start, cnt in W.host_chunks(int(w.prefix_lens[u]), w.chunk_tokens):
                oracle.unpack(store, l, hist[u][l][:, start:start + cnt], sub.user_pages(i), start)
        oracle.append(store, l, kh[l][rows], vh[l][rows], sub.page_indptr, sub.page_indices, sub.prefix_lens,
                      sub.new_indptr)
        ref = oracle.attn_incremental(store, l, qh[l][rows], sub.page_indptr, sub.page_indices, sub.prefix_lens,
                                      sub.new_indptr)
        gv = as_values(G.to_host(out[l], w.np_dtype))[rows]
        assert np.isfinite(gv).all()
        for i, u in enumerate(sampled):
            lo, hi = int(sub.new_indptr[i]), int(sub.new_indptr[i + 1])
            for h in range(H):
                r = ref[lo:hi, h]
                err = np.abs(gv[lo:hi, h] - r).max()
                tol = 2e-2 * np.abs(r).max()              # bf16 inputs, fp32 accumulation
                assert err <= tol, f"layer {l} user {u} (restored={u in miss}) head {h}: {err:.3e} > {tol:.3e}"
                worst = max(worst, err / tol)
        # the offload round trip: pages -> contiguous runs -> pinned host memory, bit for bit
        got = off_host[l].numpy().view(np.uint16)
        p = 0
        for u in evict:
            i = sampled.index(u)
            for start, cnt in W.host_chunks(int(w.total_lens[u]), w.chunk_tokens):
                want = oracle.pack(store, l, sub.user_pages(i), start, cnt)
                assert got[p:p + want.size].tobytes() == want.tobytes(), (l, u, start)
                p += want.size
        assert p == e_elems
    print(f"host_staging through pinned memory: worst error / tolerance {worst:.3f} over {len(sampled)} users x {H} heads x {L} layers")
