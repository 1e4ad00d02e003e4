"""Alg. 1 end to end on the GPU, over many steps of returning users: the cache manager decides
pages, evictions and what must come up from the host tier; the transfer pipeline brings it up
and persists whole host chunks; append and attention run per layer behind the per-layer wait.
Every step's attention output is compared with the oracle evaluated on each user's complete
token history (kept by the test), so a wrong page table, a lost or stale chunk, a missing wait
or a mis-tracked length shows up as a wrong output."""
import numpy as np
import pytest

import mts_workloads as W
import oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("order", ["append_first", "deferred_append"])
def test_returning_users_over_many_steps_with_eviction_onload_and_offload(order):
    """order: Alg. 1's (append, then attention from the pool), or the attention that reads the
    step's rows directly with one append of all layers behind the layer loop."""
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd.runtime import DeviceBatch, HostRuns, PagedKVCache, SegmentList
    L, H, D, S, chunk, num_pages, n_users = 2, 2, 64, 16, 32, 36, 7
    row = 2 * H * D * 2
    rng = np.random.default_rng(17)
    cm = mts.CacheManager(num_pages, S, chunk)
    cache = PagedKVCache(L, num_pages, S, H, D, "bf16", G.DEV, fill_byte=0xFF)
    xfer = mts.mts_xfer_create(pinned_bytes=chunk * row, num_layers=L, offload_arena_bytes=1 << 22,
                               offload_quota_tokens=1 << 20, copy_threads=2)
    compute = torch.cuda.Stream(device=G.DEV)
    full = {u: [np.zeros((3, 0, H, D), np.uint16) for _ in range(L)] for u in range(n_users)}   # K, V, Q of every token
    host_store = {u: [np.zeros((2, 0, H, D), np.uint16) for _ in range(L)] for u in range(n_users)}
    seen = dict(host_hit=0, gpu_hit=0, evicted=0, offloaded=0, refused=0)
    try:
        for step in range(40):
            users = rng.choice(n_users, size=int(rng.integers(1, 4)), replace=False)
            fresh = rng.integers(1, 25, size=len(users))
            for u, n in zip(users.tolist(), fresh.tolist()):
                for l in range(L):
                    full[u][l] = np.concatenate([full[u][l], W.normal_elements(rng, (3, n, H, D), "bf16")], axis=1)
            cached = np.array([cm.cached_length(u) for u in users])
            total = np.array([full[u][0].shape[1] for u in users.tolist()])
            new = (total - cached).astype(np.int32)             # really new tokens + those an eviction dropped
            try:
                prefix, onload, indptr, indices = cm.prepare_batch(users, new)
            except mts.MtsError as e:
                assert e.code == mts.MTS_ERR_BUSY
                seen["refused"] += 1
                for u, n in zip(users.tolist(), fresh.tolist()):     # the request is dropped: forget its tokens
                    for l in range(L):
                        full[u][l] = full[u][l][:, :-n]
                continue
            assert prefix.tolist() == cached.tolist()
            seen["evicted"] += len(cm.take_evicted())
            new_indptr = np.concatenate([[0], np.cumsum(new)]).astype(np.int32)
            batch = DeviceBatch(indptr, indices, prefix, new_indptr, G.DEV)
            ws_bytes = mts.mts_attn_workspace_bytes(cache.desc, batch.meta)
            ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=G.DEV)
            # what the host tier must bring up (Alg. 1 step 2)
            up = [i for i in range(len(users)) if onload[i] > 0]
            seen["host_hit"] += len(up)
            seen["gpu_hit"] += sum(1 for i in range(len(users)) if onload[i] == 0 and prefix[i] > 0)
            if up:
                segs = SegmentList.for_histories(up, [int(onload[i]) for i in up], chunk, G.DEV)
                su, sp = segs.seg_user.cpu().numpy(), segs.seg_pos.cpu().numpy()
                cnt = np.diff(segs.host_indptr)
                for i in up:
                    assert host_store[int(users[i])][0].shape[1] >= onload[i], "manager believes more is persisted than is"
                arrays = [[np.ascontiguousarray(host_store[int(users[su[s]])][l][:, sp[s]:sp[s] + cnt[s]])
                           for s in range(segs.num_segs)] for l in range(L)]
                on_host = HostRuns(segs, arrays)
                stride = segs.total_tokens * row
                staging = torch.empty(L * stride, dtype=torch.uint8, device=G.DEV)
                mts.mts_xfer_onload_submit(xfer, cache.desc, batch.meta, on_host.runs, staging, stride)
            outs = []
            for l in range(L):
                rows = [full[int(u)][l][:, cached[i]:total[i]] for i, u in enumerate(users)]
                k = G.to_dev(np.concatenate([r[0] for r in rows])); v = G.to_dev(np.concatenate([r[1] for r in rows]))
                q = G.to_dev(np.concatenate([r[2] for r in rows]))
                out = torch.zeros_like(q)
                if order == "append_first":
                    mts.mts_kv_append(cache.desc, l, k, v, batch.meta, stream=compute)
                if up:
                    mts.mts_xfer_onload_wait_layer(xfer, l, compute)
                if order == "append_first":
                    mts.mts_attn_incremental(cache.desc, l, q, out, batch.meta, 0.0, ws, ws_bytes, stream=compute)
                else:
                    mts.mts_attn_incremental_unappended(cache.desc, l, q, k, v, out, batch.meta, 0.0, ws, ws_bytes,
                                                        stream=compute)
                outs.append((k, v, q, out))
            if order == "deferred_append":
                k_all = torch.stack([o[0] for o in outs]); v_all = torch.stack([o[1] for o in outs])
                compute.wait_stream(torch.cuda.current_stream())      # the stacks above ran on the current stream
                mts.mts_kv_append_layers(cache.desc, 0, L, k_all, v_all, k_all.stride(0) * k_all.element_size(),
                                         batch.meta, stream=compute)
            cm.commit_batch()
            # persist whole host chunks of the users that are due (Alg. 1 step 9)
            du, dp, dc = cm.offload_due()
            if len(du):
                local = {int(u): i for i, u in enumerate(users)}
                assert all(int(u) in local for u in du), "only users of the batch just run can have become due"
                su_, sp_, sc_ = [], [], []
                for u, p, c in zip(du.tolist(), dp.tolist(), dc.tolist()):
                    for a in range(p, p + c, chunk):
                        su_.append(local[u]); sp_.append(a); sc_.append(chunk)
                osegs = SegmentList(su_, sp_, sc_, G.DEV)
                oarr = [[np.zeros((2, chunk, H, D), np.uint16) for _ in su_] for _ in range(L)]
                off_host = HostRuns(osegs, oarr)
                mts.mts_xfer_offload_submit(xfer, cache.desc, batch.meta, off_host.runs, compute)
            mts.mts_xfer_drain(xfer)
            torch.cuda.synchronize()
            if len(du):
                k_ = 0
                for u, p, c in zip(du.tolist(), dp.tolist(), dc.tolist()):
                    for a in range(p, p + c, chunk):
                        for l in range(L):
                            assert host_store[u][l].shape[1] == a or l > 0
                            host_store[u][l] = np.concatenate([host_store[u][l][:, :a], oarr[l][k_]], axis=1)
                        k_ += 1
                    cm.offload_done(u, p + c)
                    seen["offloaded"] += c
                    for l in range(L):       # what came back is what the user's history says, byte for byte
                        assert host_store[u][l].tobytes() == np.ascontiguousarray(full[u][l][:2, :p + c]).tobytes()
            # ground truth: the oracle on each user's complete history, in a store of its own
            for l in range(L):
                got = W.bf16_bits_to_f32(G.to_host(outs[l][3], np.uint16)).astype(np.float64)
                for i, u in enumerate(users.tolist()):
                    T, P = int(total[i]), int(cached[i])
                    store = oracle.PagedStore(1, oracle.pages_for(T, S), S, H, D, np.uint16)
                    pages = np.arange(oracle.pages_for(T, S))
                    oracle.unpack(store, 0, full[u][l][:2, :T], pages, 0)
                    ref = oracle.attn_incremental(store, 0, full[u][l][2, P:T], np.array([0, len(pages)]), pages,
                                                  np.array([P]), np.array([0, T - P]))
                    g = got[new_indptr[i]:new_indptr[i + 1]]
                    for h in range(H):
                        err = np.abs(g[:, h] - ref[:, h]).max()
                        assert err <= 2e-2 * np.abs(ref[:, h]).max(), f"step {step} user {u} layer {l} head {h}: {err}"
        print("serving loop:", seen, cm.stats())
        assert seen["host_hit"] > 0 and seen["gpu_hit"] > 0 and seen["evicted"] > 0 and seen["offloaded"] > 0
    finally:
        mts.mts_xfer_destroy(xfer)
        cm.close()
