"""Host-staging path (the host_staging workload, reduced size): cache-miss users' contiguous host KV
is copied with hipMemcpyAsync from pinned memory on a side stream and unpacked into pages,
layer by layer, while the compute stream appends and attends; each layer's attention waits
only for that layer's event (Alg. 1 step 8.3).  Evicted users are packed and copied back:
the round trip must be bit-exact."""
import time

import numpy as np
import pytest

import mts_workloads as W
import oracle
from helpers import draw_step_data, oracle_store_for, as_values

pytestmark = pytest.mark.gpu


def test_staged_restore_overlapped_with_attention_and_offload_roundtrip():
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd.runtime import SegmentList

    rng = np.random.default_rng(44)
    B = 24
    prefix = np.clip(np.rint(np.exp(rng.normal(np.log(2000), 0.6, size=B))), 128, 8192).astype(int)
    new = rng.integers(8, 65, size=B)
    order = rng.permutation(B)
    miss, evict = np.sort(order[:3]), np.sort(order[3:6])
    w = W.custom_workload("staging", 4004, "bf16", 2, 8, 64, 16, prefix, new, miss_users=miss,
                          evict_users=evict, chunk_tokens=1024)
    L, H, D = w.layers, w.heads, w.head_dim
    data = draw_step_data(w)
    step = G.GpuStep(w, fill_byte=0xFF)
    hits = [u for u in range(B) if u not in set(miss.tolist())]
    for l in range(L):                                  # hit users are already resident
        step.unpack_histories(data, l, users=hits)

    # pinned host copy of the miss users' histories, one buffer per layer, chunked runs
    segs = SegmentList.for_histories(miss, [w.prefix_lens[u] for u in miss], w.chunk_tokens, G.DEV)
    su, sp = segs.seg_user.cpu().numpy(), segs.seg_pos.cpu().numpy()
    cnt = np.diff(segs.host_indptr)
    n_elem = segs.total_tokens * 2 * H * D
    pinned = [torch.empty(n_elem, dtype=torch.int16, pin_memory=True) for _ in range(L)]
    for l in range(L):
        host = np.concatenate([np.ascontiguousarray(data["hist"][l][su[s]][:, sp[s]:sp[s] + cnt[s]]).reshape(-1)
                               for s in range(segs.num_segs)])
        pinned[l].numpy()[:] = host.view(np.int16)
    staging = [torch.empty(n_elem, dtype=torch.int16, device=G.DEV) for _ in range(L)]

    compute, side = torch.cuda.Stream(), torch.cuda.Stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(L + 1)]
    q = [G.to_dev(data["q"][l]) for l in range(L)]
    kn = [G.to_dev(data["k_new"][l]) for l in range(L)]
    vn = [G.to_dev(data["v_new"][l]) for l in range(L)]
    out = [torch.zeros_like(q[l]) for l in range(L)]
    torch.cuda.synchronize()

    t0 = time.perf_counter()
    ev[L].record(side)
    for l in range(L):
        mts.mts_stage_h2d_async(staging[l], pinned[l], n_elem * 2, stream=side)
        mts.mts_kv_unpack(step.cache.desc, l, staging[l], *segs.args(), step.batch.meta, stream=side)
        ev[l].record(side)
    for l in range(L):
        mts.mts_kv_append(step.cache.desc, l, kn[l], vn[l], step.batch.meta, stream=compute)
        compute.wait_event(ev[l])
        mts.mts_attn_incremental(step.cache.desc, l, q[l], out[l], step.batch.meta, 0.0, step.ws,
                                 step.ws_bytes, stream=compute)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    h2d_ms = ev[L].elapsed_time(ev[L - 1])
    print(f"staged {L * n_elem * 2 / 1e6:.1f} MB in {segs.num_segs} runs/layer: H2D+unpack {h2d_ms:.3f} ms "
          f"({L * n_elem * 2 / h2d_ms / 1e6:.1f} GB/s incl. unpack), step wall {wall * 1e3:.2f} ms")

    store = oracle_store_for(w, data)
    for l in range(L):
        ref = oracle.attn_incremental(store, l, data["q"][l], w.page_indptr, w.page_indices,
                                      w.prefix_lens, w.new_indptr)
        gv = as_values(G.to_host(out[l], w.np_dtype))
        for u in range(B):
            lo, hi = w.new_indptr[u], w.new_indptr[u + 1]
            for h in range(H):
                r = ref[lo:hi, h]
                assert np.abs(gv[lo:hi, h] - r).max() <= 2e-2 * np.abs(r).max(), (l, u, h)

    # offload: pack the evicted users (history + this step's rows), D2H into pinned memory
    lens = [int(w.total_lens[u]) for u in evict]
    esegs = SegmentList.for_histories(evict, lens, w.chunk_tokens, G.DEV)
    e_elem = esegs.total_tokens * 2 * H * D
    off_dev = torch.empty(e_elem, dtype=torch.int16, device=G.DEV)
    off_host = torch.empty(e_elem, dtype=torch.int16, pin_memory=True)
    eu, ep = esegs.seg_user.cpu().numpy(), esegs.seg_pos.cpu().numpy()
    ecnt = np.diff(esegs.host_indptr)
    for l in range(L):
        mts.mts_kv_pack(step.cache.desc, l, off_dev, *esegs.args(), step.batch.meta, stream=side)
        mts.mts_stage_d2h_async(off_host, off_dev, e_elem * 2, stream=side)
        side.synchronize()
        got = off_host.numpy().view(np.uint16)
        pos = 0
        for s in range(esegs.num_segs):
            want = oracle.pack(store, l, w.user_pages(eu[s]), int(ep[s]), int(ecnt[s]))
            assert got[pos:pos + want.size].tobytes() == want.tobytes(), (l, s)
            pos += want.size
