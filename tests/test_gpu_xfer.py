"""The transfer pipeline on the GPU (Sec. 4.2 double-buffered onload, transient offload with
admission control; Sec. 4.4 layer-wise synchronisation): histories travel from ordinary host
memory through the two pinned buffers into the onload buffer and are scattered layer by layer
while the compute stream, told to wait per layer, appends and attends; offload brings the
pages back into host memory.  Data movement is compared bit for bit with the oracle."""
import numpy as np
import pytest

import mts_workloads as W
import oracle
from helpers import draw_step_data
from test_gpu_parity import FILL, _oracle_store, check_attention

pytestmark = pytest.mark.gpu


def _history_runs(w, data, users, chunk):
    """Per-layer host arrays of every history run (pageable numpy memory)."""
    import gpu_harness as G
    from paper_2604_22881_amd.runtime import SegmentList
    segs = SegmentList.for_histories(users, [int(w.prefix_lens[u]) for u in users], chunk, G.DEV)
    su, sp = segs.seg_user.cpu().numpy(), segs.seg_pos.cpu().numpy()
    cnt = np.diff(segs.host_indptr)
    arrays = [[np.ascontiguousarray(data["hist"][l][su[s]][:, sp[s]:sp[s] + cnt[s]]) for s in range(segs.num_segs)]
              for l in range(w.layers)]
    return segs, arrays


@pytest.mark.parametrize("runs_per_dma", [1, 3])
def test_onload_then_per_layer_wait_then_attention_twice(runs_per_dma):
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd.runtime import HostRuns
    chunk = 256
    w = W.custom_workload("xfer", 41, "bf16", 3, 2, 64, 16, [700, 33, 2100, 0, 256], [5, 9, 3, 12, 1],
                          chunk_tokens=chunk)
    row = 2 * w.heads * w.head_dim * 2
    xfer = mts.mts_xfer_create(pinned_bytes=runs_per_dma * chunk * row, num_layers=w.layers, copy_threads=3)
    try:
        step = G.GpuStep(w, fill_byte=FILL)
        compute = torch.cuda.Stream(device=G.DEV)
        for rep in range(2):                                     # the second task reuses buffers, streams and events
            data = draw_step_data(w, seed_offset=rep)
            users = [u for u in range(w.batch) if w.prefix_lens[u] > 0]
            segs, arrays = _history_runs(w, data, users, chunk)
            host = HostRuns(segs, arrays)
            stride = segs.total_tokens * row
            staging = torch.empty(w.layers * stride, dtype=torch.uint8, device=G.DEV)
            mts.mts_xfer_onload_submit(xfer, step.cache.desc, step.batch.meta, host.runs, staging, stride)
            outs = []
            for l in range(w.layers):
                k, v, q = (G.to_dev(data[n][l]) for n in ("k_new", "v_new", "q"))
                out = torch.zeros_like(q)
                mts.mts_kv_append(step.cache.desc, l, k, v, step.batch.meta, stream=compute)
                mts.mts_xfer_onload_wait_layer(xfer, l, compute)                  # Alg. 1 step 8.3
                mts.mts_attn_incremental(step.cache.desc, l, q, out, step.batch.meta, 0.0, step.ws, step.ws_bytes,
                                         stream=compute)
                outs.append((k, v, q, out))
            mts.mts_xfer_drain(xfer)
            torch.cuda.synchronize()
            store = _oracle_store(w, data)
            for l in range(w.layers):
                assert np.array_equal(step.pool_image(l), G.expected_pool_image(w, store, l, FILL)), f"layer {l}"
                ref = oracle.attn_incremental(store, l, data["q"][l], w.page_indptr, w.page_indices,
                                              w.prefix_lens, w.new_indptr)
                check_attention(w, G.to_host(outs[l][3], w.np_dtype), ref)
    finally:
        mts.mts_xfer_destroy(xfer)


def test_offload_writes_host_chunks_and_admission_control_refuses_what_does_not_fit():
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd.runtime import HostRuns, SegmentList
    chunk = 128
    w = W.custom_workload("xfer_off", 43, "bf16", 2, 3, 64, 16, [300, 40, 0], [21, 7, 130], chunk_tokens=chunk)
    row = 2 * w.heads * w.head_dim * 2
    data = draw_step_data(w)
    step = G.GpuStep(w, fill_byte=FILL)
    for l in range(w.layers):
        step.unpack_histories(data, l)
    compute = torch.cuda.Stream(device=G.DEV)
    for l in range(w.layers):
        mts.mts_kv_append(step.cache.desc, l, G.to_dev(data["k_new"][l]), G.to_dev(data["v_new"][l]), step.batch.meta,
                          stream=compute)
    store = _oracle_store(w, data)
    users = [0, 2]
    totals = [int(w.total_lens[u]) for u in users]
    segs = SegmentList.for_histories(users, totals, chunk, G.DEV)          # whole sequences, chunk-sized runs
    cnt = np.diff(segs.host_indptr)
    arrays = [[np.full((2, int(n), w.heads, w.head_dim), 0xABCD, np.uint16) for n in cnt] for _ in range(w.layers)]
    host = HostRuns(segs, arrays)
    tokens = int(cnt.sum())
    arena = w.layers * tokens * row + 4096

    # (a) a task larger than the quota, and one larger than the arena, are refused and touch nothing
    small = mts.mts_xfer_create(pinned_bytes=chunk * row, num_layers=w.layers, offload_arena_bytes=arena,
                                offload_quota_tokens=tokens - 1)
    try:
        with pytest.raises(mts.MtsError) as e:
            mts.mts_xfer_offload_submit(small, step.cache.desc, step.batch.meta, host.runs, compute)
        assert e.value.code == mts.MTS_ERR_BUSY
        assert mts.mts_xfer_offload_pending_tokens(small) == 0
    finally:
        mts.mts_xfer_destroy(small)
    tight = mts.mts_xfer_create(pinned_bytes=chunk * row, num_layers=w.layers, offload_arena_bytes=arena // 2,
                                offload_quota_tokens=10 * tokens)
    try:
        with pytest.raises(mts.MtsError) as e:
            mts.mts_xfer_offload_submit(tight, step.cache.desc, step.batch.meta, host.runs, compute)
        assert e.value.code == mts.MTS_ERR_BUSY
    finally:
        mts.mts_xfer_destroy(tight)
    assert all((a == 0xABCD).all() for la in arrays for a in la)

    # (b) accepted: gather -> pinned ping-pong -> host arrays, twice in a row through one pipeline
    # pinned buffers of 2.5 runs: consecutive runs share a DMA, two at a time
    xfer = mts.mts_xfer_create(pinned_bytes=chunk * row * 5 // 2, num_layers=w.layers, offload_arena_bytes=2 * arena,
                               offload_quota_tokens=2 * tokens, copy_threads=2)
    try:
        arrays2 = [[np.zeros_like(a) for a in la] for la in arrays]
        host2 = HostRuns(segs, arrays2)
        mts.mts_xfer_offload_submit(xfer, step.cache.desc, step.batch.meta, host.runs, compute)
        mts.mts_xfer_offload_submit(xfer, step.cache.desc, step.batch.meta, host2.runs, compute)
        assert 0 <= mts.mts_xfer_offload_pending_tokens(xfer) <= 2 * tokens
        mts.mts_xfer_drain(xfer)
        assert mts.mts_xfer_offload_pending_tokens(xfer) == 0
        su, sp = segs.seg_user.cpu().numpy(), segs.seg_pos.cpu().numpy()
        for l in range(w.layers):
            for s in range(segs.num_segs):
                want = oracle.pack(store, l, w.user_pages(int(su[s])), int(sp[s]), int(cnt[s]))
                assert arrays[l][s].tobytes() == want.tobytes(), f"layer {l} run {s}"
                assert arrays2[l][s].tobytes() == want.tobytes(), f"second task, layer {l} run {s}"
    finally:
        mts.mts_xfer_destroy(xfer)
