"""GPU parity of mts_attn_incremental_staged: some users' cached prefix is NOT in the pool (their
pages still hold NaN patterns) but in a contiguous onload buffer, in host-chunk runs of the
[2][n][H][D] layout; the step's rows come from k_new / v_new.  The output must equal the oracle's
attention over the complete store, and the pool must come back untouched."""
import numpy as np
import pytest

import mts_workloads as W
import oracle
from helpers import draw_step_data
from test_gpu_parity import CASES, SCHEDULES, FILL, _case, _random_case, check_attention

pytestmark = pytest.mark.gpu


def _store(w, data, users, do_append):
    store = oracle.PagedStore(w.layers, w.num_pages, w.page_size, w.heads, w.head_dim, w.np_dtype)
    store.data.view(np.uint8)[...] = FILL
    for l in data["layers"]:
        for u in users:
            for start, cnt in W.host_chunks(int(w.prefix_lens[u]), w.chunk_tokens):
                oracle.unpack(store, l, data["hist"][l][u][:, start:start + cnt], w.user_pages(u), start)
        if do_append:
            oracle.append(store, l, data["k_new"][l], data["v_new"][l], w.page_indptr, w.page_indices,
                          w.prefix_lens, w.new_indptr)
    return store


def _run(w, staged_users, chunk, data=None):
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    data = draw_step_data(w) if data is None else data
    step = G.GpuStep(w, fill_byte=FILL)
    staged_users = [u for u in staged_users if w.prefix_lens[u] > 0]
    hit_users = [u for u in range(w.batch) if u not in staged_users]
    full = _store(w, data, range(w.batch), True)
    bare = _store(w, data, hit_users, False)
    for l in range(w.layers):
        step.unpack_histories(data, l, users=hit_users)
        # the onload buffer of this layer: every staged user's prefix in runs of `chunk` tokens
        rows, run_tok, first_run = [], [0], np.full(w.batch, -1, np.int32)
        for u in staged_users:
            first_run[u] = len(run_tok) - 1
            P = int(w.prefix_lens[u])
            for start in range(0, P, chunk):
                n = min(chunk, P - start)
                rows.append(np.ascontiguousarray(data["hist"][l][u][:, start:start + n]).reshape(-1))
                run_tok.append(run_tok[-1] + n)
        rows_dev = G.to_dev(np.concatenate(rows) if rows else np.zeros(8, w.np_dtype))
        first_dev = torch.from_numpy(first_run).to(G.DEV)
        tok_dev = torch.from_numpy(np.asarray(run_tok, np.int64)).to(G.DEV)
        q, k, v = (G.to_dev(data[n][l]) for n in ("q", "k_new", "v_new"))
        out = torch.full((max(w.total_new, 1), w.heads, w.head_dim), -1, dtype=q.dtype, device=G.DEV)
        mts.mts_attn_incremental_staged(step.cache.desc, l, q, k, v, rows_dev, first_dev, tok_dev, chunk, out,
                                        step.batch.meta, 0.0, step.ws, step.ws_bytes)
        torch.cuda.synchronize()
        got = G.to_host(out[:w.total_new], w.np_dtype)
        ref = oracle.attn_incremental(full, l, data["q"][l], w.page_indptr, w.page_indices, w.prefix_lens,
                                      w.new_indptr)
        check_attention(w, got, ref)
        assert np.array_equal(step.pool_image(l), G.expected_pool_image(w, bare, l, FILL)), "the pool was touched"
    return data, full


BF16_CASES = [n for n in CASES if CASES[n][0] == "bf16"]


@pytest.mark.parametrize("name", BF16_CASES)
@pytest.mark.parametrize("schedule", list(SCHEDULES))
def test_staged_small(name, schedule, attn_tuning):
    """Every second user staged, under every work schedule, runs of 32 tokens (many runs per user)."""
    attn_tuning(**SCHEDULES[schedule])
    w = _case(name)
    _run(w, list(range(0, w.batch, 2)), 32)


@pytest.mark.parametrize("name", BF16_CASES)
def test_staged_all_users_long_runs(name):
    w = _case(name)
    _run(w, list(range(w.batch)), 1024)


@pytest.mark.parametrize("seed", range(16))
def test_staged_random_shapes(seed):
    w = _random_case(seed)
    rng = np.random.default_rng(seed)
    staged = [u for u in range(w.batch) if rng.random() < 0.5]
    chunk = int(rng.choice([32, 64, 256, 1024]))
    if int(w.new_lens.max()) >= 256 and int(w.total_new) >= 128 * w.batch and w.head_dim in (64, 128):
        # long new segments are served by the dense-prefill kernel, which reads the pool only: the
        # staged call must refuse the shape (histories are unpacked first there), before any launch
        _refused_as_unsupported(w, chunk)
        return
    _run(w, staged, chunk)


def _refused_as_unsupported(w, chunk):
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd import binding as B
    step = G.GpuStep(w, fill_byte=FILL)
    before = step.pool_image(0)
    x = torch.zeros(max(w.total_new, 1) * w.heads * w.head_dim + 8, dtype=torch.int16, device=G.DEV)
    out = torch.full_like(x, 7)
    first = torch.full((w.batch,), -1, dtype=torch.int32, device=G.DEV)
    tok = torch.zeros(2, dtype=torch.int64, device=G.DEV)
    with pytest.raises(mts.MtsError) as e:
        mts.mts_attn_incremental_staged(step.cache.desc, 0, x, x, x, x, first, tok, chunk, out, step.batch.meta, 0.0,
                                        step.ws, step.ws_bytes)
    assert e.value.code == B.MTS_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((out == 7).all()), "the refused call wrote output rows"
    assert np.array_equal(step.pool_image(0), before), "the refused call touched the pool"


def test_staged_prefill_shape_is_refused():
    """A cache-miss shape (every user hundreds of new tokens) handed to the staged call: MTS_ERR_UNSUPPORTED."""
    w = W.custom_workload("staged_prefill_shape", 92, "bf16", 1, 2, 128, 16, [64, 0, 700], [300, 512, 260])
    _refused_as_unsupported(w, 64)


def test_staged_prefix_lengths_around_run_and_tile_boundaries():
    prefix = [31, 32, 33, 63, 64, 65, 127, 128, 129, 1]
    w = W.custom_workload("staged_edges", 91, "bf16", 1, 2, 64, 16, prefix, [3, 17, 32, 33, 64, 1, 8, 40, 5, 2])
    _run(w, list(range(w.batch)), 64)
    _run(w, [0, 3, 4, 9], 32)


def test_staged_nobody_staged_equals_the_unappended_call():
    _run(_case("bf16_ragged"), [], 64)


def test_staged_dominant_key_in_the_onload_buffer():
    """A key far into a staged history dominates: the redo with the exact max reads the onload
    buffer's K rows as well."""
    w = W.custom_workload("staged_dominant", 79, "bf16", 1, 2, 64, 16, [700, 90, 300], [20, 3, 40])
    data = draw_step_data(w)
    for u, tok in ((0, 555), (2, 37)):
        h = np.array(data["hist"][0][u])
        h[0] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(h[0]) * 0.01)
        h[0, tok] = W.f32_to_bf16_bits(np.full((w.heads, w.head_dim), 60.0, np.float32))
        data["hist"][0][u] = h
    data["q"][0] = W.f32_to_bf16_bits(np.abs(W.bf16_bits_to_f32(data["q"][0])) + 0.5)
    _run(w, [0, 2], 128, data=data)


def test_staged_is_refused_for_other_kernels():
    import torch
    import gpu_harness as G
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd import binding as B
    w = _case("f32_ragged")
    step = G.GpuStep(w, fill_byte=FILL)
    x = torch.zeros(max(w.total_new, 1) * w.heads * w.head_dim + 8, dtype=torch.float32, device=G.DEV)
    first = torch.full((w.batch,), -1, dtype=torch.int32, device=G.DEV)
    tok = torch.zeros(2, dtype=torch.int64, device=G.DEV)
    with pytest.raises(mts.MtsError) as e:
        mts.mts_attn_incremental_staged(step.cache.desc, 0, x, x, x, x, first, tok, 64, x, step.batch.meta, 0.0,
                                        step.ws, step.ws_bytes)
    assert e.value.code == B.MTS_ERR_UNSUPPORTED
    for chunk in (0, 48, -32):
        with pytest.raises(mts.MtsError) as e:
            mts.mts_attn_incremental_staged(step.cache.desc, 0, x, x, x, x, first, tok, chunk, x, step.batch.meta,
                                            0.0, step.ws, step.ws_bytes)
        assert e.value.code == B.MTS_ERR_INVALID_ARG
