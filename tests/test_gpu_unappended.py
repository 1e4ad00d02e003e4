"""GPU parity of mts_attn_incremental_unappended / mts_attn_pointwise_unappended: the step's K/V
rows are handed over as [token][H][D] arrays and the pool holds only the cached prefixes, its
slots for the new tokens still filled with NaN patterns.  The output must equal the oracle's
attention over the store WITH the rows appended (same tolerances as the appended calls), and -
where the streaming matrix-core kernel serves the call - the pool must come back untouched.
Shapes served by the other kernels (fp32, long new segments) are appended by the call itself."""
import numpy as np
import pytest

import mts_workloads as W
import oracle
from helpers import draw_step_data, as_values
from test_gpu_parity import (CASES, EDGE_CASES, PREFILL_CASES, SCHEDULES, FILL, _case, _oracle_store, _random_case,
                             check_attention)
from test_gpu_pointwise import _check as check_pointwise

from conftest import KERNEL_PLAIN, KERNEL_PREFILL, KERNEL_STREAMING  # noqa: F401

pytestmark = pytest.mark.gpu


def _served_by_streaming_kernel(w):
    # the library's own routing: long new segments go to the workgroup-per-query-block kernel,
    # which exists for head_dim 64 and 128
    long_new = int(w.new_lens.max()) >= 256 and int(w.total_new) >= 128 * w.batch and w.head_dim in (64, 128)
    return w.dtype == "bf16" and not long_new


def _run(w, data=None, inv_norm=None, sm_scale=0.0, concurrent_append=False):
    import torch
    import gpu_harness as G
    data = draw_step_data(w) if data is None else data
    step = G.GpuStep(w, fill_byte=FILL)
    bare = _oracle_store(w, data, do_append=False)
    full = _oracle_store(w, data, do_append=True)
    side = torch.cuda.Stream() if concurrent_append else None
    for l in range(w.layers):
        step.unpack_histories(data, l)
        got = step.attention_unappended(data, l, sm_scale=sm_scale, inv_norm=inv_norm,
                                        append_stream=side.cuda_stream if side else None)
        if inv_norm is None:
            ref = oracle.attn_incremental(full, l, data["q"][l], w.page_indptr, w.page_indices, w.prefix_lens,
                                          w.new_indptr, sm_scale=(sm_scale or None))
            check_attention(w, got, ref)
        else:
            ref = oracle.attn_pointwise(full, l, data["q"][l], w.page_indptr, w.page_indices, w.prefix_lens,
                                        w.new_indptr, inv_norm, sm_scale=(sm_scale or None))
            check_pointwise(w, got, ref)
        appended = concurrent_append or not _served_by_streaming_kernel(w)
        want = G.expected_pool_image(w, full if appended else bare, l, FILL)
        assert np.array_equal(step.pool_image(l), want), "pool image after the call"
    return step, data, full


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("schedule", list(SCHEDULES))
def test_unappended_small(name, schedule, attn_tuning):
    """Every small case under every work schedule: share boundaries fall inside, before and after
    the tiles that mix pool tokens with new rows."""
    attn_tuning(**SCHEDULES[schedule])
    _run(_case(name))


@pytest.mark.parametrize("name", list(CASES))
def test_unappended_pointwise_small(name, attn_tuning):
    attn_tuning(min_tiles=1)
    w = _case(name)
    _run(w, inv_norm=1.0 / max(1, int(w.total_lens.max())))


@pytest.mark.parametrize("seed", range(24))
def test_unappended_random_shapes(seed):
    _run(_random_case(seed))


@pytest.mark.parametrize("name", list(EDGE_CASES))
def test_unappended_edge_shapes(name):
    rng = np.random.default_rng(len(name))
    dtype, L, H, D, S, prefix, new = EDGE_CASES[name](rng)
    _run(W.custom_workload(name, 300 + len(name), dtype, L, H, D, S, np.asarray(prefix), np.asarray(new)))


@pytest.mark.parametrize("name", ["prefill_d64", "prefill_mixed_lengths"])
@pytest.mark.parametrize("prefill", [KERNEL_STREAMING, None])
def test_unappended_long_new_segments(name, prefill, attn_tuning):
    """Several query tiles per user through the streaming kernel (later query tiles see the new
    rows of earlier ones), and the same cases as the library routes them by itself (appended by
    the call, then the workgroup-per-query-block kernel)."""
    dtype, L, H, D, S, prefix, new, chunk = PREFILL_CASES[name]
    w = W.custom_workload(name, 200 + len(name), dtype, L, H, D, S, prefix, new, chunk_tokens=chunk)
    if prefill is not None:
        attn_tuning(kernel=prefill)
        import torch
        import gpu_harness as G
        data = draw_step_data(w)
        step = G.GpuStep(w, fill_byte=FILL)
        full = _oracle_store(w, data, do_append=True)
        step.unpack_histories(data, 0)
        got = step.attention_unappended(data, 0)
        check_attention(w, got, oracle.attn_incremental(full, 0, data["q"][0], w.page_indptr, w.page_indices,
                                                        w.prefix_lens, w.new_indptr))
        bare = _oracle_store(w, data, do_append=False)
        assert np.array_equal(step.pool_image(0), G.expected_pool_image(w, bare, 0, FILL))
    else:
        _run(w)


def test_unappended_explicit_scale():
    _run(_case("bf16_ragged"), sm_scale=0.3)


def test_unappended_with_the_append_on_another_stream():
    """The use the call is for: mts_kv_append of the same layer runs on a second stream while the
    attention reads the rows directly.  Same output, and the pool ends up appended."""
    w = W.custom_workload("side_append", 31, "bf16", 2, 4, 64, 16, [700, 90, 300, 0, 2049, 15],
                          [20, 3, 40, 64, 33, 17])
    _run(w, concurrent_append=True)


def test_unappended_late_dominant_key_among_the_new_rows():
    """The reference max of a segment comes from its first tile; here the key that dominates is
    one of the new rows, so the redo with the exact max has to read k_new as well."""
    w = W.custom_workload("dominant_new", 78, "bf16", 1, 2, 64, 16, [700, 90, 300], [20, 3, 40])
    data = draw_step_data(w)
    for u in range(w.batch):                           # small logits everywhere ...
        h = np.array(data["hist"][0][u])
        h[0] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(h[0]) * 0.01)
        data["hist"][0][u] = h
    k = W.bf16_bits_to_f32(data["k_new"][0]) * 0.01
    lo, lo2 = int(w.new_indptr[0]), int(w.new_indptr[2])
    k[lo + 2] = 60.0                                   # ... but one huge key among user 0's new rows
    k[lo2 + 35] = 60.0                                 # and one late in user 2's
    data["k_new"][0] = W.f32_to_bf16_bits(k)
    data["q"][0] = W.f32_to_bf16_bits(np.abs(W.bf16_bits_to_f32(data["q"][0])) + 0.5)
    _, _, full = _run(w, data=data)
    ref = oracle.attn_incremental(full, 0, data["q"][0], w.page_indptr, w.page_indices, w.prefix_lens, w.new_indptr)
    # sanity of the construction: queries at or after the dominant row return its value row
    assert np.allclose(ref[lo + 2:lo + 20, 0], as_values(data["v_new"][0][lo + 2, 0]), atol=1e-6)


def test_unappended_bad_arguments():
    import torch
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd import binding as B
    import gpu_harness as G
    w = _case("bf16_ragged")
    step = G.GpuStep(w, fill_byte=FILL)
    x = torch.zeros(max(w.total_new, 1) * w.heads * w.head_dim + 8, dtype=torch.int16, device=G.DEV)
    for k, v in ((None, x), (x, None), (x[1:], x)):
        with pytest.raises(mts.MtsError) as e:
            mts.mts_attn_incremental_unappended(step.cache.desc, 0, x, k, v, x, step.batch.meta, 0.0, step.ws,
                                                step.ws_bytes)
        assert e.value.code == B.MTS_ERR_INVALID_ARG
