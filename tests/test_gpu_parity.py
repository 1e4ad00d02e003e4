"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Data movement is compared bit for bit (whole pool image and packed runs);
attention within the stated tolerances:
  fp32 : max |gpu - oracle| <= 1e-5
  bf16 : per (user, head) tile, max |gpu - oracle| <= 2e-2 * max |oracle|
"""
import os

import numpy as np
import pytest

import mts_workloads as W
import oracle
from helpers import draw_step_data, as_values

from conftest import KERNEL_PLAIN, KERNEL_PREFILL, KERNEL_STREAMING  # noqa: F401

pytestmark = pytest.mark.gpu

FILL = 0xFF          # unowned pool bytes: NaN patterns in both element types


def _harness():
    import gpu_harness
    return gpu_harness


def _oracle_store(w, data, do_append=True):
    store = oracle.PagedStore(w.layers, w.num_pages, w.page_size, w.heads, w.head_dim, w.np_dtype)
    store.data.view(np.uint8)[...] = FILL
    for l in data["layers"]:
        for u in range(w.batch):
            pages = w.user_pages(u)
            for start, cnt in W.host_chunks(int(w.prefix_lens[u]), w.chunk_tokens):
                oracle.unpack(store, l, data["hist"][l][u][:, start:start + cnt], pages, start)
        if do_append:
            oracle.append(store, l, data["k_new"][l], data["v_new"][l], w.page_indptr, w.page_indices,
                          w.prefix_lens, w.new_indptr)
    return store


def check_attention(w, got, ref):
    """Apply the tolerance of the workload's element type; returns the worst ratio to it."""
    worst = 0.0
    gv = as_values(got)
    assert np.isfinite(gv).all(), "non-finite attention output"
    for u in range(w.batch):
        lo, hi = int(w.new_indptr[u]), int(w.new_indptr[u + 1])
        if hi == lo:
            continue
        for h in range(w.heads):
            r = ref[lo:hi, h]
            if np.isnan(r).all():
                continue                     # (user, head) not sampled by the oracle
            err = np.abs(gv[lo:hi, h] - r).max()
            tol = 1e-5 if w.dtype == "f32" else 2e-2 * np.abs(r).max()
            assert err <= tol, f"user {u} head {h}: err {err:.3e} > tol {tol:.3e}"
            worst = max(worst, err / tol)
    return worst


CASES = {
    # name: (dtype, L, H, D, S, prefix, new, chunk)
    "f32_ragged": ("f32", 2, 3, 32, 16, [40, 16, 1, 0, 31, 100], [5, 16, 1, 3, 2, 33], 24),
    "bf16_ragged": ("bf16", 2, 3, 64, 16, [40, 16, 1, 0, 31, 300], [5, 16, 1, 3, 2, 64], 40),
    "bf16_d128_s32": ("bf16", 1, 2, 128, 32, [70, 0, 129, 513], [17, 40, 1, 32], 64),
    "bf16_d32": ("bf16", 1, 4, 32, 16, [255, 7], [9, 48], 16),
    "f32_d128_s64": ("f32", 1, 2, 128, 64, [65, 3], [2, 70], 1024),
    "bf16_multi_qtile": ("bf16", 1, 2, 64, 16, [100, 0, 37], [150, 70, 65], 1024),
    "bf16_empty_users": ("bf16", 1, 2, 64, 16, [50, 20, 0], [0, 4, 0], 1024),
}


def _case(name):
    dtype, L, H, D, S, prefix, new, chunk = CASES[name]
    return W.custom_workload(name, 100 + len(name), dtype, L, H, D, S, prefix, new, chunk_tokens=chunk)


@pytest.mark.parametrize("name", list(CASES))
def test_unpack_append_pool_image_and_pack(name):
    """unpack and append write exactly the owned slots; pack returns them byte for byte."""
    G = _harness()
    w = _case(name)
    data = draw_step_data(w)
    step = G.GpuStep(w, fill_byte=FILL)
    rng = np.random.default_rng(5)
    for l in range(w.layers):
        step.unpack_histories(data, l)
        store = _oracle_store(w, data, do_append=False)
        assert np.array_equal(step.pool_image(l), G.expected_pool_image(w, store, l, FILL)), "after unpack"
        step.append(data, l)
        store = _oracle_store(w, data, do_append=True)
        assert np.array_equal(step.pool_image(l), G.expected_pool_image(w, store, l, FILL)), "after append"
        # whole users and random sub-ranges
        users, pos, cnt = [], [], []
        for u in range(w.batch):
            T = int(w.total_lens[u])
            if T == 0:
                continue
            users += [u, u]
            a = int(rng.integers(0, T)); n = int(rng.integers(1, T - a + 1))
            pos += [0, a]; cnt += [T, n]
        got = step.pack(l, users, pos, cnt)
        for u, p, n, g in zip(users, pos, cnt, got):
            want = oracle.pack(store, l, w.user_pages(u), p, n)
            assert g.tobytes() == want.tobytes(), f"pack user {u} [{p},{p+n})"
        # the pool itself is unchanged by pack
        assert np.array_equal(step.pool_image(l), G.expected_pool_image(w, store, l, FILL))


SCHEDULES = {
    "default": {},
    # one kv tile per wavefront: every (query tile, head) longer than 32 keys is cut and merged
    "one_tile_shares": {"min_tiles": 1},
    # a single workgroup: each wavefront walks through several (user, head) segments
    "four_waves": {"max_waves": 4, "min_tiles": 1},
    "odd_shares": {"min_tiles": 3, "max_waves": 28},
}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("schedule", list(SCHEDULES))
def test_attention_small(name, schedule, attn_tuning):
    """Element by element against the oracle, under several work schedules: share boundaries
    that cut through (query tile, head)s exercise the partial accumulators and the merge
    kernel; shares that span several users exercise the segment loop."""
    G = _harness()
    w = _case(name)
    attn_tuning(**SCHEDULES[schedule])
    data = draw_step_data(w)
    step = G.GpuStep(w, fill_byte=FILL)
    store = _oracle_store(w, data)
    for l in range(w.layers):
        step.unpack_histories(data, l)
        step.append(data, l)
        got = step.attention(data, l)
        ref = oracle.attn_incremental(store, l, data["q"][l], w.page_indptr, w.page_indices,
                                      w.prefix_lens, w.new_indptr)
        check_attention(w, got, ref)


PREFILL_CASES = {
    # long new segments: the workgroup-per-query-block kernel is chosen by the library itself
    "prefill_d64": ("bf16", 1, 3, 64, 16, [100, 0, 37], [300, 520, 257], 1024),
    "prefill_d128_s32": ("bf16", 1, 2, 128, 32, [0, 70], [600, 256], 1024),
    "prefill_d128_s64": ("bf16", 1, 2, 128, 64, [513], [449], 1024),
    "prefill_mixed_lengths": ("bf16", 1, 2, 64, 16, [0, 900, 15, 64], [1025, 1, 31, 129], 1024),
}
# short and ragged segments through the same kernel, forced on
FORCED_PREFILL = ["bf16_ragged", "bf16_d128_s32", "bf16_multi_qtile", "bf16_empty_users"]


def _attention_matches_oracle(w):
    G = _harness()
    data = draw_step_data(w)
    step = G.GpuStep(w, fill_byte=FILL)
    store = _oracle_store(w, data)
    for l in range(w.layers):
        step.unpack_histories(data, l)
        step.append(data, l)
        got = step.attention(data, l)
        ref = oracle.attn_incremental(store, l, data["q"][l], w.page_indptr, w.page_indices,
                                      w.prefix_lens, w.new_indptr)
        check_attention(w, got, ref)


@pytest.mark.parametrize("name", list(PREFILL_CASES))
def test_attention_long_new_segments(name):
    """Blocks of 256 queries per workgroup: several blocks per user, a ragged last block,
    wavefronts without queries, prefixes that end inside a tile."""
    dtype, L, H, D, S, prefix, new, chunk = PREFILL_CASES[name]
    _attention_matches_oracle(W.custom_workload(name, 200 + len(name), dtype, L, H, D, S, prefix, new,
                                                chunk_tokens=chunk))


@pytest.mark.parametrize("name", FORCED_PREFILL)
def test_attention_small_through_the_prefill_kernel(name, attn_tuning):
    attn_tuning(kernel=KERNEL_PREFILL)
    _attention_matches_oracle(_case(name))


@pytest.mark.parametrize("name", ["prefill_d64", "prefill_d128_s32"])
def test_long_new_segments_through_the_streaming_kernel(name, attn_tuning):
    """The two matrix-core kernels are interchangeable: the same cases with the other one."""
    attn_tuning(kernel=KERNEL_STREAMING)
    dtype, L, H, D, S, prefix, new, chunk = PREFILL_CASES[name]
    _attention_matches_oracle(W.custom_workload(name, 200 + len(name), dtype, L, H, D, S, prefix, new,
                                                chunk_tokens=chunk))


def test_tiny_reuse_config_matches_oracle_and_recompute():
    """The tiny reuse-versus-recompute configuration (1 user, L2 H4 D32 fp32, prefix 256 + 16 new, block 16)."""
    G = _harness()
    w = W.make_workload("tiny_reuse")
    data = draw_step_data(w)
    step = G.GpuStep(w, fill_byte=FILL)
    store = _oracle_store(w, data)
    for l in range(w.layers):
        step.unpack_histories(data, l)
        step.append(data, l)
        got = step.attention(data, l)
        ref = oracle.attn_incremental(store, l, data["q"][l], w.page_indptr, w.page_indices,
                                      w.prefix_lens, w.new_indptr)
        check_attention(w, got, ref)
        k_all = np.concatenate([data["hist"][l][0][0], data["k_new"][l]])
        v_all = np.concatenate([data["hist"][l][0][1], data["v_new"][l]])
        q_all = np.concatenate([np.zeros((256, w.heads, w.head_dim), np.float32), data["q"][l]])
        full = oracle.full_recompute(q_all, k_all, v_all)[256:]
        assert np.abs(as_values(got) - full).max() <= 1e-5


def test_explicit_scale_and_plain_kernel_agree(attn_tuning):
    """sm_scale is honoured, and the plain kernel gives the same answer as the MFMA kernel."""
    G = _harness()
    w = _case("bf16_ragged")
    data = draw_step_data(w, layers=[0])
    step = G.GpuStep(w, fill_byte=FILL)
    store = _oracle_store(w, data)
    step.unpack_histories(data, 0)
    step.append(data, 0)
    ref = oracle.attn_incremental(store, 0, data["q"][0], w.page_indptr, w.page_indices,
                                  w.prefix_lens, w.new_indptr, sm_scale=0.3)
    check_attention(w, step.attention(data, 0, sm_scale=0.3), ref)
    attn_tuning(kernel=KERNEL_PLAIN)
    check_attention(w, step.attention(data, 0, sm_scale=0.3), ref)


def test_empty_batch_and_no_new_tokens_are_noops():
    import torch
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd.runtime import DeviceBatch, PagedKVCache
    cache = PagedKVCache(1, 4, 16, 2, 64, "bf16", fill_byte=FILL)
    before = cache.pool.clone()
    empty = DeviceBatch(np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(1, np.int32))
    assert mts.mts_kv_append(cache.desc, 0, None, None, empty.meta) == 0
    assert mts.mts_attn_incremental(cache.desc, 0, None, None, empty.meta) == 0
    assert mts.mts_kv_unpack(cache.desc, 0, None, 0, None, None, None, 0, empty.meta) == 0
    assert mts.mts_kv_pack(cache.desc, 0, None, 0, None, None, None, 0, empty.meta) == 0
    idle = DeviceBatch([0, 2], [1, 3], [20], [0, 0])
    assert mts.mts_kv_append(cache.desc, 0, None, None, idle.meta) == 0
    assert mts.mts_attn_incremental(cache.desc, 0, None, None, idle.meta) == 0
    torch.cuda.synchronize()
    assert torch.equal(before, cache.pool)


@pytest.mark.parametrize("prefill", [None, KERNEL_PREFILL])
def test_late_dominant_key_redoes_the_segment_with_the_exact_max(prefill, attn_tuning):
    """Both matrix-core kernels (streaming; workgroup-per-query-block, forced on).
    The reference max of a segment is taken from its first tile.  A key far later whose
    logit exceeds it by hundreds overflows the fp32 weights, which the kernel must detect and
    repair by redoing the segment with the exact max: the output is then that key's value row."""
    if prefill is not None:
        attn_tuning(kernel=prefill)
    G = _harness()
    w = W.custom_workload("dominant", 77, "bf16", 1, 2, 64, 16, [700, 90, 300], [20, 3, 40])
    data = draw_step_data(w)
    for u, tok in ((0, 555), (2, 37)):                 # small logits everywhere, one huge key
        h = np.array(data["hist"][0][u])
        h[0] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(h[0]) * 0.01)
        h[0, tok] = W.f32_to_bf16_bits(np.full((w.heads, w.head_dim), 60.0, np.float32))
        data["hist"][0][u] = h
    lo, hi = w.new_indptr[0], w.new_indptr[1]
    lo2, hi2 = w.new_indptr[2], w.new_indptr[3]
    q = W.bf16_bits_to_f32(data["q"][0]).copy()
    q[lo:hi] = np.abs(q[lo:hi]) + 0.5                  # positive queries: logit = 60 * sum(q) / 8 >> 100
    q[lo2:hi2] = np.abs(q[lo2:hi2]) + 0.5
    data["q"][0] = W.f32_to_bf16_bits(q)
    step = G.GpuStep(w, fill_byte=FILL)
    store = _oracle_store(w, data)
    step.unpack_histories(data, 0)
    step.append(data, 0)
    got = step.attention(data, 0)
    ref = oracle.attn_incremental(store, 0, data["q"][0], w.page_indptr, w.page_indices,
                                  w.prefix_lens, w.new_indptr)
    check_attention(w, got, ref)
    # sanity of the construction: the dominant key really takes all the weight
    assert np.allclose(ref[lo:hi, 0], as_values(data["hist"][0][0][1, 555, 0]), atol=1e-6)


@pytest.mark.parametrize("schedule", ["default", "one_tile_shares"])
@pytest.mark.parametrize("prefill", [None, KERNEL_PREFILL])
def test_large_values_overflow_the_numerator_before_the_denominator(prefill, schedule, attn_tuning):
    """Values of magnitude ~100 and one late key whose logit lies 85 nats above the first tile's:
    against the first tile's reference the softmax denominator stays just below the overflow
    test (e^85 = 8e36) while weight x value passes the fp32 range.  The kernels must notice the
    overflowed numerators and redo the segment with the exact max; the oracle (fp64) is finite."""
    fields = dict(SCHEDULES[schedule])
    if prefill is not None:
        fields["kernel"] = prefill
    attn_tuning(**fields)
    G = _harness()
    w = W.custom_workload("big_values", 78, "bf16", 1, 2, 64, 16, [700, 300, 64], [20, 40, 7])
    data = draw_step_data(w)
    late = {0: 555, 1: 237, 2: 50}
    for u, tok in late.items():
        h = np.array(data["hist"][0][u])
        h[0] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(h[0]) * 0.01)          # logits ~ 0 everywhere ...
        h[0, tok] = W.f32_to_bf16_bits(np.full((w.heads, w.head_dim), 10.625, np.float32))   # ... but here: 85 nats
        h[1] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(h[1]) * 100.0)         # values ~ N(0, 100^2)
        data["hist"][0][u] = h
    data["k_new"][0] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(data["k_new"][0]) * 0.01)
    data["v_new"][0] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(data["v_new"][0]) * 100.0)
    data["q"][0] = W.f32_to_bf16_bits(np.ones_like(W.bf16_bits_to_f32(data["q"][0])))   # q.k_late / 8 = 85
    step = G.GpuStep(w, fill_byte=FILL)
    store = _oracle_store(w, data)
    step.unpack_histories(data, 0)
    step.append(data, 0)
    got = step.attention(data, 0)
    ref = oracle.attn_incremental(store, 0, data["q"][0], w.page_indptr, w.page_indices,
                                  w.prefix_lens, w.new_indptr)
    assert np.isfinite(as_values(got)).all()
    check_attention(w, got, ref)
    # sanity of the construction: the late key takes all the weight, and its values are large
    lo = int(w.new_indptr[0])
    assert np.allclose(ref[lo, 0], as_values(data["hist"][0][0][1, 555, 0]), rtol=1e-6)
    assert np.abs(ref).max() > 100


EDGE_CASES = {
    # the largest batch the schedule takes (its metadata fills ~64 KiB of LDS), tiny users
    "batch_4096": lambda rng: ("bf16", 1, 1, 64, 16, rng.integers(0, 40, 4096), rng.integers(0, 4, 4096)),
    # many heads, smallest head_dim
    "heads_40_d32": lambda rng: ("bf16", 1, 40, 32, 16, [130, 0, 17], [9, 33, 1]),
    # one very long history, few new tokens: hundreds of wavefronts share one (user, head)
    "one_long_user": lambda rng: ("bf16", 1, 2, 128, 16, [70001], [5]),
    # every new segment is a single token (decode shape) over page-aligned and unaligned prefixes
    "decode_like": lambda rng: ("bf16", 1, 4, 64, 32, [0, 1, 31, 32, 33, 1024, 1025], [1] * 7),
}


@pytest.mark.parametrize("name", list(EDGE_CASES))
def test_attention_edge_shapes(name):
    rng = np.random.default_rng(len(name))
    dtype, L, H, D, S, prefix, new = EDGE_CASES[name](rng)
    w = W.custom_workload(name, 300 + len(name), dtype, L, H, D, S, np.asarray(prefix), np.asarray(new))
    _attention_matches_oracle(w)


def _random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.integers(1, 7))
    H, D, S = int(rng.integers(1, 6)), int(rng.choice([32, 64, 128])), int(rng.choice([16, 32, 64]))
    long_new = seed % 4 == 0                       # every fourth case has prefill-sized new segments
    prefix = rng.integers(0, 700, B) * (rng.random(B) > 0.2)
    new = rng.integers(0, 600 if long_new else 70, B)
    if new.sum() == 0:
        new[0] = 1
    return W.custom_workload(f"rand{seed}", 500 + seed, "bf16", 1, H, D, S, prefix.astype(np.int64), new.astype(np.int64),
                             chunk_tokens=int(rng.choice([64, 256, 1024])))


@pytest.mark.parametrize("seed", range(24))
def test_attention_random_shapes(seed):
    """Seeded random shapes (users, heads, head_dim, page size, ragged prefixes and new segments,
    empty users): whichever kernel the library picks must agree with the oracle."""
    _attention_matches_oracle(_random_case(seed))


@pytest.mark.parametrize("seed", range(12))
def test_data_movement_random_shapes(seed):
    """Long and short runs at unaligned positions, both element types, every head_dim / page size:
    the pool image after unpack and append, and packs of random sub-ranges, bit for bit."""
    G = _harness()
    rng = np.random.default_rng(2000 + seed)
    dtype = "f32" if seed % 3 == 0 else "bf16"
    H, D, S = int(rng.integers(1, 4)), int(rng.choice([32, 64, 128])), int(rng.choice([16, 32, 64]))
    B = int(rng.integers(1, 5))
    prefix = rng.integers(0, 900, B)
    new = rng.integers(0, 400, B)
    w = W.custom_workload(f"mv{seed}", 700 + seed, dtype, 1, H, D, S, prefix.astype(np.int64), new.astype(np.int64),
                          chunk_tokens=int(rng.choice([100, 129, 256, 1000])))
    data = draw_step_data(w)
    step = G.GpuStep(w, fill_byte=FILL)
    step.unpack_histories(data, 0)
    store = _oracle_store(w, data, do_append=False)
    assert np.array_equal(step.pool_image(0), G.expected_pool_image(w, store, 0, FILL)), "after unpack"
    step.append(data, 0)
    store = _oracle_store(w, data, do_append=True)
    assert np.array_equal(step.pool_image(0), G.expected_pool_image(w, store, 0, FILL)), "after append"
    users, pos, cnt = [], [], []
    for u in range(w.batch):
        T = int(w.total_lens[u])
        for _ in range(3):
            if T == 0:
                continue
            a = int(rng.integers(0, T)); n = int(rng.integers(1, T - a + 1))
            users.append(u); pos.append(a); cnt.append(n)
    if users:
        got = step.pack(0, users, pos, cnt)
        for u, p, n, g in zip(users, pos, cnt, got):
            assert g.tobytes() == oracle.pack(store, 0, w.user_pages(u), p, n).tobytes(), f"pack user {u} [{p},{p+n})"
    assert np.array_equal(step.pool_image(0), G.expected_pool_image(w, store, 0, FILL)), "pack must not write the pool"


@pytest.mark.parametrize("dtype,D,S", [("bf16", 64, 16), ("f32", 32, 32), ("bf16", 128, 64)])
def test_several_layers_in_one_launch(dtype, D, S):
    """mts_kv_unpack_layers / mts_kv_pack_layers on a range of layers inside a larger cache: the
    layers of the range hold exactly what the oracle's unpack wrote, the layers outside it and the
    padding between the per-layer staging blocks stay untouched, and the packed runs equal the
    oracle's pack bit for bit."""
    import torch
    import paper_2604_22881_amd as mts
    from paper_2604_22881_amd.runtime import SegmentList
    G = _harness()
    L, lo, cnt_l = 4, 1, 2
    prefix, new = [300, 17, 0, 129, 640], [5, 0, 40, 3, 200]
    w = W.custom_workload("layers", 4242, dtype, L, 3, D, S, prefix, new, chunk_tokens=200)
    data = draw_step_data(w, layers=range(lo, lo + cnt_l))
    step = G.GpuStep(w, fill_byte=FILL)
    H, es = w.heads, w.elem_bytes
    row = 2 * H * D                                           # elements per token (K and V)

    # ---- unpack: runs of every history, layer blocks `stride` elements apart (padded) ----
    users = [u for u in range(w.batch) if prefix[u] > 0]
    segs = SegmentList.for_histories(users, [prefix[u] for u in users], w.chunk_tokens, G.DEV)
    su, sp, sc = segs.seg_user.cpu().numpy(), segs.seg_pos.cpu().numpy(), np.diff(segs.host_indptr)
    stride = segs.total_tokens * row + 24                     # 24 elements of padding: 48 or 96 bytes
    host = np.zeros(cnt_l * stride, dtype=w.np_dtype)
    for i in range(cnt_l):
        parts = [np.ascontiguousarray(data["hist"][lo + i][su[s]][:, sp[s]:sp[s] + sc[s]]).reshape(-1)
                 for s in range(segs.num_segs)]
        host[i * stride:i * stride + segs.total_tokens * row] = np.concatenate(parts)
    mts.mts_kv_unpack_layers(step.cache.desc, lo, cnt_l, G.to_dev(host), stride * es, *segs.args(), step.batch.meta)
    torch.cuda.synchronize()
    store = _oracle_store(w, data, do_append=False)
    for l in range(L):
        assert np.array_equal(step.pool_image(l), G.expected_pool_image(w, store, l, FILL)), f"layer {l} after unpack"

    for l in range(lo, lo + cnt_l):
        step.append(data, l)
    store = _oracle_store(w, data, do_append=True)

    # ---- pack: random sub-ranges and whole users, all layers of the range in one launch ----
    rng = np.random.default_rng(9)
    pu, pp, pc = [], [], []
    for u in range(w.batch):
        T = int(w.total_lens[u])
        if T == 0:
            continue
        a = int(rng.integers(0, T)); n = int(rng.integers(1, T - a + 1))
        pu += [u, u]; pp += [0, a]; pc += [T, n]
    psegs = SegmentList(pu, pp, pc, G.DEV)
    pstride = psegs.total_tokens * row + 8
    guard = 12345 if dtype == "bf16" else 0.5
    out = torch.full((cnt_l * pstride,), guard, dtype=torch.float32 if dtype == "f32" else torch.int16, device=G.DEV)
    mts.mts_kv_pack_layers(step.cache.desc, lo, cnt_l, out, pstride * es, *psegs.args(), step.batch.meta)
    torch.cuda.synchronize()
    flat = G.to_host(out, w.np_dtype)
    for i in range(cnt_l):
        off = i * pstride
        for u, p, n in zip(pu, pp, pc):
            want = oracle.pack(store, lo + i, w.user_pages(u), p, n)
            assert flat[off:off + want.size].tobytes() == want.tobytes(), f"layer {lo + i} user {u} [{p},{p + n})"
            off += want.size
        pad = flat[off:(i + 1) * pstride]
        assert pad.size == 8 and (pad == flat.dtype.type(guard)).all(), "padding between layers was written"
        # the one-layer call returns the same bytes
        single = step.pack(lo + i, pu, pp, pc)
        assert b"".join(g.tobytes() for g in single) == flat[i * pstride:i * pstride + psegs.total_tokens * row].tobytes()
    for l in range(L):
        assert np.array_equal(step.pool_image(l), G.expected_pool_image(w, store, l, FILL)), f"layer {l} after pack"


@pytest.mark.parametrize("dtype,D,S", [("bf16", 64, 16), ("f32", 32, 32), ("bf16", 128, 64)])
def test_append_several_layers_in_one_launch(dtype, D, S):
    """mts_kv_append_layers on a range of layers inside a larger cache (row buffers a padded
    stride apart): those layers hold exactly what the oracle's append wrote after the histories,
    the others are untouched."""
    import torch
    import paper_2604_22881_amd as mts
    G = _harness()
    L, lo, cnt_l = 4, 1, 3
    prefix, new = [300, 17, 0, 129, 640], [5, 0, 40, 3, 200]
    w = W.custom_workload("append_layers", 4243, dtype, L, 3, D, S, prefix, new, chunk_tokens=200)
    data = draw_step_data(w, layers=range(lo, lo + cnt_l))
    step = G.GpuStep(w, fill_byte=FILL)
    for l in range(lo, lo + cnt_l):
        step.unpack_histories(data, l)
    n = w.total_new * w.heads * D
    stride = n + 40                                           # elements; 80 or 160 bytes of padding
    k = np.zeros(cnt_l * stride, dtype=w.np_dtype)
    v = np.zeros(cnt_l * stride, dtype=w.np_dtype)
    for i in range(cnt_l):
        k[i * stride:i * stride + n] = np.ascontiguousarray(data["k_new"][lo + i]).reshape(-1)
        v[i * stride:i * stride + n] = np.ascontiguousarray(data["v_new"][lo + i]).reshape(-1)
    mts.mts_kv_append_layers(step.cache.desc, lo, cnt_l, G.to_dev(k), G.to_dev(v), stride * w.elem_bytes,
                             step.batch.meta)
    torch.cuda.synchronize()
    store = _oracle_store(w, data, do_append=True)
    for l in range(L):
        assert np.array_equal(step.pool_image(l), G.expected_pool_image(w, store, l, FILL)), f"layer {l}"
