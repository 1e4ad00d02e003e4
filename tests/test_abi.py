"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments on the host before anything is launched (no GPU needed: every call here either
is host-only or fails validation)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2604_22881_amd as mts
from paper_2604_22881_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # aligned, never dereferenced: validation fails first


def _desc(**kw):
    d = dict(pool=FAKE, layer_stride_bytes=1 << 20, dtype=B.MTS_BF16, num_layers=2, num_pages=8,
             page_size=16, num_heads=4, head_dim=64)
    d.update(kw)
    return B.CacheDesc(**d)


def _meta(**kw):
    d = dict(batch=2, page_indptr=FAKE, page_indices=FAKE, prefix_lens=FAKE, new_indptr=FAKE,
             total_new=10, max_new=8, max_total_len=100, total_pages=8)
    d.update(kw)
    return B.BatchMeta(**d)


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "mtserve.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(mts_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert mts.mts_version() >= 100


def test_page_bytes_and_pages_for():
    assert mts.mts_page_bytes(_desc()) == 2 * 4 * 16 * 64 * 2
    assert mts.mts_page_bytes(_desc(dtype=B.MTS_F32, head_dim=32, page_size=32)) == 2 * 4 * 32 * 32 * 4
    # App. C.1: 32-token pages, H4 D128 bf16 -> 64 KiB per page and layer
    assert mts.mts_page_bytes(_desc(page_size=32, head_dim=128)) == 65536
    assert mts.mts_pages_for(40008, 32) == 1251 and mts.mts_pages_for(0, 16) == 0
    assert mts.mts_pages_for(17, 16) == 2
    with pytest.raises(mts.MtsError):
        mts.mts_pages_for(-1, 16)


@pytest.mark.parametrize("dtype,D,S", [(B.MTS_BF16, 64, 16), (B.MTS_BF16, 128, 32), (B.MTS_F32, 32, 16),
                                       (B.MTS_F32, 128, 64), (B.MTS_BF16, 32, 64)])
def test_elem_offset_is_a_bijection_with_16_byte_granules(dtype, D, S):
    H = 3
    d = _desc(dtype=dtype, head_dim=D, page_size=S, num_heads=H)
    es = 2 if dtype == B.MTS_BF16 else 4
    G = 16 // es
    offs = np.array([[[[mts.mts_elem_offset(d, kv, h, s, x) for x in range(D)] for s in range(S)]
                      for h in range(H)] for kv in (0, 1)])
    assert sorted(offs.reshape(-1).tolist()) == list(range(0, 2 * H * S * D * es, es))
    # K: G consecutive dims of one token share a granule; V: G consecutive tokens of one dim do
    k, v = offs[0], offs[1]
    assert (np.diff(k.reshape(H, S, D // G, G), axis=-1) == es).all()
    assert (k[..., ::G] % 16 == 0).all()
    vt = v.transpose(0, 2, 1).reshape(H, D, S // G, G)
    assert (np.diff(vt, axis=-1) == es).all() and (vt[..., 0] % 16 == 0).all()
    # a head's K block precedes its V block, heads are contiguous runs of 2*S*D*es bytes
    for h in range(H):
        base = h * 2 * S * D * es
        assert k[h].min() == base and k[h].max() < base + S * D * es <= v[h].min()
    with pytest.raises(mts.MtsError):
        mts.mts_elem_offset(d, 2, 0, 0, 0)
    with pytest.raises(mts.MtsError):
        mts.mts_elem_offset(d, 0, 0, S, 0)


def test_workspace_query_is_host_only():
    d = _desc(head_dim=128)
    small = _meta(batch=4, total_new=64, max_new=16, max_total_len=200, total_pages=60)
    big = _meta(batch=32, total_new=1024, max_new=32, max_total_len=16416, total_pages=330000 // 16)
    assert mts.mts_attn_workspace_bytes(d, small) >= 0
    assert mts.mts_attn_workspace_bytes(d, big) > 0
    assert mts.mts_attn_workspace_bytes(_desc(dtype=B.MTS_F32), small) == 0


def _code(fn, *a, **k):
    with pytest.raises(mts.MtsError) as e:
        fn(*a, **k)
    assert mts.mts_last_error() != ""
    return e.value.code


def test_bad_descriptors_are_rejected():
    m = _meta()
    assert _code(mts.mts_kv_append, _desc(dtype=7), 0, FAKE, FAKE, m, stream=0) == B.MTS_ERR_UNSUPPORTED
    assert _code(mts.mts_kv_append, _desc(head_dim=48), 0, FAKE, FAKE, m, stream=0) == B.MTS_ERR_UNSUPPORTED
    assert _code(mts.mts_kv_append, _desc(page_size=8), 0, FAKE, FAKE, m, stream=0) == B.MTS_ERR_UNSUPPORTED
    assert _code(mts.mts_kv_append, _desc(pool=None), 0, FAKE, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_append, _desc(pool=FAKE + 8), 0, FAKE, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_append, _desc(layer_stride_bytes=1024), 0, FAKE, FAKE, m, stream=0) == B.MTS_ERR_SHAPE
    assert _code(mts.mts_kv_append, _desc(), 2, FAKE, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_append, _desc(), -1, FAKE, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_append, _desc(num_heads=0), 0, FAKE, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG


def test_bad_batches_and_buffers_are_rejected():
    d = _desc()
    assert _code(mts.mts_kv_append, d, 0, FAKE, FAKE, _meta(batch=-1), stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_append, d, 0, FAKE, FAKE, _meta(total_new=-3), stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_append, d, 0, FAKE, FAKE, _meta(total_new=17), stream=0) == B.MTS_ERR_SHAPE
    assert _code(mts.mts_kv_append, d, 0, FAKE, FAKE, _meta(max_total_len=4), stream=0) == B.MTS_ERR_SHAPE
    assert _code(mts.mts_kv_append, d, 0, None, FAKE, _meta(), stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_append, d, 0, FAKE + 4, FAKE, _meta(), stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_append, d, 0, FAKE, FAKE, _meta(new_indptr=None), stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_attn_incremental, d, 0, None, FAKE, _meta(), stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_attn_incremental, d, 0, FAKE, FAKE, _meta(), sm_scale=-1.0, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_attn_incremental, d, 0, FAKE, FAKE, _meta(), sm_scale=float("nan"), stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_attn_incremental, d, 0, FAKE, FAKE, _meta(page_indices=None), stream=0) == B.MTS_ERR_INVALID_ARG
    for bad in (0.0, -0.5, float("nan"), float("inf")):
        assert _code(mts.mts_attn_pointwise, d, 0, FAKE, FAKE, _meta(), bad, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_attn_pointwise, d, 0, None, FAKE, _meta(), 0.5, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_attn_pointwise, d, 0, FAKE, FAKE, _meta(), 0.5, sm_scale=-1.0, stream=0) == B.MTS_ERR_INVALID_ARG


def test_missing_or_short_workspace_is_rejected():
    d = _desc(head_dim=128)
    big = _meta(batch=32, total_new=1024, max_new=32, max_total_len=16416, total_pages=330000 // 16)
    need = mts.mts_attn_workspace_bytes(d, big)
    assert need > 0
    assert _code(mts.mts_attn_incremental, d, 0, FAKE, FAKE, big, workspace=None, workspace_bytes=0,
                 stream=0) == B.MTS_ERR_WORKSPACE
    assert _code(mts.mts_attn_incremental, d, 0, FAKE, FAKE, big, workspace=FAKE, workspace_bytes=need - 1,
                 stream=0) == B.MTS_ERR_WORKSPACE
    assert _code(mts.mts_attn_incremental, d, 0, FAKE, FAKE, big, workspace=FAKE + 16, workspace_bytes=need,
                 stream=0) == B.MTS_ERR_WORKSPACE


def test_bad_segments_are_rejected():
    d, m = _desc(), _meta()
    assert _code(mts.mts_kv_unpack, d, 0, FAKE, -1, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_unpack, d, 0, FAKE, 2, None, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_unpack, d, 0, None, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_unpack, d, 0, FAKE + 2, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_unpack, d, 0, FAKE, 2, FAKE, FAKE, FAKE, -4, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_pack, d, 0, None, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_pack, d, 5, FAKE, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_kv_pack, d, 0, FAKE, 2, FAKE, FAKE, FAKE, 4, _meta(batch=0), stream=0) == B.MTS_ERR_SHAPE
    assert _code(mts.mts_stage_h2d_async, None, FAKE, 16, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_stage_d2h_async, FAKE, FAKE, -1, stream=0) == B.MTS_ERR_INVALID_ARG


def test_bad_layer_ranges_are_rejected():
    d, m = _desc(), _meta()          # the descriptor has 2 layers
    for fn in (mts.mts_kv_unpack_layers, mts.mts_kv_pack_layers):
        assert _code(fn, d, 0, 3, FAKE, 4096, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
        assert _code(fn, d, 1, 2, FAKE, 4096, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
        assert _code(fn, d, 2, 0, FAKE, 4096, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
        assert _code(fn, d, 0, -1, FAKE, 4096, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
        assert _code(fn, d, 0, 2, FAKE, 4096 + 8, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
        assert _code(fn, d, 0, 2, FAKE, -4096, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
        assert _code(fn, d, 0, 2, None, 4096, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
        assert _code(fn, d, 0, 2, FAKE, 4096, 2, None, FAKE, FAKE, 4, m, stream=0) == B.MTS_ERR_INVALID_ARG
        assert _code(fn, d, 0, 2, FAKE, 4096, 2, FAKE, FAKE, FAKE, 4, _meta(batch=0), stream=0) == B.MTS_ERR_SHAPE
        # nothing to move: accepted without touching a pointer
        assert fn(d, 0, 0, None, 0, 2, FAKE, FAKE, FAKE, 4, m, stream=0) == 0
        assert fn(d, 0, 2, None, 0, 0, None, None, None, 0, m, stream=0) == 0


def test_bad_append_layers_arguments_are_rejected():
    d, m = _desc(), _meta()          # the descriptor has 2 layers
    fn = mts.mts_kv_append_layers
    assert _code(fn, d, 0, 3, FAKE, FAKE, 4096, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 1, 2, FAKE, FAKE, 4096, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 0, -1, FAKE, FAKE, 4096, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 0, 2, None, FAKE, 4096, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 0, 2, FAKE, FAKE + 4, 4096, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 0, 2, FAKE, FAKE, 4100, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert fn(d, 0, 0, None, None, 0, m, stream=0) == 0
    assert fn(d, 0, 2, None, None, 0, _meta(total_new=0, max_new=0), stream=0) == 0


def test_unappended_attention_arguments():
    d, m = _desc(), _meta()
    fn = mts.mts_attn_incremental_unappended
    assert _code(fn, d, 0, FAKE, None, FAKE, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 0, FAKE, FAKE, FAKE + 2, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(mts.mts_attn_pointwise_unappended, d, 0, FAKE, FAKE, FAKE, FAKE, m, 0.0, stream=0) == B.MTS_ERR_INVALID_ARG
    # which shapes the unappended calls append by themselves: fp32 caches and long new segments
    assert mts.mts_attn_unappended_appends(d, m) is False
    assert mts.mts_attn_unappended_appends(_desc(dtype=B.MTS_F32), m) is True
    long_new = _meta(batch=2, total_new=1024, max_new=512, max_total_len=600, total_pages=8)
    assert mts.mts_attn_unappended_appends(d, long_new) is True


def test_staged_attention_arguments():
    d, m = _desc(), _meta()
    fn = mts.mts_attn_incremental_staged
    ok = (d, 0, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 64, FAKE, m)
    assert _code(fn, d, 0, FAKE, FAKE, FAKE, None, FAKE, FAKE, 64, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 0, FAKE, FAKE, FAKE, FAKE, None, FAKE, 64, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 0, FAKE, FAKE, FAKE, FAKE, FAKE, None, 64, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 0, FAKE, FAKE, FAKE, FAKE + 2, FAKE, FAKE, 64, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    for chunk in (0, 48, -64):
        assert _code(fn, d, 0, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, chunk, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    assert _code(fn, d, 0, FAKE, None, FAKE, FAKE, FAKE, FAKE, 64, FAKE, m, stream=0) == B.MTS_ERR_INVALID_ARG
    # shapes the streaming bf16 kernel does not serve
    assert _code(fn, _desc(dtype=B.MTS_F32), *ok[1:], workspace=FAKE, workspace_bytes=1 << 30, stream=0) == B.MTS_ERR_UNSUPPORTED
    long_new = _meta(batch=2, total_new=1024, max_new=512, max_total_len=600, total_pages=8)
    assert _code(fn, *ok[:-1], long_new, stream=0) == B.MTS_ERR_UNSUPPORTED


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()


def test_transfer_pipeline_rejects_bad_arguments():
    """Host-side validation of the mts_xfer_* calls; creating a pipeline needs a GPU, so without
    one the call must come back with an error code, not crash."""
    for kw in (dict(pinned_bytes=0, num_layers=2), dict(pinned_bytes=1 << 20, num_layers=0),
               dict(pinned_bytes=1 << 20, num_layers=2, copy_threads=0),
               dict(pinned_bytes=1 << 20, num_layers=2, offload_arena_bytes=-1)):
        with pytest.raises(mts.MtsError) as e:
            mts.mts_xfer_create(**kw)
        assert e.value.code == B.MTS_ERR_INVALID_ARG
    lib = B.lib()
    assert lib.mts_xfer_destroy(None) == B.MTS_OK
    assert lib.mts_xfer_drain(None) == B.MTS_ERR_INVALID_ARG
    assert lib.mts_xfer_onload_wait_layer(None, 0, None) == B.MTS_ERR_INVALID_ARG
    assert lib.mts_xfer_offload_pending_tokens(None) == B.MTS_ERR_INVALID_ARG
    runs = B.XferRuns(0, None, None, None, 0, None, None)
    assert lib.mts_xfer_onload_submit(None, C.byref(_desc()), C.byref(_meta()), C.byref(runs), None, 0) == B.MTS_ERR_INVALID_ARG
    try:
        h = mts.mts_xfer_create(pinned_bytes=1 << 16, num_layers=2)
    except mts.MtsError as err:
        assert err.code == B.MTS_ERR_HIP          # no device here
    else:
        mts.mts_xfer_destroy(h)


def test_shapes_beyond_the_schedule_are_refused_not_launched():
    d = _desc()
    too_many_users = _meta(batch=4097, total_new=4097, max_new=1, max_total_len=10, total_pages=4097)
    with pytest.raises(mts.MtsError) as e:
        mts.mts_attn_workspace_bytes(d, too_many_users)
    assert e.value.code == B.MTS_ERR_UNSUPPORTED
    assert _code(mts.mts_attn_incremental, d, 0, FAKE, FAKE, too_many_users, workspace=FAKE, workspace_bytes=1 << 30,
                 stream=0) == B.MTS_ERR_UNSUPPORTED
    assert _code(mts.mts_kv_append, d, 0, FAKE, FAKE, _meta(batch=70000), stream=0) == B.MTS_ERR_INVALID_ARG


def test_random_descriptors_and_metadata_never_crash():
    """Whatever the scalar fields say, every entry point returns a code (or succeeds as a no-op):
    the host-side checks run before any device work, so this needs no GPU."""
    rng = np.random.default_rng(4)
    pick = lambda *v: v[int(rng.integers(0, len(v)))]
    codes = {B.MTS_ERR_INVALID_ARG, B.MTS_ERR_UNSUPPORTED, B.MTS_ERR_SHAPE, B.MTS_ERR_WORKSPACE, B.MTS_ERR_HIP}
    for _ in range(400):
        d = _desc(pool=pick(FAKE, 0, FAKE + 4), layer_stride_bytes=int(pick(1 << 20, 0, -16, 100, 1 << 40)),
                  dtype=int(pick(B.MTS_BF16, B.MTS_F32, 7, -1)), num_layers=int(pick(2, 0, -3, 1 << 20)),
                  num_pages=int(pick(8, 0, -1, 1 << 30)), page_size=int(pick(16, 32, 64, 0, 8, 48, -16)),
                  num_heads=int(pick(4, 0, -2, 1 << 16)), head_dim=int(pick(64, 32, 128, 0, 24, 256, -64)))
        m = _meta(batch=int(pick(2, 0, -1, 5000, 1 << 30)), page_indptr=pick(FAKE, 0), page_indices=pick(FAKE, 0),
                  prefix_lens=pick(FAKE, 0), new_indptr=pick(FAKE, 0), total_new=int(pick(10, 0, -5, 1 << 30)),
                  max_new=int(pick(8, 0, -1, 300, 1 << 30)), max_total_len=int(pick(100, 0, -1, 1 << 30)),
                  total_pages=int(pick(8, 0, -1, 1 << 30)))
        layer = int(pick(0, 1, -1, 99))
        calls = [
            lambda: mts.mts_page_bytes(d),
            lambda: mts.mts_attn_workspace_bytes(d, m),
            lambda: mts.mts_kv_unpack(d, layer, None, 2, None, None, None, 4, m, stream=0),
            lambda: mts.mts_kv_pack_layers(d, layer, 2, None, 64, 2, None, None, None, 4, m, stream=0),
            lambda: mts.mts_kv_append(d, layer, None, None, m, stream=0),
            lambda: mts.mts_kv_append_layers(d, layer, 3, None, None, 64, m, stream=0),
            lambda: mts.mts_attn_incremental(d, layer, None, None, m, stream=0),
            lambda: mts.mts_attn_pointwise(d, layer, None, None, m, 0.5, stream=0),
            lambda: mts.mts_attn_incremental_unappended(d, layer, None, None, None, None, m, stream=0),
            lambda: mts.mts_attn_incremental_staged(d, layer, None, None, None, None, None, None, 64, None, m, stream=0),
            lambda: mts.mts_attn_unappended_appends(d, m),
        ]
        for call in calls:
            try:
                call()                        # no-op shapes (empty batch, nothing to move) succeed
            except mts.MtsError as e:
                assert e.code in codes and mts.mts_last_error() != ""
