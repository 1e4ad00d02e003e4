"""Pins for the oracle's paged store: unpack / append / pack are exact index
maps (Sec. 3.2 steps 3, 5, 6; Sec. 4.1 store shape)."""
import numpy as np
import pytest

import mts_workloads as W
import oracle
from helpers import draw_step_data, oracle_store_for

SENTINEL_F32 = np.float32(-777.25)
SENTINEL_BF16 = np.uint16(0xABCD)


def _w(dtype="bf16", S=16, prefix=(40, 16, 1, 0, 31), new=(5, 16, 1, 3, 2), H=3, D=8, chunk=16):
    return W.custom_workload("t", 17, dtype, 2, H, D, S, list(prefix), list(new), chunk_tokens=chunk)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("S,chunk", [(16, 16), (16, 24), (4, 10), (1, 3)])
def test_pack_after_unpack_is_identity(dtype, S, chunk):
    w = _w(dtype, S=S, chunk=chunk)
    data = draw_step_data(w)
    store = oracle_store_for(w, data, do_append=False)
    for l in range(w.layers):
        for u in range(w.batch):
            P = int(w.prefix_lens[u])
            got = oracle.pack(store, l, w.user_pages(u), 0, P)
            assert got.dtype == w.np_dtype and got.shape == (2, P, w.heads, w.head_dim)
            assert np.array_equal(got, data["hist"][l][u])
            # any sub-range, not only page-aligned ones
            if P > 3:
                assert np.array_equal(oracle.pack(store, l, w.user_pages(u), 2, P - 3),
                                      data["hist"][l][u][:, 2:P - 1])


def test_token_lands_in_page_t_div_s_slot_t_mod_s():
    """Read every token back directly from the [L, N, 2, S, H, D] tensor."""
    w = _w("f32", S=4)
    data = draw_step_data(w)
    store = oracle_store_for(w, data, do_append=False)
    for u in range(w.batch):
        pages = w.user_pages(u)
        for t in range(int(w.prefix_lens[u])):
            for kv in (0, 1):
                assert np.array_equal(store.data[1, pages[t // 4], kv, t % 4], data["hist"][1][u][kv, t])


@pytest.mark.parametrize("dtype,sentinel", [("f32", SENTINEL_F32), ("bf16", SENTINEL_BF16)])
def test_unowned_slots_are_untouched(dtype, sentinel):
    w = _w(dtype)
    data = draw_step_data(w)
    store = oracle_store_for(w, data, fill=sentinel)
    owned = np.zeros(store.data.shape[:4], dtype=bool)       # [L][page][2][slot]
    for u in range(w.batch):
        pages = w.user_pages(u)
        for t in range(int(w.total_lens[u])):
            owned[:, pages[t // w.page_size], :, t % w.page_size] = True
    assert (store.data[~owned] == sentinel).all()
    assert owned.sum() == w.layers * 2 * int(w.total_lens.sum())


def test_append_then_pack_is_concatenation():
    w = _w("bf16")
    data = draw_step_data(w)
    store = oracle_store_for(w, data)
    for l in range(w.layers):
        for u in range(w.batch):
            lo, hi = w.new_indptr[u], w.new_indptr[u + 1]
            want = np.concatenate([data["hist"][l][u],
                                   np.stack([data["k_new"][l][lo:hi], data["v_new"][l][lo:hi]])], axis=1)
            assert np.array_equal(oracle.pack(store, l, w.user_pages(u), 0, int(w.total_lens[u])), want)


def test_layers_are_independent():
    w = _w("f32")
    data = draw_step_data(w, layers=[1])
    store = oracle_store_for(w, data, fill=SENTINEL_F32)
    assert (store.data[0] == SENTINEL_F32).all()


def test_range_checks():
    w = _w("f32")
    store = oracle.PagedStore(w.layers, w.num_pages, w.page_size, w.heads, w.head_dim, np.float32)
    pages = w.user_pages(0)
    seg = np.zeros((2, 5, w.heads, w.head_dim), np.float32)
    with pytest.raises(ValueError):
        oracle.unpack(store, 0, seg, pages, len(pages) * w.page_size - 4)
    with pytest.raises(ValueError):
        oracle.pack(store, 0, pages, -1, 2)


def test_bf16_decode_is_exact():
    bits = np.array([0x0000, 0x3F80, 0xBF80, 0x4049, 0x0001, 0x7F7F, 0x8000], dtype=np.uint16)
    want = [0.0, 1.0, -1.0, 3.140625, 2.0 ** -133, (2 - 2 ** -7) * 2.0 ** 127, -0.0]
    got = oracle.decode_values(bits)
    assert got.tolist() == want and np.signbit(got[-1])
