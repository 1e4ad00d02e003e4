"""Pins for the oracle's attention (Sec. 2, Eq. 6-7): reuse equals full
recompute, closed forms, invariances, and a library cross-check on the CPU.
Each pin is chosen so that a dropped term, a wrong sign or index, a transposed
operand, a wrong scale or an off-by-one in the mask makes at least one fail."""
import math

import numpy as np
import pytest
import torch

import mts_workloads as W
import oracle
from helpers import draw_step_data, oracle_store_for, as_values


def _reuse_and_recompute(w, layer=0):
    data = draw_step_data(w, layers=[layer])
    store = oracle_store_for(w, data)
    got = oracle.attn_incremental(store, layer, data["q"][layer], w.page_indptr, w.page_indices,
                                  w.prefix_lens, w.new_indptr)
    worst = 0.0
    for u in range(w.batch):
        P, n = int(w.prefix_lens[u]), int(w.new_lens[u])
        lo, hi = int(w.new_indptr[u]), int(w.new_indptr[u + 1])
        if n == 0:
            continue
        hist = data["hist"][layer][u]
        k_all = np.concatenate([hist[0], data["k_new"][layer][lo:hi]])
        v_all = np.concatenate([hist[1], data["v_new"][layer][lo:hi]])
        # queries of the prefix rows are irrelevant to the rows compared: draw any
        q_all = np.concatenate([W.normal_elements(np.random.default_rng(u), (P, w.heads, w.head_dim), w.dtype),
                                data["q"][layer][lo:hi]])
        full = oracle.full_recompute(q_all, k_all, v_all)
        worst = max(worst, float(np.abs(full[P:] - got[lo:hi]).max()))
    return worst


def test_reuse_equals_recompute_tiny_config():
    """The tiny reuse-versus-recompute configuration: prefix 256 + 16 new tokens, fp32, block size 16."""
    w = W.make_workload("tiny_reuse")
    assert _reuse_and_recompute(w, layer=1) < 1e-12


@pytest.mark.parametrize("S,prefix,new,dtype", [
    (1, [5, 0], [3, 4], "f32"),
    (2, [7, 1, 0], [2, 6, 1], "bf16"),
    (16, [33, 16, 15], [9, 1, 17], "bf16"),
    (16, [0], [20], "f32"),
    (4, [10, 3], [0, 5], "f32"),        # a user with no new tokens
])
def test_reuse_equals_recompute_random(S, prefix, new, dtype):
    w = W.custom_workload("t", 5 + S, dtype, 1, 2, 8, S, prefix, new)
    assert _reuse_and_recompute(w) < 1e-12


def _small(dtype="f32", S=4, prefix=(9, 0, 5), new=(4, 6, 1), H=2, D=8, seed=3):
    w = W.custom_workload("t", seed, dtype, 1, H, D, S, list(prefix), list(new))
    data = draw_step_data(w)
    return w, data


def _run(w, data, sm_scale=None):
    store = oracle_store_for(w, data)
    return oracle.attn_incremental(store, 0, data["q"][0], w.page_indptr, w.page_indices,
                                   w.prefix_lens, w.new_indptr, sm_scale=sm_scale)


def test_constant_values_give_constant_output():
    """Softmax weights sum to one: V == c  =>  o == c."""
    w, data = _small()
    data["hist"][0] = [np.stack([h[0], np.full_like(h[1], 2.5)]) for h in data["hist"][0]]
    data["v_new"][0] = np.full_like(data["v_new"][0], 2.5)
    out = _run(w, data)
    assert np.allclose(out, 2.5, atol=1e-13)


def test_zero_keys_give_running_mean():
    """K == 0 => uniform weights over the visible rows: o_i = mean(V[0 .. P+i])."""
    w, data = _small()
    data["hist"][0] = [np.stack([np.zeros_like(h[0]), h[1]]) for h in data["hist"][0]]
    data["k_new"][0] = np.zeros_like(data["k_new"][0])
    out = _run(w, data)
    for u in range(w.batch):
        P = int(w.prefix_lens[u]); lo, hi = w.new_indptr[u], w.new_indptr[u + 1]
        v_all = as_values(np.concatenate([data["hist"][0][u][1], data["v_new"][0][lo:hi]]))
        for i in range(hi - lo):
            assert np.allclose(out[lo + i], v_all[:P + i + 1].mean(axis=0), atol=1e-13)


def test_first_token_without_prefix_returns_its_value():
    """P = 0, first new token sees only itself."""
    w, data = _small(prefix=(0,), new=(3,))
    out = _run(w, data)
    assert np.allclose(out[0], as_values(data["v_new"][0][0]), atol=1e-15)


def test_dominant_key_selects_its_value():
    """One visible key aligned with the query and very long => o = that key's V row."""
    w, data = _small(prefix=(6,), new=(2,), H=1, D=8)
    q = np.zeros((2, 1, 8), np.float32); q[:, 0, 0] = 1.0
    hist = np.array(data["hist"][0][0]); hist[0] = 0.0; hist[0, 4, 0, 0] = 500.0
    data["q"][0], data["hist"][0] = q, [hist]
    data["k_new"][0] = np.zeros_like(data["k_new"][0])
    out = _run(w, data)
    assert np.allclose(out[:, 0], as_values(hist[1, 4, 0]), atol=1e-12)


def test_future_new_tokens_are_hidden():
    """Changing K/V of new token j must not change the output of new token i < j,
    and must change the output of token j itself."""
    w, data = _small(prefix=(5,), new=(4,))
    base = _run(w, data)
    data["k_new"][0] = data["k_new"][0].copy(); data["v_new"][0] = data["v_new"][0].copy()
    data["k_new"][0][2] += 1.0; data["v_new"][0][2] -= 3.0
    out = _run(w, data)
    assert np.array_equal(out[:2], base[:2])
    assert np.abs(out[2] - base[2]).max() > 1e-3 and np.abs(out[3] - base[3]).max() > 1e-3


def test_prefix_is_fully_visible():
    """Every new token's output depends on prefix row 0 and on the last prefix row."""
    w, data = _small(prefix=(5,), new=(3,))
    base = _run(w, data)
    for row in (0, 4):
        d2 = dict(data); h = np.array(data["hist"][0][0]); h[1, row] += 4.0; d2["hist"] = {0: [h]}
        out = _run(w, d2)
        assert (np.abs(out - base).reshape(3, -1).max(axis=1) > 1e-4).all()


def test_key_shift_invariance():
    """Adding one vector c to every key shifts all logits of a query by q.c: no change."""
    w, data = _small()
    base = _run(w, data)
    c = np.linspace(-1, 1, w.head_dim).astype(np.float32)
    data["hist"][0] = [np.stack([h[0] + c, h[1]]) for h in data["hist"][0]]
    data["k_new"][0] = data["k_new"][0] + c
    assert np.allclose(_run(w, data), base, atol=1e-12)


def test_physical_page_permutation_invariance():
    """Only the logical order of a user's pages matters, not which physical pages."""
    w, data = _small(S=2)
    base = _run(w, data)
    w2 = W.custom_workload("t", 99, w.dtype, 1, w.heads, w.head_dim, w.page_size,
                           w.prefix_lens, w.new_lens, pool_factor=3.0)
    assert not np.array_equal(w2.page_indices, w.page_indices)
    assert np.array_equal(_run(w2, data), base)


def test_scale_default_and_override():
    """Default scale is 1/sqrt(D); an explicit scale is used as given."""
    w, data = _small()
    assert np.array_equal(_run(w, data), _run(w, data, sm_scale=1.0 / math.sqrt(w.head_dim)))
    assert np.abs(_run(w, data, sm_scale=1.0) - _run(w, data)).max() > 1e-3


def test_heads_are_independent():
    w, data = _small()
    base = _run(w, data)
    data["q"][0] = data["q"][0].copy(); data["q"][0][:, 1] *= -1
    out = _run(w, data)
    assert np.array_equal(out[:, 0], base[:, 0]) and np.abs(out[:, 1] - base[:, 1]).max() > 1e-3


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("prefix", [0, 37])
def test_against_library_sdpa_on_cpu(dtype, prefix):
    """Textbook scaled-dot-product attention from the library (CPU, fp64) with the
    same visibility rule written as an explicit boolean mask."""
    n, H, D, S = 12, 3, 16, 16
    w = W.custom_workload("t", 21, dtype, 1, H, D, S, [prefix], [n])
    data = draw_step_data(w)
    got = _run(w, data)
    k_all = as_values(np.concatenate([data["hist"][0][0][0], data["k_new"][0]]))
    v_all = as_values(np.concatenate([data["hist"][0][0][1], data["v_new"][0]]))
    q = as_values(data["q"][0])
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]          # [1][H][n][D]
    tk = torch.from_numpy(k_all).permute(1, 0, 2)[None]
    tv = torch.from_numpy(v_all).permute(1, 0, 2)[None]
    if prefix == 0:
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    else:
        visible = torch.arange(prefix + n)[None, :] <= (prefix + torch.arange(n))[:, None]
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=visible)
    ref = ref[0].permute(1, 0, 2).numpy()
    assert np.abs(ref - got).max() < 1e-12


def test_user_and_head_selection_matches_full_run():
    w, data = _small()
    store = oracle_store_for(w, data)
    full = _run(w, data)
    part = oracle.attn_incremental(store, 0, data["q"][0], w.page_indptr, w.page_indices,
                                   w.prefix_lens, w.new_indptr, users=[1], heads=[1])
    lo, hi = w.new_indptr[1], w.new_indptr[2]
    assert np.array_equal(part[lo:hi, 1], full[lo:hi, 1])
    assert np.isnan(part[lo:hi, 0]).all() and np.isnan(part[:lo]).all()
