"""Pins for the oracle's pointwise-aggregated attention (Sec. 2, Eq. 3; the definition is
stated in oracle/mts_oracle.py): o_i = inv_norm * sum_{j<=p_i} silu(s q_i.k_j) v_j.
Chosen so that a dropped normaliser, a wrong scale, softmax left in by mistake, a transposed
operand or an off-by-one in the mask fails at least one."""
import math

import numpy as np
import pytest

import mts_workloads as W
import oracle
from helpers import draw_step_data, oracle_store_for


def _small(dtype="f32", S=4, prefix=(9, 0, 5), new=(4, 6, 1), H=2, D=8, seed=3):
    w = W.custom_workload("t", seed, dtype, 1, H, D, S, list(prefix), list(new))
    return w, draw_step_data(w)


def _run(w, data, store=None, **kw):
    store = oracle_store_for(w, data) if store is None else store
    return oracle.attn_pointwise(store, 0, data["q"][0], w.page_indptr, w.page_indices,
                                 w.prefix_lens, w.new_indptr, **kw)


@pytest.mark.parametrize("S,prefix,new,dtype", [
    (1, [5, 0], [3, 4], "f32"),
    (2, [7, 1, 0], [2, 6, 1], "bf16"),
    (16, [33, 16, 15], [9, 1, 17], "bf16"),
    (4, [10, 3], [0, 5], "f32"),
])
def test_reuse_equals_term_by_term_recompute(S, prefix, new, dtype):
    """Paged matrix form against the unpaged term-by-term loop (independent code paths)."""
    w = W.custom_workload("t", 5 + S, dtype, 1, 2, 8, S, prefix, new)
    data = draw_step_data(w)
    got = _run(w, data, inv_norm=0.125, sm_scale=0.4)
    for u in range(w.batch):
        P, n = int(w.prefix_lens[u]), int(w.new_lens[u])
        lo, hi = int(w.new_indptr[u]), int(w.new_indptr[u + 1])
        if n == 0:
            continue
        hist = data["hist"][0][u]
        k_all = np.concatenate([hist[0], data["k_new"][0][lo:hi]])
        v_all = np.concatenate([hist[1], data["v_new"][0][lo:hi]])
        q_all = np.concatenate([W.normal_elements(np.random.default_rng(u), (P, 2, 8), dtype), data["q"][0][lo:hi]])
        full = oracle.full_recompute_pointwise(q_all, k_all, v_all, 0.125, sm_scale=0.4)
        assert np.abs(full[P:] - got[lo:hi]).max() < 1e-12


def test_worked_single_key_values():
    """One user, one token, D = 1: o = inv_norm * silu(s q k) v, by hand.
    q = 2, k = 3, s = 0.5 -> x = 3, silu(3) = 3 / (1 + e^-3); v = 4, inv_norm = 0.25."""
    w = W.custom_workload("one", 1, "f32", 1, 1, 1, 4, [0], [1])
    store = oracle.PagedStore(1, w.num_pages, 4, 1, 1, np.float32)
    k = np.full((1, 1, 1), 3.0, np.float32); v = np.full((1, 1, 1), 4.0, np.float32)
    oracle.append(store, 0, k, v, w.page_indptr, w.page_indices, w.prefix_lens, w.new_indptr)
    q = np.full((1, 1, 1), 2.0, np.float32)
    out = oracle.attn_pointwise(store, 0, q, w.page_indptr, w.page_indices, w.prefix_lens, w.new_indptr,
                                inv_norm=0.25, sm_scale=0.5)
    want = 0.25 * (3.0 / (1.0 + math.exp(-3.0))) * 4.0
    assert abs(out[0, 0, 0] - want) < 1e-15
    assert abs(want - 2.857722380259) < 1e-9          # 3 / (1 + e^-3) = 2.8577223803...


def test_zero_queries_give_zero_output_not_an_average():
    """silu(0) = 0, so q = 0 gives exactly 0 (softmax would give the mean of V)."""
    w, data = _small()
    data["q"][0] = np.zeros_like(data["q"][0])
    out = _run(w, data, inv_norm=1.0)
    assert np.all(out == 0.0)


def test_odd_part_is_linear_attention():
    """silu(x) - silu(-x) = x, hence out(q) - out(-q) = inv_norm * s * (Q K^T masked) V:
    a plain matrix product, evaluated here with its own masking."""
    w, data = _small(prefix=(9, 0, 5), new=(4, 6, 1))
    store = oracle_store_for(w, data)
    plus = _run(w, data, store, inv_norm=0.3, sm_scale=0.7)
    data_neg = dict(data); data_neg["q"] = {0: -data["q"][0]}
    minus = _run(w, data_neg, store, inv_norm=0.3, sm_scale=0.7)
    for u in range(w.batch):
        P = int(w.prefix_lens[u]); lo, hi = int(w.new_indptr[u]), int(w.new_indptr[u + 1])
        hist = data["hist"][0][u]
        K = np.concatenate([hist[0], data["k_new"][0][lo:hi]]).astype(np.float64)
        V = np.concatenate([hist[1], data["v_new"][0][lo:hi]]).astype(np.float64)
        for h in range(w.heads):
            A = np.tril(data["q"][0][lo:hi, h].astype(np.float64) @ K[:, h].T, k=P)     # keys j <= P + i
            want = 0.3 * 0.7 * (A @ V[:, h])
            assert np.abs((plus - minus)[lo:hi, h] - want).max() < 1e-12


def test_linear_in_values_and_in_the_normaliser():
    w, data = _small()
    a = _run(w, data, inv_norm=0.5)
    b = _run(w, data, inv_norm=1.5)
    assert np.abs(3.0 * a - b).max() < 1e-12
    d2 = dict(data)
    d2["hist"] = {0: [h.copy() for h in data["hist"][0]]}
    for h in d2["hist"][0]:
        h[1] *= 2.0
    d2["v_new"] = {0: 2.0 * data["v_new"][0]}
    assert np.abs(_run(w, d2, inv_norm=0.5) - 2.0 * a).max() < 1e-12


def test_future_tokens_do_not_matter():
    """Changing K/V of a later new token leaves every earlier row unchanged, and changes the
    later ones: the mask is j <= p, not j < p and not absent."""
    w, data = _small(prefix=(3,), new=(6,))
    base = _run(w, data, inv_norm=1.0)
    d2 = dict(data)
    k2, v2 = data["k_new"][0].copy(), data["v_new"][0].copy()
    k2[4] += 1.0; v2[4] -= 2.0
    d2["k_new"], d2["v_new"] = {0: k2}, {0: v2}
    out = _run(w, d2, inv_norm=1.0)
    assert np.array_equal(out[:4], base[:4])
    assert np.all(np.abs(out[4:] - base[4:]).max(axis=(1, 2)) > 1e-6)


def test_saturation_limits():
    """Large positive logits pass through (silu(x) -> x), large negative ones vanish."""
    w = W.custom_workload("sat", 2, "f32", 1, 1, 2, 4, [2], [1])
    store = oracle.PagedStore(1, w.num_pages, 4, 1, 2, np.float32)
    hist = np.zeros((2, 2, 1, 2), np.float32)
    hist[0, 0, 0] = [50.0, 0.0]; hist[1, 0, 0] = [1.0, 2.0]       # key 0: logit +50
    hist[0, 1, 0] = [-50.0, 0.0]; hist[1, 1, 0] = [7.0, 7.0]      # key 1: logit -50
    oracle.unpack(store, 0, hist, w.user_pages(0), 0)
    k = np.zeros((1, 1, 2), np.float32); v = np.full((1, 1, 2), 9.0, np.float32)   # own key: logit 0
    oracle.append(store, 0, k, v, w.page_indptr, w.page_indices, w.prefix_lens, w.new_indptr)
    q = np.array([[[1.0, 0.0]]], np.float32)
    out = oracle.attn_pointwise(store, 0, q, w.page_indptr, w.page_indices, w.prefix_lens, w.new_indptr,
                                inv_norm=1.0, sm_scale=1.0)
    assert np.allclose(out[0, 0], [50.0, 100.0], rtol=0, atol=1e-9)
