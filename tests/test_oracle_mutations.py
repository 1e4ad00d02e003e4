"""The pins must be able to fail: plant typical mistakes in the oracle (on the
CPU, by patching it) and check that a pin notices each of them."""
import numpy as np
import pytest

import oracle
from oracle import mts_oracle
import test_oracle_attention as TA
import test_oracle_cache as TC


def _fails(fn, *args):
    try:
        fn(*args)
    except AssertionError:
        return True
    return False


def test_wrong_scale_is_caught(monkeypatch):
    real = mts_oracle.attn_incremental

    def mutant(store, layer, q, *a, sm_scale=None, **kw):
        return real(store, layer, q, *a, sm_scale=1.0 / store.D if sm_scale is None else sm_scale, **kw)
    monkeypatch.setattr(oracle, "attn_incremental", mutant)
    assert _fails(TA.test_against_library_sdpa_on_cpu, "f32", 37)
    assert _fails(TA.test_reuse_equals_recompute_tiny_config)


def test_softmax_over_wrong_axis_is_caught(monkeypatch):
    def mutant(z):
        e = np.exp(z - z.max())
        return e / e.sum(axis=0, keepdims=True)
    monkeypatch.setattr(mts_oracle, "_softmax_rows", mutant)
    assert _fails(TA.test_constant_values_give_constant_output)
    assert _fails(TA.test_reuse_equals_recompute_tiny_config)


def test_unmasked_future_is_caught(monkeypatch):
    def mutant(z):                       # treats hidden (-inf) logits as zero logits
        z = np.where(np.isinf(z), 0.0, z)
        e = np.exp(z - z.max(axis=-1, keepdims=True))
        return e / e.sum(axis=-1, keepdims=True)
    monkeypatch.setattr(mts_oracle, "_softmax_rows", mutant)
    assert _fails(TA.test_future_new_tokens_are_hidden)
    assert _fails(TA.test_first_token_without_prefix_returns_its_value)


def test_swapped_page_and_slot_is_caught(monkeypatch):
    def mutant(self, page_list, t):
        return int(page_list[(t // self.S)]), (self.S - 1) - t % self.S
    monkeypatch.setattr(mts_oracle.PagedStore, "slot", mutant)
    assert _fails(TC.test_token_lands_in_page_t_div_s_slot_t_mod_s)


def test_k_v_planes_swapped_in_pack_is_caught(monkeypatch):
    real = mts_oracle.pack
    monkeypatch.setattr(oracle, "pack", lambda *a, **k: real(*a, **k)[::-1].copy())
    assert _fails(TC.test_pack_after_unpack_is_identity, "bf16", 16, 16)
    assert _fails(TC.test_append_then_pack_is_concatenation)
