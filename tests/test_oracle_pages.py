"""Pins for the oracle's page and byte arithmetic: the sizes the paper prints
(App. C.1, App. D.2 capacity table, Sec. 1 storage claim)."""
import os

import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_page_arithmetic.txt")


def _load():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                k, v = line.split()
                vals[k] = int(v)
    return vals


G = _load()


def test_onload_pages_round_per_user():
    assert G["batch"] * G["max_len"] == G["peak_tokens"]
    assert oracle.onload_pages(G["batch"], G["max_len"], G["model_page_size"]) == G["onload_pages"]
    # rounding the whole batch at once does NOT give the printed page count
    assert oracle.pages_for(G["peak_tokens"], G["model_page_size"]) != G["onload_pages"]
    assert G["primary_pages"] + G["onload_pages"] == G["total_pages"]


def test_store_bytes_matches_appendix():
    b = oracle.store_bytes(G["model_layers"], G["total_pages"], G["model_page_size"],
                           G["model_heads"], G["model_head_dim"], G["elem_bytes"])
    assert b == G["store_mib"] * 2**20


@pytest.mark.parametrize("gb", [10, 15, 20, 25, 30])
def test_capacity_table(gb):
    b = oracle.store_bytes(G["model_layers"], G[f"capacity_pages_{gb}gb"], G["model_page_size"],
                           G["model_heads"], G["model_head_dim"], G["elem_bytes"])
    assert b == gb * 2**30


def test_storage_claim():
    per_tok = oracle.kv_bytes_per_token(G["model_layers"], G["model_heads"], G["model_head_dim"], G["elem_bytes"])
    assert per_tok == 16384
    total = per_tok * G["claim_users"] * G["claim_tokens"]
    assert total == 163_840_000_000 and total > G["claim_exceeds_gb"] * 10**9


@pytest.mark.parametrize("length,S,want", [(0, 16, 0), (1, 16, 1), (16, 16, 1), (17, 16, 2),
                                           (40008, 32, 1251), (272, 16, 17), (1, 1, 1)])
def test_pages_for(length, S, want):
    assert oracle.pages_for(length, S) == want


def test_attended_pairs_complexity():
    """Sec. 2: reuse costs O((T - P_pre) T), recompute O(T^2)."""
    for P, n in [(0, 5), (256, 16), (1000, 1), (7, 9)]:
        reuse, full = oracle.attended_pairs(P, n)
        T = P + n
        assert full == T * (T + 1) // 2
        assert reuse == full - P * (P + 1) // 2        # the rows reuse skips
        assert n * P < reuse <= n * T
