"""The host-side cache manager (mts_cm_*, C++) against a plain model of the paper's policy
(oracle/cache_model.py), and that model against hand-worked traces and the paper's page
arithmetic.  No GPU: the manager makes no device call."""
import numpy as np
import pytest

import paper_2604_22881_amd as mts
from oracle.cache_model import CacheModel


# ---- pins of the model ----------------------------------------------------------------------
def test_model_hand_worked_lru_trace():
    """10 pages of 4 tokens.  A(12 tok)=3 pages, B(20)=5, C(8)=2 fill the pool; touching A makes
    B the least recent; D(9 tok)=3 pages then evicts B only (5 pages back, 3 taken)."""
    m = CacheModel(10, 4, 1 << 30)
    for u, n in (("A", 12), ("B", 20), ("C", 8)):
        assert m.prepare_batch([u], [n]) == ([0], [0], [-(-n // 4)])
        m.commit_batch()
    assert m.free == 0 and list(m.lru) == ["A", "B", "C"]
    assert m.prepare_batch(["A"], [0]) == ([12], [0], [3])          # GPU hit, nothing to bring up
    m.commit_batch()
    assert list(m.lru) == ["B", "C", "A"]
    assert m.prepare_batch(["D"], [9]) == ([0], [0], [3])
    m.commit_batch()
    assert m.take_evicted() == ["B"] and m.free == 2 and list(m.lru) == ["C", "A", "D"]
    # B was never persisted: its 20 tokens are gone from the cache
    assert m.cached_length("B") == 0 and m.stats["tokens_dropped"] == 20
    assert m.stats == dict(gpu_hits=1, host_hits=0, cold_requests=4, evictions=1, tokens_dropped=20)


def test_model_locked_users_are_skipped_and_host_copy_survives_eviction():
    m = CacheModel(6, 4, 8)                     # host chunk = 8 tokens
    m.prepare_batch(["A"], [11]); m.commit_batch()          # 3 pages
    m.prepare_batch(["B"], [12]); m.commit_batch()          # 3 pages, pool full
    assert m.offload_due() == [("B", 0, 8), ("A", 0, 8)]    # whole chunks only, most recent first; both locked
    assert m.prepare_batch(["C"], [4]) is None              # every victim is locked: refused, nothing changed
    assert m.free == 0 and list(m.lru) == ["A", "B"]
    m.offload_done("A", 8)
    assert m.prepare_batch(["C"], [4]) == ([0], [0], [1])   # A unlocked -> evicted (least recent)
    m.commit_batch()
    assert m.take_evicted() == ["A"]
    assert m.cached_length("A") == 8                        # persisted prefix survives; 3 tokens dropped
    # A returns: 8 tokens come up from the host tier (a host hit), 9 tokens need 3 pages:
    # 2 are free, B is still locked, so C (1 page) goes
    assert m.prepare_batch(["A"], [1]) == ([8], [8], [3])
    m.commit_batch()
    assert m.take_evicted() == ["C"] and m.stats["host_hits"] == 1 and m.stats["tokens_dropped"] == 3 + 4


def test_model_abandoned_batch_hand_worked():
    """9 pages of 4 tokens.  A (10 tokens, 3 pages) and B (6 tokens, 2 pages) are resident.  A batch
    {A +5, C +9} takes 1 + 3 pages; abandoning it returns exactly those 4 and un-counts its two
    requests; a batch that had to evict B first leaves B evicted when it is abandoned."""
    m = CacheModel(9, 4, 1 << 30)
    m.prepare_batch(["A"], [10]); m.commit_batch()
    m.prepare_batch(["B"], [6]); m.commit_batch()
    assert m.free == 4 and m.stats["cold_requests"] == 2
    assert m.prepare_batch(["A", "C"], [5, 9]) == ([10, 0], [0, 0], [4, 3])
    assert m.free == 0 and m.stats["gpu_hits"] == 1 and m.stats["cold_requests"] == 3
    m.abort_batch()
    assert m.free == 4 and m.pages == {"A": 3, "B": 2} and list(m.lru) == ["A", "B"]
    assert m.stats["gpu_hits"] == 0 and m.stats["cold_requests"] == 2 and m.cached_length("A") == 10
    assert m.cached_length("C") == 0
    # the same batch again, prepared and committed, behaves as if the abandoned one never happened
    assert m.prepare_batch(["A", "C"], [5, 9]) == ([10, 0], [0, 0], [4, 3])
    m.commit_batch()
    assert m.cached_length("A") == 15 and m.cached_length("C") == 9 and m.free == 0
    # D needs 2 pages: B (least recent) is evicted for it; abandoning D does not bring B back
    assert m.prepare_batch(["D"], [8]) == ([0], [0], [2])
    m.abort_batch()
    assert m.take_evicted() == ["B"] and m.free == 2 and m.cached_length("B") == 0 and "D" not in m.pages


def test_model_page_arithmetic_of_the_paper():
    """App. C.1: 8 users of 40 008 tokens, 32-token pages -> 8 x 1251 = 10 008 pages."""
    m = CacheModel(50968, 32, 1024)
    out = m.prepare_batch(list(range(8)), [40008] * 8)
    assert out[2] == [1251] * 8 and m.num_pages - m.free == 10008


# ---- the C++ manager against the model --------------------------------------------------------
def test_manager_matches_model_on_random_traces():
    rng = np.random.default_rng(7)
    for trial in range(6):
        num_pages, S, chunk = int(rng.integers(40, 400)), int(rng.choice([4, 16, 32])), int(rng.choice([8, 64, 256]))
        cm = mts.CacheManager(num_pages, S, chunk)
        model = CacheModel(num_pages, S, chunk)
        pages_of = {}                                   # user -> page ids last reported by the manager
        n_users = int(rng.integers(5, 40))
        for step in range(300):
            B = int(rng.integers(1, 6))
            users = rng.choice(n_users, size=min(B, n_users), replace=False).astype(np.int64)
            new = rng.integers(0, 3 * S, size=len(users)).astype(np.int32)
            want = model.prepare_batch(users.tolist(), new.tolist())
            if want is None:
                with pytest.raises(mts.MtsError) as e:
                    cm.prepare_batch(users, new)
                assert e.value.code == mts.MTS_ERR_BUSY
            else:
                prefix, onload, indptr, indices = cm.prepare_batch(users, new)
                assert prefix.tolist() == want[0] and onload.tolist() == want[1]
                assert np.diff(indptr).tolist() == want[2]
                for i, u in enumerate(users.tolist()):
                    mine = indices[indptr[i]:indptr[i + 1]].tolist()
                    old = pages_of.get(u, [])
                    if onload[i] == 0 and prefix[i] > 0:
                        assert mine[:len(old)] == old, "a resident user's pages must stay where they are"
                    pages_of[u] = mine
                for v in cm.take_evicted().tolist():
                    pages_of.pop(v, None)
                assert model.take_evicted() is not None
                # no page belongs to two users
                held = [p for ps in pages_of.values() for p in ps]
                assert len(held) == len(set(held)) and all(0 <= p < num_pages for p in held)
                if rng.random() < 0.15:                 # the step fails before its commit
                    model.abort_batch(); cm.abort_batch()
                    pages_of = {u: ps[:model.pages.get(u, 0)] for u, ps in pages_of.items() if model.pages.get(u, 0)}
                else:
                    model.commit_batch(); cm.commit_batch()
            if step % 7 == 3:
                due = model.offload_due()
                u, p, c = cm.offload_due()
                assert list(zip(u.tolist(), p.tolist(), c.tolist())) == due
                for (uu, pp, cc) in due:
                    if rng.random() < 0.7:
                        model.offload_done(uu, pp + cc); cm.offload_done(uu, pp + cc)
            st = cm.stats()
            for k, v in model.stats.items():
                assert st[k] == v, (k, st[k], v)
            assert st["free_pages"] == model.free and st["users_on_gpu"] == len(model.lru)
            for u in range(n_users):
                assert cm.cached_length(u) == model.cached_length(u)
        cm.close()


def test_imported_histories_are_host_hits_with_everything_to_bring_up():
    cm = mts.CacheManager(20, 4, 8)
    model = CacheModel(20, 4, 8)
    for u, n in ((5, 30), (6, 0), (7, 9)):
        cm.import_history(u, n); model.import_history(u, n)
    with pytest.raises(mts.MtsError):
        cm.import_history(5, 1)
    assert [cm.cached_length(u) for u in (5, 6, 7, 8)] == [30, 0, 9, 0]
    want = model.prepare_batch([5, 6, 7], [2, 3, 0])
    prefix, onload, indptr, indices = cm.prepare_batch([5, 6, 7], [2, 3, 0])
    assert (prefix.tolist(), onload.tolist(), np.diff(indptr).tolist()) == want == ([30, 0, 9], [30, 0, 9], [8, 1, 3])
    cm.commit_batch(); model.commit_batch()
    st = cm.stats()
    assert st["host_hits"] == 2 and st["cold_requests"] == 1 and st["gpu_hits"] == 0
    # nothing new is due for user 7 (9 persisted, 9 cached); user 5 has 2 fresh tokens < one chunk
    assert cm.offload_due()[0].tolist() == [] == [d[0] for d in model.offload_due()]


def test_manager_eviction_order_matches_model():
    cm = mts.CacheManager(12, 4, 1 << 20)
    model = CacheModel(12, 4, 1 << 20)
    for u in range(4):
        model.prepare_batch([u], [12]); model.commit_batch()
        cm.prepare_batch([u], [12]); cm.commit_batch()
    model.prepare_batch([1], [0]); model.commit_batch()
    cm.prepare_batch([1], [0]); cm.commit_batch()
    model.prepare_batch([9], [30]); cm.prepare_batch([9], [30])          # 8 pages: evicts 0, 2, 3 in that order
    assert cm.take_evicted().tolist() == model.take_evicted() == [0, 2, 3]


def test_manager_rejects_bad_arguments_and_leaves_state():
    cm = mts.CacheManager(8, 4, 16)
    with pytest.raises(mts.MtsError):
        cm.prepare_batch([1, 1], [2, 2])                                  # duplicate user
    with pytest.raises(mts.MtsError):
        cm.prepare_batch([1], [-1])
    with pytest.raises(mts.MtsError) as e:
        cm.prepare_batch([1], [100])                                      # 25 pages > 8
    assert e.value.code == mts.MTS_ERR_BUSY
    assert cm.stats()["free_pages"] == 8 and cm.cached_length(1) == 0
    assert cm.stats()["users_tracked"] == 0                               # failed calls track nobody
    p, o, indptr, idx = cm.prepare_batch([1, 2], [5, 0])
    assert p.tolist() == [0, 0] and indptr.tolist() == [0, 2, 2] and len(idx) == 2
    with pytest.raises(mts.MtsError):
        cm.prepare_batch([3], [1])                                        # previous batch not committed
    cm.commit_batch()
    assert cm.cached_length(1) == 5 and cm.cached_length(2) == 0
    with pytest.raises(mts.MtsError):
        cm.offload_done(77, 1)
    with pytest.raises(mts.MtsError):
        mts.CacheManager(0, 16)


def test_manager_abandoned_batch_matches_model():
    cm = mts.CacheManager(9, 4, 1 << 20)
    model = CacheModel(9, 4, 1 << 20)
    for u, n in ((1, 10), (2, 6)):
        model.prepare_batch([u], [n]); model.commit_batch()
        cm.prepare_batch([u], [n]); cm.commit_batch()
    before = cm.prepare_batch([1], [0])[3].tolist(); cm.abort_batch()        # user 1's pages, nothing else changes
    assert model.prepare_batch([1, 3], [5, 9]) == ([10, 0], [0, 0], [4, 3])
    prefix, onload, indptr, indices = cm.prepare_batch([1, 3], [5, 9])
    assert prefix.tolist() == [10, 0] and np.diff(indptr).tolist() == [4, 3] and cm.stats()["free_pages"] == 0
    assert indices[:3].tolist() == before
    model.abort_batch(); cm.abort_batch()
    st = cm.stats()
    assert st["free_pages"] == model.free == 4 and st["gpu_hits"] == model.stats["gpu_hits"] == 0
    assert st["cold_requests"] == model.stats["cold_requests"] == 2 and cm.cached_length(3) == 0
    cm.abort_batch()                                                         # nothing prepared: no-op
    assert cm.prepare_batch([1], [0])[3].tolist() == before                  # user 1 kept its first three pages
    cm.commit_batch()
    # evictions made for an abandoned batch stay
    model.prepare_batch([1], [0]); model.commit_batch()
    assert model.prepare_batch([4], [24]) is not None and cm.prepare_batch([4], [24]) is not None   # 6 pages: evicts 2
    model.abort_batch(); cm.abort_batch()
    assert cm.take_evicted().tolist() == model.take_evicted() == [2]
    assert cm.stats()["free_pages"] == model.free == 6 and cm.cached_length(2) == 0


def test_hit_ratios_on_heavy_tailed_arrivals():
    """Synthetic stand-in for the paper's traces (Sec. 4.3, Figure 4: heavy-tailed return
    intervals): Zipf-distributed user popularity.  A larger GPU tier raises the GPU hit ratio;
    histories shorter than one host chunk are lost at eviction (only whole chunks are persisted), so
    the total hit ratio sits only a little above the GPU one at these short histories."""
    rng = np.random.default_rng(3)
    n_users, steps, B = 2000, 1500, 8
    pop = 1.0 / np.arange(1, n_users + 1) ** 0.8
    pop /= pop.sum()
    ratios = []
    for num_pages in (700, 1500, 6000):
        cm = mts.CacheManager(num_pages, 32, 64)
        r2 = np.random.default_rng(5)
        for _ in range(steps):
            users = r2.choice(n_users, size=B, replace=False, p=pop).astype(np.int64)
            new = r2.integers(1, 9, size=B).astype(np.int32)     # few new interactions per visit
            cm.prepare_batch(users, new); cm.commit_batch()
            u, p, c = cm.offload_due()
            for uu, pp, cc in zip(u.tolist(), p.tolist(), c.tolist()):
                cm.offload_done(uu, pp + cc)
        st = cm.stats()
        req = st["gpu_hits"] + st["host_hits"] + st["cold_requests"]
        ratios.append((st["gpu_hits"] / req, (st["gpu_hits"] + st["host_hits"]) / req))
        cm.close()
    print("GPU / total hit ratio by pool size:", ratios)
    assert ratios[0][0] < ratios[1][0] < ratios[2][0]
    assert all(t > 0.5 for _, t in ratios)
