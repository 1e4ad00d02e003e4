"""Plain model of the host-side KVCacheManager: TEST INFRASTRUCTURE ONLY.

What is modelled, and where the paper states it:

* Sec. 3.1 (KVCacheManager): sequence-length tracking, LRU replacement and a page
  table whose entries each track one fixed-length segment of a user's cache.
* Sec. 4.3 (Allocation and Eviction Policy): pages are drawn from the free pool;
  when it is exhausted, pages are reclaimed from the least-recently-used users;
  reclamation is a metadata operation, the host tier being the backup.
* Sec. 4.3 (User Locking Protocol): users under offload are skipped as victims.
* Sec. 4.2 (Transient Offload Pipeline): offload of a user is triggered once its
  not-yet-persisted tokens reach the host chunk size; whole chunks are persisted.
* App. C.1: a user of length T needs ceil(T / S) pages (rounding per user).

Readings where the paper is silent: a whole user is evicted at a time; users of
the batch being prepared are never victims; evicting a user whose newest tokens
were not persisted yet drops those tokens from the cache (its cached length falls
back to the persisted length); a batch that cannot be placed even after evicting
every eligible user is refused and leaves the state untouched; a prepared batch
that is abandoned (its step failed before the commit of Alg. 1 step 7) gives back
the pages that prepare allotted and takes back its request counts, while users
evicted to make room for it stay evicted.

Written with an ordered dict and lists for clarity, not speed.  Which physical
page ids a user receives is not modelled (any free page is as good as another):
the model tracks page COUNTS, and tests check ids for disjointness instead.
"""
from __future__ import annotations

from collections import OrderedDict


class CacheModel:
    def __init__(self, num_pages: int, page_size: int, host_chunk_tokens: int):
        self.num_pages, self.S, self.chunk = num_pages, page_size, host_chunk_tokens
        self.free = num_pages
        self.total = {}              # user -> tokens cached on either tier
        self.host = {}               # user -> tokens persisted in the host tier
        self.pages = {}              # user -> pages held in the GPU tier
        self.lru = OrderedDict()     # users in the GPU tier, least recent first
        self.locked = set()
        self.evicted = []
        self.batch = None
        self.stats = dict(gpu_hits=0, host_hits=0, cold_requests=0, evictions=0, tokens_dropped=0)

    def pages_for(self, n: int) -> int:
        return -(-n // self.S)

    def import_history(self, user, total_len: int):
        """A user whose whole history is persisted in the host tier and absent from the GPU."""
        assert user not in self.total
        self.total[user] = self.host[user] = total_len

    def cached_length(self, user) -> int:
        return self.total.get(user, 0)

    def prepare_batch(self, users, new_tokens):
        """Returns (prefix_lens, onload_lens, pages_per_user) or None if refused."""
        assert self.batch is None and len(set(users)) == len(users)
        in_batch = set(users)
        need = sum(self.pages_for(self.total.get(u, 0) + n) - self.pages.get(u, 0) for u, n in zip(users, new_tokens))
        victims = [v for v in self.lru if v not in self.locked and v not in in_batch]     # least recent first
        if self.free + sum(self.pages[v] for v in victims) < need:
            return None
        for v in victims:
            if self.free >= need:
                break
            self._evict(v)
        prefix, onload, counts = [], [], []
        for u, n in zip(users, new_tokens):
            t = self.total.get(u, 0)
            on_gpu = u in self.lru
            prefix.append(t)
            onload.append(0 if on_gpu else t)
            key = "cold_requests" if t == 0 else ("gpu_hits" if on_gpu else "host_hits")
            self.stats[key] += 1
            want = self.pages_for(t + n)
            self.free -= want - self.pages.get(u, 0)
            self.pages[u] = want
            counts.append(want)
        self.batch = list(zip(users, new_tokens))
        return prefix, onload, counts

    def abort_batch(self):
        """The prepared batch will not run: every user goes back to the pages its cached tokens
        need in the GPU tier (none if it is not there), and the batch's requests are uncounted."""
        for u, _ in self.batch:
            t = self.total.get(u, 0)
            on_gpu = u in self.lru
            keep = self.pages_for(t) if on_gpu else 0
            self.free += self.pages.get(u, 0) - keep
            if keep:
                self.pages[u] = keep
            else:
                self.pages.pop(u, None)
            key = "cold_requests" if t == 0 else ("gpu_hits" if on_gpu else "host_hits")
            self.stats[key] -= 1
        self.batch = None

    def _evict(self, v):
        del self.lru[v]
        self.free += self.pages.pop(v)
        self.stats["tokens_dropped"] += self.total[v] - self.host.get(v, 0)
        self.total[v] = self.host.get(v, 0)
        self.evicted.append(v)
        self.stats["evictions"] += 1

    def commit_batch(self):
        for u, n in self.batch:
            self.total[u] = self.total.get(u, 0) + n
            self.lru.pop(u, None)
            if self.total[u] > 0:
                self.lru[u] = True            # most recent at the end
        self.batch = None

    def offload_due(self):
        """[(user, from_pos, count)], most recent user first; locks them."""
        due = []
        for u in reversed(self.lru):
            fresh = self.total[u] - self.host.get(u, 0)
            if u in self.locked or fresh < self.chunk:
                continue
            due.append((u, self.host.get(u, 0), fresh // self.chunk * self.chunk))
            self.locked.add(u)
        return due

    def offload_done(self, user, persisted_len):
        assert self.host.get(user, 0) <= persisted_len <= self.total[user]
        self.host[user] = persisted_len
        self.locked.discard(user)

    def take_evicted(self):
        out, self.evicted = self.evicted, []
        return out
