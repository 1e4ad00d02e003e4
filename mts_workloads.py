"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module only DRAWS inputs: user-history shapes, block tables and random
element values.  It contains none of the method (no attention, no cache index
maps beyond counting how many pages a user must be given) and imports neither
the HIP binding nor the oracle, so both can be fed from it.

The five named workloads are the synthetic stand-ins for the paper's trace
replays (Sec. 5.1; App. B dataset statistics): lengths follow the ranges of the
dataset table, model shapes follow the HSTU configurations of Sec. 5.1, and the
miss fraction follows the >98.5 % total hit ratio of Table 1.  No item of
either dataset is reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

WORKLOADS = ("tiny_reuse", "batched_incremental", "long_history", "host_staging", "miss_prefill")
_BASE_SEED = 1000


@dataclass
class Workload:
    name: str
    seed: int
    dtype: str            # "f32" or "bf16"
    batch: int
    layers: int
    heads: int
    head_dim: int
    page_size: int
    prefix_lens: np.ndarray      # [B] int32, tokens cached before the step
    new_lens: np.ndarray         # [B] int32, tokens processed in the step
    new_indptr: np.ndarray       # [B+1] int32
    page_indptr: np.ndarray      # [B+1] int32
    page_indices: np.ndarray     # [page_indptr[B]] int32, physical page ids
    num_pages: int               # pool size (pages per layer)
    miss_users: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    evict_users: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    chunk_tokens: int = 1024     # host chunk granularity (Sec. 4.1, CPU tier)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.uint16

    @property
    def total_new(self) -> int:
        return int(self.new_indptr[-1])

    @property
    def total_lens(self) -> np.ndarray:
        return self.prefix_lens + self.new_lens

    def user_pages(self, u: int) -> np.ndarray:
        return self.page_indices[self.page_indptr[u]:self.page_indptr[u + 1]]

    def kv_row_bytes(self) -> int:
        """Bytes of one token's K and V over all heads, one layer."""
        return 2 * self.heads * self.head_dim * self.elem_bytes


# --------------------------------------------------------------------------
# element values
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns -> the float32 values they denote."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_elements(rng: np.random.Generator, shape, dtype: str, scale: float = 1.0) -> np.ndarray:
    """N(0, scale^2) draws stored as float32 values or as bf16 bit patterns."""
    x = rng.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


# --------------------------------------------------------------------------
# shapes and block tables
# --------------------------------------------------------------------------
def _ceil_div(a, b):
    return (a + b - 1) // b


def scattered_block_tables(rng, total_lens, page_size, pool_factor=1.5):
    """Give every user ceil(T/S) pages drawn from a random permutation of a pool
    ``pool_factor`` times as large as the demand, so that a user's pages are
    physically scattered as after long churn of the free list (Sec. 4.1: any
    free page may go to any user)."""
    need = _ceil_div(np.asarray(total_lens, dtype=np.int64), page_size)
    page_indptr = np.zeros(len(need) + 1, dtype=np.int32)
    page_indptr[1:] = np.cumsum(need)
    total = int(page_indptr[-1])
    num_pages = max(1, int(np.ceil(pool_factor * total)))
    perm = rng.permutation(num_pages).astype(np.int32)
    return page_indptr, perm[:total].copy(), num_pages


def _lognormal_lengths(rng, count, median, sigma, lo, hi):
    x = np.exp(rng.normal(np.log(median), sigma, size=count))
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


def custom_workload(name, seed, dtype, layers, heads, head_dim, page_size,
                    prefix_lens, new_lens, pool_factor=1.5, miss_users=(), evict_users=(),
                    chunk_tokens=1024) -> Workload:
    """Assemble a workload from explicit per-user lengths (used by edge-case tests)."""
    rng = np.random.default_rng([seed, 7])      # block-table stream, apart from the length draws
    prefix_lens = np.asarray(prefix_lens, dtype=np.int32)
    new_lens = np.asarray(new_lens, dtype=np.int32)
    new_indptr = np.zeros(len(new_lens) + 1, dtype=np.int32)
    new_indptr[1:] = np.cumsum(new_lens)
    page_indptr, page_indices, num_pages = scattered_block_tables(
        rng, prefix_lens + new_lens, page_size, pool_factor)
    return Workload(name=name, seed=seed, dtype=dtype, batch=len(prefix_lens), layers=layers,
                    heads=heads, head_dim=head_dim, page_size=page_size,
                    prefix_lens=prefix_lens, new_lens=new_lens, new_indptr=new_indptr,
                    page_indptr=page_indptr, page_indices=page_indices, num_pages=num_pages,
                    miss_users=np.asarray(miss_users, dtype=np.int32),
                    evict_users=np.asarray(evict_users, dtype=np.int32),
                    chunk_tokens=chunk_tokens)


def make_workload(name: str, seed: int | None = None) -> Workload:
    """One seeded draw of a named workload.

    tiny_reuse           1 user, L2 H4 D32 fp32, prefix 256, 16 new tokens
    batched_incremental  64 users, L4 H8 D64 bf16, prefix ~ lognormal(median 1500,
                         sigma 0.6) clipped to [128, 4096], new ~ U{8..64};
                         1 user (ceil of 1.5 %) is restored from a staged host
                         copy and 1 other user is packed for offload
    long_history         32 users, L8 H8 D128 bf16, prefix ~ U{4096..16384}, 32 new
    host_staging         256 users, L4 H8 D64 bf16, prefix ~ lognormal(median 2000,
                         sigma 0.6) clipped to [128, 8192], new ~ U{8..64};
                         4 miss users (ceil of 1.5 %), 4 other users evicted
    miss_prefill         16 users, L8 H16 D128 bf16, prefix 0, 4096 new tokens
    """
    if name not in WORKLOADS:
        raise KeyError(f"unknown workload {name!r}; choose from {WORKLOADS}")
    idx = WORKLOADS.index(name)
    seed = _BASE_SEED + idx + 1 if seed is None else seed
    rng = np.random.default_rng(seed)
    miss = evict = ()
    if name == "tiny_reuse":
        dtype, L, H, D = "f32", 2, 4, 32
        prefix, new = np.array([256]), np.array([16])
    elif name == "batched_incremental":
        dtype, L, H, D = "bf16", 4, 8, 64
        prefix = _lognormal_lengths(rng, 64, 1500, 0.6, 128, 4096)
        new = rng.integers(8, 65, size=64)
        order = rng.permutation(64)
        miss, evict = order[:1], order[1:2]
    elif name == "long_history":
        dtype, L, H, D = "bf16", 8, 8, 128
        prefix = rng.integers(4096, 16385, size=32)
        new = np.full(32, 32)
    elif name == "host_staging":
        dtype, L, H, D = "bf16", 4, 8, 64
        prefix = _lognormal_lengths(rng, 256, 2000, 0.6, 128, 8192)
        new = rng.integers(8, 65, size=256)
        order = rng.permutation(256)
        miss, evict = order[:4], order[4:8]
    else:  # miss_prefill
        dtype, L, H, D = "bf16", 8, 16, 128
        prefix, new = np.zeros(16, dtype=np.int64), np.full(16, 4096)
    w = custom_workload(name, seed, dtype, L, H, D, 16, prefix, new,
                        miss_users=np.sort(np.asarray(miss, dtype=np.int32)),
                        evict_users=np.sort(np.asarray(evict, dtype=np.int32)))
    return w


def with_page_size(w: Workload, page_size: int) -> Workload:
    """The same users, lengths and roles with the pool cut into pages of another size (block
    tables redrawn from the workload's seed)."""
    if page_size == w.page_size:
        return w
    return custom_workload(w.name, w.seed, w.dtype, w.layers, w.heads, w.head_dim, page_size,
                           w.prefix_lens, w.new_lens, miss_users=w.miss_users, evict_users=w.evict_users,
                           chunk_tokens=w.chunk_tokens)


def host_chunks(length: int, chunk_tokens: int):
    """Token ranges [(start, count), ...] of a history kept on the host in
    fixed-size chunks (Sec. 4.1, CPU tier); the last chunk may be short."""
    return [(s, min(chunk_tokens, length - s)) for s in range(0, length, chunk_tokens)]
