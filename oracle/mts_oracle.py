"""Plain, slow, fp64 CPU statement of what the hot path computes.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is modelled, and where the paper defines it:

* The GPU tier of the cache is one pre-allocated tensor of shape
  ``[L, N_pages, 2, S_page, H, D]`` (Sec. 4.1, "GPU Tier (Fine-grained
  Paging)"; App. C.1 gives the same shape for ``cache_table``).  The oracle
  keeps exactly that arrangement.  A user owns an ordered list of page ids;
  token ``t`` of the user lives in page ``list[t // S]``, slot ``t % S``
  (Sec. 3.1, KVCacheManager: each page-table entry tracks one fixed-length
  segment of the user's KV cache).
* Cache Scattering (Sec. 3.2 step 3, Sec. 4.2): contiguous onload-buffer data
  is redistributed into the user's pages -> :func:`unpack`.
* Cache Update (Sec. 3.2 step 5; Alg. 1 step 8.2): the K/V of the tokens
  processed in this step are written behind the cached prefix -> :func:`append`.
* Cache Offload, gather half (Sec. 3.2 step 6, Sec. 4.2): dispersed pages are
  collected into a contiguous buffer -> :func:`pack`.
* Model Inference with reuse (Sec. 2, Eq. 6-7; Alg. 1 step 8.4): the new
  tokens' queries attend to ``[K_pre; k_delta]`` / ``[V_pre; v_delta]`` read
  through the page table -> :func:`attn_incremental`.
* The recompute baseline (Sec. 5.1 "RE"; Sec. 2 cost O(T^2)): causal attention
  over all T tokens on contiguous tensors, knowing nothing of pages ->
  :func:`full_recompute`.  Reuse must reproduce its last ``T - P_pre`` rows.

* The pointwise variant of the same step -> :func:`attn_pointwise` and
  :func:`full_recompute_pointwise`.  Sec. 2 (Eq. 1-3) takes its backbone from
  the HSTU line of work and leaves ``Attention`` undefined; that line of work
  aggregates with an elementwise SiLU of the scaled logits and a length
  normaliser instead of a softmax.  The definition used here,
  ``o_i = inv_norm * sum_{j<=p_i} silu(s * q_i . k_j) v_j``, is this build's
  statement of it (the paper prints no formula): parity of the GPU path is
  per this definition.

Readings taken where the paper is silent: ``Attention`` is scaled-dot-product
softmax attention with scale 1/sqrt(D) unless given; no positional bias; one
head count for Q, K and V; causal order among the new tokens and full view of
the prefix.  The contiguous (host / onload-buffer) layout of a run of ``n``
tokens of one user and one layer is ``[2 (K, V)][n][H][D]``.

Element types: ``float32`` arrays hold values; ``uint16`` arrays hold bfloat16
bit patterns.  All arithmetic is float64.
"""
from __future__ import annotations

import math

import numpy as np


# --------------------------------------------------------------------------
# page / byte arithmetic (Sec. 4.1; App. C.1)
# --------------------------------------------------------------------------
def pages_for(length: int, page_size: int) -> int:
    """Pages one user needs for ``length`` tokens: the ceiling of length / S_page.

    Rounding is per user: a page belongs to exactly one user (Sec. 4.1).
    """
    if length < 0 or page_size <= 0:
        raise ValueError("length >= 0 and page_size > 0 required")
    return (length + page_size - 1) // page_size


def onload_pages(batch: int, max_len: int, page_size: int) -> int:
    """Onload-buffer capacity N_o in pages (App. C.1).

    Each of the ``batch`` users may bring ``max_len`` tokens and every user's
    run is rounded up to whole pages, so N_o = batch * ceil(max_len / S_page).
    (The appendix prints the quotient for the whole batch at once, which does
    not reproduce its own page total; the per-user rounding does.)
    """
    return batch * pages_for(max_len, page_size)


def store_bytes(L: int, n_pages: int, page_size: int, H: int, D: int, elem_bytes: int) -> int:
    """Bytes of a ``[L, N_pages, 2, S_page, H, D]`` store (App. C.1)."""
    return L * n_pages * 2 * page_size * H * D * elem_bytes


def kv_bytes_per_token(L: int, H: int, D: int, elem_bytes: int) -> int:
    """K and V bytes one token occupies over all layers (Sec. 1, storage claim)."""
    return L * 2 * H * D * elem_bytes


def attended_pairs(prefix: int, new: int) -> tuple[int, int]:
    """(query, key) pairs evaluated with reuse and with recompute (Sec. 2).

    With reuse only the ``new`` queries run, query i seeing prefix + i + 1 keys;
    recompute runs all T = prefix + new queries causally.
    """
    T = prefix + new
    reuse = sum(prefix + i + 1 for i in range(new))
    recompute = T * (T + 1) // 2
    return reuse, recompute


# --------------------------------------------------------------------------
# element decoding
# --------------------------------------------------------------------------
def decode_values(raw: np.ndarray) -> np.ndarray:
    """Stored elements -> float64 values (exact for both element types)."""
    raw = np.asarray(raw)
    if raw.dtype == np.uint16:  # bfloat16 = the upper half of an IEEE float32
        as_f32 = (raw.astype(np.uint32) << np.uint32(16)).view(np.float32)
        return as_f32.astype(np.float64)
    if raw.dtype == np.float32:
        return raw.astype(np.float64)
    raise TypeError(f"unsupported element type {raw.dtype}")


# --------------------------------------------------------------------------
# the paged store and the three data-movement operations
# --------------------------------------------------------------------------
class PagedStore:
    """GPU-tier Paged Store ``[L, N_pages, 2, S_page, H, D]`` (Sec. 4.1)."""

    def __init__(self, L, n_pages, page_size, H, D, dtype, fill=None):
        dtype = np.dtype(dtype)
        if dtype not in (np.dtype(np.float32), np.dtype(np.uint16)):
            raise TypeError("dtype must be float32 or uint16 (bf16 bits)")
        self.L, self.n_pages, self.S, self.H, self.D = L, n_pages, page_size, H, D
        self.data = np.zeros((L, n_pages, 2, page_size, H, D), dtype=dtype)
        if fill is not None:
            self.data[...] = fill

    def slot(self, page_list, t):
        """(page id, slot) of a user's token ``t`` given the user's page list."""
        return int(page_list[t // self.S]), t % self.S


def _check_run(store, page_list, pos, n):
    if pos < 0 or n < 0:
        raise ValueError("negative position or length")
    if pos + n > len(page_list) * store.S:
        raise ValueError("token range exceeds the user's allocated pages")


def unpack(store: PagedStore, layer: int, segment: np.ndarray, page_list, dst_pos: int) -> None:
    """Scatter a contiguous run into the user's pages (Sec. 3.2 step 3).

    ``segment`` is ``[2][n][H][D]``; its token ``i`` becomes the user's token
    ``dst_pos + i``.  Only those n slots change.
    """
    n = segment.shape[1]
    _check_run(store, page_list, dst_pos, n)
    for i in range(n):
        page, slot = store.slot(page_list, dst_pos + i)
        store.data[layer, page, 0, slot] = segment[0, i]
        store.data[layer, page, 1, slot] = segment[1, i]


def pack(store: PagedStore, layer: int, page_list, src_pos: int, n: int) -> np.ndarray:
    """Gather the user's tokens ``src_pos .. src_pos+n-1`` into ``[2][n][H][D]``
    (Sec. 3.2 step 6, the gather kernel of Sec. 4.2)."""
    _check_run(store, page_list, src_pos, n)
    out = np.empty((2, n, store.H, store.D), dtype=store.data.dtype)
    for i in range(n):
        page, slot = store.slot(page_list, src_pos + i)
        out[0, i] = store.data[layer, page, 0, slot]
        out[1, i] = store.data[layer, page, 1, slot]
    return out


def append(store: PagedStore, layer: int, k_new, v_new, page_indptr, page_indices,
           prefix_lens, new_indptr) -> None:
    """Write this step's K/V behind each user's prefix (Alg. 1 step 8.2).

    ``k_new`` / ``v_new`` are ``[N][H][D]``, ragged over users by
    ``new_indptr``; user u's i-th new token gets position ``prefix_lens[u] + i``.
    The pages are already allocated (Sec. 3.2 step 1).
    """
    B = len(prefix_lens)
    for u in range(B):
        pages = page_indices[page_indptr[u]:page_indptr[u + 1]]
        lo, hi = int(new_indptr[u]), int(new_indptr[u + 1])
        _check_run(store, pages, int(prefix_lens[u]), hi - lo)
        for i in range(hi - lo):
            page, slot = store.slot(pages, int(prefix_lens[u]) + i)
            store.data[layer, page, 0, slot] = k_new[lo + i]
            store.data[layer, page, 1, slot] = v_new[lo + i]


# --------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------
def _softmax_rows(z: np.ndarray) -> np.ndarray:
    """Row-wise softmax; entries equal to -inf get weight zero."""
    top = z.max(axis=-1, keepdims=True)
    e = np.exp(z - top)
    return e / e.sum(axis=-1, keepdims=True)


def attn_incremental(store: PagedStore, layer: int, q, page_indptr, page_indices,
                     prefix_lens, new_indptr, sm_scale=None, users=None, heads=None) -> np.ndarray:
    """New-token queries over cached prefix plus new K/V (Sec. 2, Eq. 6-7).

    For user u, head h and new token i (absolute position p = P_u + i):
    ``o = sum_j softmax_j(s * q_i . K_j) V_j`` over j in [0, p], where rows
    0..P_u-1 are the cached prefix and rows P_u.. the tokens appended in this
    step; all rows are read from the pages (Alg. 1 runs step 8.2 before 8.4).

    ``q`` is ``[N][H][D]``.  Returns float64 ``[N][H][D]``; rows of users or heads
    not selected by ``users`` / ``heads`` (when given) are left as NaN.
    """
    D, H = store.D, store.H
    s = (1.0 / math.sqrt(D)) if sm_scale is None else float(sm_scale)
    qv = decode_values(q)
    out = np.full(qv.shape, np.nan, dtype=np.float64)
    B = len(prefix_lens)
    for u in (range(B) if users is None else users):
        P = int(prefix_lens[u])
        lo, hi = int(new_indptr[u]), int(new_indptr[u + 1])
        n = hi - lo
        if n == 0:
            continue
        T = P + n
        pages = np.asarray(page_indices[page_indptr[u]:page_indptr[u + 1]])
        _check_run(store, pages, 0, T)
        # logical view of the user's sequence: [T][H][D], token t from page t//S
        need = pages[: pages_for(T, store.S)]
        kv = store.data[layer, need]                      # [pages][2][S][H][D]
        K = decode_values(kv[:, 0].reshape(-1, H, D)[:T])
        V = decode_values(kv[:, 1].reshape(-1, H, D)[:T])
        pos = P + np.arange(n)[:, None]                   # query positions
        hidden = np.arange(T)[None, :] > pos              # key after the query
        for h in (range(H) if heads is None else heads):
            z = s * (qv[lo:hi, h] @ K[:, h].T)            # [n][T]
            z[hidden] = -np.inf
            w = _softmax_rows(z)
            out[lo:hi, h] = w @ V[:, h]
    return out


def full_recompute(q, k, v, sm_scale=None) -> np.ndarray:
    """Causal attention over a whole contiguous sequence, row by row.

    ``q, k, v`` are ``[T][H][D]``.  Token p sees tokens 0..p.  This is what the
    recompute baseline evaluates (Sec. 5.1) and what reuse must match on its
    last rows (Sec. 2).  Written without any paging and without the masked
    matrix form used above, so that the two can check each other.
    """
    qv, kv, vv = decode_values(q), decode_values(k), decode_values(v)
    T, H, D = qv.shape
    s = (1.0 / math.sqrt(D)) if sm_scale is None else float(sm_scale)
    out = np.zeros((T, H, D), dtype=np.float64)
    for h in range(H):
        for p in range(T):
            logits = np.array([s * float(np.dot(qv[p, h], kv[j, h])) for j in range(p + 1)])
            weights = np.exp(logits - logits.max())
            total = weights.sum()
            acc = np.zeros(D)
            for j in range(p + 1):
                acc += (weights[j] / total) * vv[j, h]
            out[p, h] = acc
    return out


def _silu(z: np.ndarray) -> np.ndarray:
    """x * sigmoid(x), written so that neither branch overflows."""
    e = np.exp(-np.abs(z))
    return np.where(z >= 0, z / (1.0 + e), z * e / (1.0 + e))


def attn_pointwise(store: PagedStore, layer: int, q, page_indptr, page_indices,
                   prefix_lens, new_indptr, inv_norm, sm_scale=None, users=None, heads=None) -> np.ndarray:
    """Pointwise-aggregated variant of :func:`attn_incremental` (Sec. 2, Eq. 3 with the
    HSTU-style aggregation; see the module docstring for the definition taken).

    For user u, head h and new token i at absolute position p = P_u + i:
    ``o = inv_norm * sum_{j in [0, p]} silu(s * q_i . K_j) V_j``; rows are read from
    the pages exactly as in the softmax form.  ``inv_norm`` is one scalar for the call.
    """
    D, H = store.D, store.H
    s = (1.0 / math.sqrt(D)) if sm_scale is None else float(sm_scale)
    qv = decode_values(q)
    out = np.full(qv.shape, np.nan, dtype=np.float64)
    B = len(prefix_lens)
    for u in (range(B) if users is None else users):
        P = int(prefix_lens[u])
        lo, hi = int(new_indptr[u]), int(new_indptr[u + 1])
        n = hi - lo
        if n == 0:
            continue
        T = P + n
        pages = np.asarray(page_indices[page_indptr[u]:page_indptr[u + 1]])
        _check_run(store, pages, 0, T)
        need = pages[: pages_for(T, store.S)]
        kv = store.data[layer, need]                      # [pages][2][S][H][D]
        K = decode_values(kv[:, 0].reshape(-1, H, D)[:T])
        V = decode_values(kv[:, 1].reshape(-1, H, D)[:T])
        pos = P + np.arange(n)[:, None]
        hidden = np.arange(T)[None, :] > pos              # key after the query
        for h in (range(H) if heads is None else heads):
            w = _silu(s * (qv[lo:hi, h] @ K[:, h].T))     # [n][T]
            w[hidden] = 0.0
            out[lo:hi, h] = float(inv_norm) * (w @ V[:, h])
    return out


def full_recompute_pointwise(q, k, v, inv_norm, sm_scale=None) -> np.ndarray:
    """The pointwise form over a whole contiguous sequence, term by term (no pages, no
    matrix form): token p aggregates tokens 0..p.  Reuse must match its last rows."""
    qv, kv, vv = decode_values(q), decode_values(k), decode_values(v)
    T, H, D = qv.shape
    s = (1.0 / math.sqrt(D)) if sm_scale is None else float(sm_scale)
    out = np.zeros((T, H, D), dtype=np.float64)
    for h in range(H):
        for p in range(T):
            acc = np.zeros(D)
            for j in range(p + 1):
                x = s * float(np.dot(qv[p, h], kv[j, h]))
                acc += (x / (1.0 + math.exp(-x)) if x > -700.0 else 0.0) * vv[j, h]
            out[p, h] = float(inv_norm) * acc
    return out
