"""Device-side holders for the arguments of the C ABI: the paged pool, the per-batch
metadata and segment lists.  They allocate and upload; they compute nothing of the method.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _dev_i32(a, device):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)


class PagedKVCache:
    """The GPU tier's paged pool (Sec. 4.1) as one device allocation, plus its descriptor."""

    def __init__(self, layers, num_pages, page_size, heads, head_dim, dtype, device="cuda:0",
                 fill_byte=None):
        self.dtype = dtype
        es = 4 if dtype == "f32" else 2
        self.desc = B.CacheDesc(None, 0, B.MTS_F32 if dtype == "f32" else B.MTS_BF16, layers,
                                num_pages, page_size, heads, head_dim)
        self.page_bytes = B.mts_page_bytes(self.desc)
        assert self.page_bytes == 2 * heads * page_size * head_dim * es
        stride = (num_pages * self.page_bytes + 255) // 256 * 256
        self.pool = torch.empty(layers * stride, dtype=torch.uint8, device=device)
        if fill_byte is not None:
            self.pool.fill_(fill_byte)
        self.desc.pool = self.pool.data_ptr()
        self.desc.layer_stride_bytes = stride
        self.layer_stride = stride
        self.device = device

    def layer_bytes(self, layer):
        """uint8 view of one layer's pages: [num_pages][page_bytes]."""
        v = self.pool[layer * self.layer_stride: layer * self.layer_stride + self.desc.num_pages * self.page_bytes]
        return v.view(self.desc.num_pages, self.page_bytes)


class DeviceBatch:
    """Per-batch metadata (page table in CSR form, prefix lengths, ragged new-token offsets)
    uploaded to the device, with the host-side bounds the launch shapes need."""

    def __init__(self, page_indptr, page_indices, prefix_lens, new_indptr, device="cuda:0"):
        page_indptr = np.asarray(page_indptr, dtype=np.int32)
        new_indptr = np.asarray(new_indptr, dtype=np.int32)
        prefix_lens = np.asarray(prefix_lens, dtype=np.int32)
        batch = len(prefix_lens)
        new_lens = np.diff(new_indptr) if batch else np.zeros(0, np.int32)
        self.page_indptr = _dev_i32(page_indptr, device)
        self.page_indices = _dev_i32(page_indices if len(page_indices) else np.zeros(1, np.int32), device)
        self.prefix_lens = _dev_i32(prefix_lens if batch else np.zeros(1, np.int32), device)
        self.new_indptr = _dev_i32(new_indptr, device)
        self.meta = B.BatchMeta(
            batch, self.page_indptr.data_ptr(), self.page_indices.data_ptr(),
            self.prefix_lens.data_ptr(), self.new_indptr.data_ptr(),
            int(new_indptr[-1]) if batch else 0,
            int(new_lens.max()) if batch else 0,
            int((prefix_lens + new_lens).max()) if batch else 0,
            int(page_indptr[-1]) if batch else 0)

    @classmethod
    def from_workload(cls, w, device="cuda:0"):
        return cls(w.page_indptr, w.page_indices, w.prefix_lens, w.new_indptr, device)

    @classmethod
    def from_workload_users(cls, w, users, device="cuda:0"):
        """The batch made of a subset of the workload's users, in the order given: their page lists,
        prefix lengths and a ragged offset array over their own rows.  Returns (batch, rows)."""
        users = [int(u) for u in users]
        pages = [w.user_pages(u) for u in users]
        indptr = np.concatenate([[0], np.cumsum([len(p) for p in pages])]).astype(np.int32)
        indices = np.concatenate(pages).astype(np.int32) if pages else np.zeros(0, np.int32)
        new = np.asarray([w.new_lens[u] for u in users], dtype=np.int32)
        new_indptr = np.concatenate([[0], np.cumsum(new)]).astype(np.int32)
        prefix = np.asarray([w.prefix_lens[u] for u in users], dtype=np.int32)
        return cls(indptr, indices, prefix, new_indptr, device), int(new_indptr[-1])


class SegmentList:
    """Runs of tokens in a contiguous staging buffer: (user, first pool token, token count)."""

    def __init__(self, users, positions, counts, device="cuda:0"):
        counts = np.asarray(counts, dtype=np.int64)
        indptr = np.zeros(len(counts) + 1, dtype=np.int64)
        indptr[1:] = np.cumsum(counts)
        self.num_segs = len(counts)
        self.total_tokens = int(indptr[-1])
        self.max_seg_tokens = int(counts.max()) if len(counts) else 0
        self.host_indptr = indptr
        self.seg_user = _dev_i32(users if self.num_segs else np.zeros(1, np.int32), device)
        self.seg_pos = _dev_i32(positions if self.num_segs else np.zeros(1, np.int32), device)
        self.seg_tok_indptr = torch.from_numpy(indptr).to(device)

    @classmethod
    def for_histories(cls, users, lengths, chunk_tokens, device="cuda:0"):
        """Each user's tokens [0, length) cut into host-chunk sized runs (Sec. 4.1 CPU tier)."""
        su, sp, sc = [], [], []
        for u, n in zip(users, lengths):
            for start in range(0, int(n), int(chunk_tokens)):
                su.append(int(u)); sp.append(start); sc.append(min(int(chunk_tokens), int(n) - start))
        return cls(su, sp, sc, device)

    def args(self):
        return (self.num_segs, self.seg_user, self.seg_pos, self.seg_tok_indptr, self.max_seg_tokens)


class HostRuns:
    """The host side of a transfer task: for every (layer, run) a contiguous numpy array in the
    [2][n][H][D] layout (ordinary pageable memory, standing in for host chunks), and the
    mts_xfer_runs structure that points at them.  Keeps everything it points to alive."""

    def __init__(self, segs: SegmentList, arrays):
        """arrays[layer][run] : C-contiguous numpy arrays."""
        import ctypes as C
        self.segs = segs
        self.arrays = arrays
        layers = len(arrays)
        ptrs = (C.c_void_p * max(1, layers * segs.num_segs))()
        for l in range(layers):
            assert len(arrays[l]) == segs.num_segs
            for s, a in enumerate(arrays[l]):
                assert a.flags["C_CONTIGUOUS"]
                ptrs[l * segs.num_segs + s] = a.ctypes.data
        self._ptrs = ptrs
        self._indptr = np.ascontiguousarray(segs.host_indptr, dtype=np.int64)
        self.runs = B.XferRuns(segs.num_segs, segs.seg_user.data_ptr(), segs.seg_pos.data_ptr(),
                               segs.seg_tok_indptr.data_ptr(), segs.max_seg_tokens,
                               self._indptr.ctypes.data, C.addressof(ptrs))

