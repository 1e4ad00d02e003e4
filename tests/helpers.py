"""Shared test plumbing: seeded element data for a workload and an oracle store
filled the way the serving path fills the GPU tier (history scattered chunk by
chunk, then the step's K/V appended)."""
import numpy as np

import mts_workloads as W
import oracle


def draw_step_data(w, layers=None, seed_offset=0):
    """Per-layer element data for one step of workload ``w``.

    Returns dict with, for each selected layer l: ``hist[l][u]`` = the user's
    cached history in host layout [2][P_u][H][D]; ``k_new[l]``, ``v_new[l]``,
    ``q[l]`` = [N][H][D].  Stored as float32 values or bf16 bit patterns.
    """
    layers = list(range(w.layers)) if layers is None else list(layers)
    rng = np.random.default_rng([w.seed, 11, seed_offset])
    H, D = w.heads, w.head_dim
    data = {"layers": layers, "hist": {}, "k_new": {}, "v_new": {}, "q": {}}
    for l in layers:
        data["hist"][l] = [W.normal_elements(rng, (2, int(P), H, D), w.dtype) for P in w.prefix_lens]
        data["k_new"][l] = W.normal_elements(rng, (w.total_new, H, D), w.dtype)
        data["v_new"][l] = W.normal_elements(rng, (w.total_new, H, D), w.dtype)
        data["q"][l] = W.normal_elements(rng, (w.total_new, H, D), w.dtype)
    return data


def oracle_store_for(w, data, fill=None, do_append=True):
    """Oracle Paged Store holding the histories (unpacked in host-chunk sized
    runs) and, if asked, this step's appended K/V, for the layers in ``data``."""
    store = oracle.PagedStore(w.layers, w.num_pages, w.page_size, w.heads, w.head_dim, w.np_dtype, fill=fill)
    for l in data["layers"]:
        for u in range(w.batch):
            pages = w.user_pages(u)
            for start, cnt in W.host_chunks(int(w.prefix_lens[u]), w.chunk_tokens):
                oracle.unpack(store, l, data["hist"][l][u][:, start:start + cnt], pages, start)
        if do_append:
            oracle.append(store, l, data["k_new"][l], data["v_new"][l], w.page_indptr,
                          w.page_indices, w.prefix_lens, w.new_indptr)
    return store


def as_values(raw):
    """Stored elements (float32 or bf16 bits) -> float64, for comparisons in tests."""
    raw = np.asarray(raw)
    if raw.dtype == np.uint16:
        return W.bf16_bits_to_f32(raw).astype(np.float64)
    return raw.astype(np.float64)
