/*
 * mtserve.h - C ABI of the MI355X (gfx950) hot path of cross-request KV reuse for
 * generative-recommendation serving: incremental-prefill attention over a paged GPU
 * KV cache, and the kernels that move KV between the contiguous host layout and the
 * paged GPU layout.
 *
 * The operations are the device half of the paper's seven-step workflow (Sec. 3.2):
 *   step 3  Cache Scattering  -> mts_kv_unpack
 *   step 4  Model Inference   -> mts_attn_incremental   (Sec. 2, Eq. 6-7; Alg. 1 step 8.4)
 *   step 5  Cache Update      -> mts_kv_append          (Alg. 1 step 8.2)
 *   step 6  Cache Offload     -> mts_kv_pack            (gather kernel of Sec. 4.2)
 * Page allocation, LRU and the host chunk store are the caller's business (the paper's
 * KVCacheManager, Sec. 3.1); this library consumes the page table it produces.
 *
 * General rules
 *   - Every function returns an int32 status (MTS_OK = 0, errors < 0) unless stated.
 *     Nothing throws, aborts, allocates, frees, or synchronises the host.
 *   - All device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) of the CURRENT device.  Pointers marked "device" must be valid on
 *     that device until the enqueued work has finished.  The caller owns every buffer.
 *   - Arguments are validated on the host before anything is launched; a call that returns
 *     an error has launched nothing.  mts_last_error() describes the last error of the
 *     calling thread.
 *   - The kernel entry points may be called from several host threads and may be captured into
 *     a HIP graph.  The first attention call of a process queries the device (occupancy, LDS
 *     limits): make one call outside stream capture before capturing.  One pattern is known to
 *     crash a capture on ROCm 7 (host side): making a stream wait, inside the capture, for an
 *     event that was recorded on that same stream.  mts_xfer_onload_wait_layer issues a
 *     hipStreamWaitEvent on the caller's stream for an event of the pipeline's own scatter stream,
 *     which is not part of the caller's capture: it must not be called under stream capture.
 *   - Device-resident metadata (page ids, lengths) cannot be validated on the host.  The
 *     kernels skip any access whose page id is outside [0, num_pages) or whose token lies
 *     beyond the user's page list, so bad metadata gives wrong results, not a fault.
 *
 * Paged pool layout (fixed by this header; the paper's [L, N_pages, 2, S_page, H, D] of
 * Sec. 4.1 is replaced by an arrangement whose 16-byte granules are MFMA operands):
 *   layer l        at pool + l * layer_stride_bytes
 *   page  p        at + p * page_bytes,            page_bytes = 2 * H * S * D * es
 *   head  h        at + h * (2 * S * D * es)       (K block, then V block, S*D*es bytes each)
 *   a page of S tokens is S/16 sub-blocks of 16 tokens; sub-block b at + b * 16 * D * es
 *   inside a 16-token K sub-block, with G = 16 / es elements per granule,
 *     element (token t, dim d) sits at element index
 *       ((half * (D/G) + d/G) * 8 + slot) * G + d % G
 *     where half = (t / 4) % 2 and slot = (t / 8) * 4 + t % 4;
 *   inside a 16-token V sub-block the block is transposed:
 *     element (token t, dim d) sits at element index  d * 16 + t.
 *   mts_elem_offset() evaluates this map on the host.
 *
 * Contiguous ("host") layout of a run of n tokens of one user and one layer:
 *   [2 (K plane, V plane)][n][H][D], i.e. what is kept in host chunks and what the onload
 *   and offload buffers hold (Sec. 4.1 CPU tier, Sec. 4.2).
 *
 * Supported: dtype f32 or bf16; head_dim in {32, 64, 128}; page_size in {16, 32, 64};
 * any num_heads >= 1.
 */
#ifndef MTSERVE_H
#define MTSERVE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  MTS_OK = 0,
  MTS_ERR_INVALID_ARG = -1, /* null pointer, negative count, layer out of range, bad alignment */
  MTS_ERR_UNSUPPORTED = -2, /* dtype / head_dim / page_size outside the supported set */
  MTS_ERR_SHAPE = -3,       /* sizes inconsistent with each other */
  MTS_ERR_WORKSPACE = -4,   /* workspace missing or too small */
  MTS_ERR_HIP = -5,         /* the HIP runtime refused a launch or a copy */
  MTS_ERR_BUSY = -6         /* admission control refused the task (offload quota / buffer space); nothing was enqueued */
};

enum { MTS_F32 = 0, MTS_BF16 = 1 };

/* The paged pool (Sec. 4.1 "Paged Store").  Plain data, read during the call only. */
typedef struct mts_cache_desc {
  void*   pool;               /* device, 256-byte aligned */
  int64_t layer_stride_bytes; /* >= num_pages * page_bytes, multiple of 256 */
  int32_t dtype;              /* MTS_F32 or MTS_BF16 */
  int32_t num_layers;
  int32_t num_pages;          /* pages per layer */
  int32_t page_size;          /* tokens per page, S */
  int32_t num_heads;          /* H (queries, keys and values share it) */
  int32_t head_dim;           /* D */
} mts_cache_desc;

/* Per-batch metadata in the paper's vocabulary (Alg. 1 step 8.2: position / offsets /
 * indices / indptr).  The int32 arrays are DEVICE arrays; the scalars are host copies the
 * launch shapes are derived from and must bound the device contents. */
typedef struct mts_batch_meta {
  int32_t        batch;         /* B, users in the batch */
  const int32_t* page_indptr;   /* device [B+1]: user u owns page_indices[page_indptr[u] .. page_indptr[u+1]) */
  const int32_t* page_indices;  /* device [total_pages]: physical page ids in logical order */
  const int32_t* prefix_lens;   /* device [B]: P_u, tokens valid in the cache before this step */
  const int32_t* new_indptr;    /* device [B+1]: ragged offsets of the step's tokens in q/k_new/v_new/out */
  int32_t        total_new;     /* = new_indptr[B] */
  int32_t        max_new;       /* >= max_u n_u */
  int32_t        max_total_len; /* >= max_u (P_u + n_u) */
  int32_t        total_pages;   /* = page_indptr[B] */
} mts_batch_meta;

/* Bytes of one page of one layer: 2 * H * S * D * es.  Returns < 0 on a bad descriptor. */
int64_t mts_page_bytes(const mts_cache_desc* cache);

/* ceil(len / page_size): pages ONE user needs (rounding is per user, App. C.1). */
int32_t mts_pages_for(int32_t len, int32_t page_size);

/* Byte offset inside a page of element (kv: 0 = K, 1 = V; head; token slot in [0, S);
 * dim in [0, D)) under the layout stated above.  Host-only; < 0 on bad arguments. */
int64_t mts_elem_offset(const mts_cache_desc* cache, int32_t kv, int32_t head,
                        int32_t slot, int32_t dim);

/*
 * Cache Scattering (Sec. 3.2 step 3; Sec. 4.2 scatter kernel).
 * For segment s in [0, num_segs): user u = seg_user[s]; the run of n_s =
 * seg_tok_indptr[s+1] - seg_tok_indptr[s] tokens that starts at element
 * seg_tok_indptr[s] * 2*H*D of `staging` (contiguous layout [2][n_s][H][D]) becomes the
 * user's tokens seg_pos[s] .. seg_pos[s]+n_s-1 in layer `layer`.  Exactly those slots are
 * written, byte for byte; nothing else in the pool changes.
 *   staging         device, 16-byte aligned; filled e.g. by hipMemcpyAsync from pinned host
 *   seg_user        device int32 [num_segs], values in [0, meta->batch)
 *   seg_pos         device int32 [num_segs], first destination token of the run
 *   seg_tok_indptr  device int64 [num_segs+1], non-decreasing token offsets
 *   max_seg_tokens  host, >= max_s n_s (launch shape)
 * Uses meta->page_indptr / page_indices only.  num_segs == 0 is a no-op.
 */
int32_t mts_kv_unpack(const mts_cache_desc* cache, int32_t layer, const void* staging,
                      int32_t num_segs, const int32_t* seg_user, const int32_t* seg_pos,
                      const int64_t* seg_tok_indptr, int32_t max_seg_tokens,
                      const mts_batch_meta* meta, void* stream);

/*
 * Cache Offload, gather half (Sec. 3.2 step 6; Sec. 4.2 gather kernel).  Exact inverse of
 * mts_kv_unpack: tokens seg_pos[s] .. +n_s-1 of user seg_user[s] are copied from the pages
 * into `staging_out` (device, 16-byte aligned) in the contiguous layout, ready for a
 * device-to-host copy.  The pool is not modified.
 */
int32_t mts_kv_pack(const mts_cache_desc* cache, int32_t layer, void* staging_out,
                    int32_t num_segs, const int32_t* seg_user, const int32_t* seg_pos,
                    const int64_t* seg_tok_indptr, int32_t max_seg_tokens,
                    const mts_batch_meta* meta, void* stream);

/*
 * The same two operations for `layer_count` consecutive layers, starting at `layer_begin`, in
 * ONE launch: the runs of layer layer_begin + i lie i * staging_layer_stride_bytes further in the
 * staging buffer (the stride a multiple of 16).  A restored or offloaded user costs a few
 * megabytes per layer, which a launch per layer moves in little more than its fixed cost; this
 * is the variant for callers that do not need one event per layer (the offload after the layer
 * loop, Alg. 1 step 9; a restore that is awaited as a whole).  layer_count == 0 is a no-op.
 */
int32_t mts_kv_unpack_layers(const mts_cache_desc* cache, int32_t layer_begin, int32_t layer_count,
                             const void* staging, int64_t staging_layer_stride_bytes, int32_t num_segs,
                             const int32_t* seg_user, const int32_t* seg_pos,
                             const int64_t* seg_tok_indptr, int32_t max_seg_tokens,
                             const mts_batch_meta* meta, void* stream);
int32_t mts_kv_pack_layers(const mts_cache_desc* cache, int32_t layer_begin, int32_t layer_count,
                           void* staging_out, int64_t staging_layer_stride_bytes, int32_t num_segs,
                           const int32_t* seg_user, const int32_t* seg_pos,
                           const int64_t* seg_tok_indptr, int32_t max_seg_tokens,
                           const mts_batch_meta* meta, void* stream);

/*
 * Cache Update (Sec. 3.2 step 5; Alg. 1 step 8.2).  k_new / v_new are device [total_new][H][D]
 * (16-byte aligned), ragged over users by meta->new_indptr; user u's i-th row is written at
 * token position prefix_lens[u] + i of layer `layer`.  The pages must already be in the
 * user's page list.  total_new == 0 is a no-op.
 */
int32_t mts_kv_append(const mts_cache_desc* cache, int32_t layer, const void* k_new,
                      const void* v_new, const mts_batch_meta* meta, void* stream);

/*
 * The same for `layer_count` consecutive layers in one launch: layer layer_begin + i takes its
 * rows from k_new / v_new + i * rows_layer_stride_bytes (a multiple of 16).  For callers that
 * keep every layer's rows until the end of the step - the attention calls that read them
 * directly (mts_attn_*_unappended below) need no append in between - and then write all of
 * them to the pool at once.  layer_count == 0 is a no-op.
 */
int32_t mts_kv_append_layers(const mts_cache_desc* cache, int32_t layer_begin, int32_t layer_count,
                             const void* k_new, const void* v_new, int64_t rows_layer_stride_bytes,
                             const mts_batch_meta* meta, void* stream);

/* Workspace mts_attn_incremental needs for this cache and batch shape (host-only, >= 0;
 * < 0 on bad arguments).  The workspace is device memory, 256-byte aligned, needs no
 * initialisation and may be reused by later calls on the same stream (never by calls that
 * overlap in time). */
int64_t mts_attn_workspace_bytes(const mts_cache_desc* cache, const mts_batch_meta* meta);

/*
 * Tuning and testing override of the attention launch plan.  Process-wide and read by every
 * attention call and by mts_attn_workspace_bytes: set it before the calls it is meant for, never
 * while another thread is inside one, and query the workspace size under the same setting as
 * the call.  A field of 0 keeps the automatic choice; NULL resets everything.  Results are the
 * same operation under every setting (the parity tests force schedules and kernels with it).
 */
enum { MTS_ATTN_KERNEL_AUTO = 0, MTS_ATTN_KERNEL_STREAMING = 1, MTS_ATTN_KERNEL_PREFILL = 2, MTS_ATTN_KERNEL_PLAIN = 3 };
typedef struct mts_attn_tuning {
  int32_t min_tiles; /* least kv tiles (32 tokens) of a wavefront's share in the streaming kernel */
  int32_t max_waves; /* most wavefronts of a streaming launch (multiple of 4, <= 1024) */
  int32_t pair_cost; /* schedule allowance per (query tile, head), in tiles */
  int32_t kernel;    /* MTS_ATTN_KERNEL_*: force the split-kv streaming kernel, the dense-prefill kernel
                        (where it applies) or the plain fp32-accumulate kernel */
} mts_attn_tuning;
int32_t mts_attn_set_tuning(const mts_attn_tuning* tuning);

/*
 * Incremental-prefill attention (Sec. 2, Eq. 6-7; Alg. 1 step 8.4).  For user u, head h and
 * new token i at absolute position p = prefix_lens[u] + i:
 *     out[i, h, :] = sum_j softmax_j(sm_scale * q[i, h, :] . K[j, h, :]) * V[j, h, :],  j in [0, p]
 * with K/V rows 0..p read from the user's pages of layer `layer`: the whole cached prefix is
 * visible and the new tokens are causal among themselves.  The step's own K/V must already
 * have been appended (mts_kv_append enqueued earlier on the same stream), as Alg. 1 orders it.
 * prefix_lens[u] == 0 gives plain causal prefill (the cache-miss / recompute shape).
 *   q, out     device [total_new][H][D], cache dtype, 16-byte aligned; out is overwritten
 *   sm_scale   logit scale; 0 selects 1/sqrt(D)
 * Logits, softmax statistics and accumulators are fp32.  For bf16 the softmax weights are
 * rounded to bf16 before the weighted sum of V (matrix-core operand) and the result is
 * rounded to bf16 (nearest even).
 */
int32_t mts_attn_incremental(const mts_cache_desc* cache, int32_t layer, const void* q,
                             void* out, const mts_batch_meta* meta, float sm_scale,
                             void* workspace, int64_t workspace_bytes, void* stream);

/*
 * mts_attn_incremental for callers that cannot allocate device memory or hand over a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operation, arguments, preconditions and results as mts_attn_incremental, but the split-kv
 * partials live in a buffer the library owns: a file-scope device array of
 * MTS_NOALLOC_SCRATCH_BYTES, one copy on every GPU the library is loaded on, held until the
 * process ends.  The call allocates and frees nothing.  Shapes whose workspace
 * (mts_attn_workspace_bytes) exceeds that size are refused with MTS_ERR_WORKSPACE before anything
 * is launched.  All calls on one GPU share the one buffer: calls that overlap in time on the same
 * GPU (different streams, different host threads) race and give wrong results; calls ordered on
 * one stream are safe.  The first call on a device looks the buffer's address up in the runtime:
 * make it outside stream capture.
 */
#define MTS_NOALLOC_SCRATCH_BYTES (40ll << 20)
int32_t mts_attn_incremental_noalloc(const mts_cache_desc* cache, int32_t layer, const void* q,
                                     void* out, const mts_batch_meta* meta, float sm_scale,
                                     void* stream);

/*
 * Pointwise-aggregated variant of mts_attn_incremental: the same queries, keys, visibility and
 * paged reads, with the aggregation of the HSTU-style backbone the paper serves (Sec. 2, Eq. 1-3;
 * the paper prints no formula for its Attention, so this header states the one computed):
 *     out[i, h, :] = inv_norm * sum_j silu(sm_scale * q[i, h, :] . K[j, h, :]) * V[j, h, :],  j in [0, p]
 * with silu(x) = x / (1 + exp(-x)).  No softmax statistics exist, so split-kv pieces simply add.
 *   sm_scale   logit scale; 0 selects 1/sqrt(D)
 *   inv_norm   normaliser, finite and > 0 (e.g. 1 / longest sequence of the batch)
 * Everything else (arguments, workspace from mts_attn_workspace_bytes, preconditions, errors,
 * precision: fp32 logits and accumulators, weights rounded to bf16 for the matrix cores) is as
 * for mts_attn_incremental.
 */
int32_t mts_attn_pointwise(const mts_cache_desc* cache, int32_t layer, const void* q, void* out,
                           const mts_batch_meta* meta, float sm_scale, float inv_norm,
                           void* workspace, int64_t workspace_bytes, void* stream);

/*
 * The same two attentions for a layer whose append has not happened: the context of user u is
 * the cached prefix in the pool (positions 0 .. prefix_lens[u]-1) followed by this step's rows
 * taken from k_new / v_new directly (Sec. 2: K = [K_pre ; k_delta], V = [V_pre ; v_delta]).  The
 * result equals mts_kv_append followed by mts_attn_incremental / mts_attn_pointwise, but the call
 * does not read the pool's slots of the new tokens, so mts_kv_append of the same layer may run
 * on another stream at the same time (or later): the copy leaves the layer's critical path.
 * The caller still appends before anything else reads those slots (the next step, a pack).
 *   k_new, v_new   device [total_new][H][D], cache dtype, 16-byte aligned, as for mts_kv_append
 * For long new segments (the shapes served by the dense-prefill kernel) and for fp32 caches
 * every key is read from the pool: there the call enqueues the append itself, on `stream`,
 * before the attention (a caller's own append then rewrites the same bytes;
 * mts_attn_unappended_appends tells which case a shape falls in).  Everything else is as for the
 * two calls above.
 */
/* 1 if the two calls below append by themselves for this shape (the caller then skips its own
 * mts_kv_append), 0 if they leave the pool alone, < 0 on a bad descriptor.  Host only. */
int32_t mts_attn_unappended_appends(const mts_cache_desc* cache, const mts_batch_meta* meta);
int32_t mts_attn_incremental_unappended(const mts_cache_desc* cache, int32_t layer, const void* q,
                                        const void* k_new, const void* v_new, void* out,
                                        const mts_batch_meta* meta, float sm_scale, void* workspace,
                                        int64_t workspace_bytes, void* stream);
int32_t mts_attn_pointwise_unappended(const mts_cache_desc* cache, int32_t layer, const void* q,
                                      const void* k_new, const void* v_new, void* out,
                                      const mts_batch_meta* meta, float sm_scale, float inv_norm,
                                      void* workspace, int64_t workspace_bytes, void* stream);

/*
 * mts_attn_incremental_unappended for a batch in which some users' cached prefix has not been
 * scattered yet and still lies in the contiguous onload buffer (Sec. 4.1: the buffer doubles as
 * an inference area, so that a restored user's attention need not wait for the scatter kernel).
 *   staged_rows       device, the layer's runs one after another, each [2][n][H][D] as for
 *                     mts_kv_unpack, 16-byte aligned
 *   staged_first_run  device [batch]: index of the first run of user u's prefix, or -1 if the
 *                     prefix is in the pool; a staged user's prefix is covered by consecutive runs
 *                     of exactly chunk_tokens tokens each, the last one holding the rest
 *   staged_run_tok    device [runs + 1]: token offset of every run in staged_rows (run s starts
 *                     at element staged_run_tok[s] * 2 * H * D), as seg_tok_indptr of mts_kv_unpack
 *   chunk_tokens      tokens per run, a positive multiple of 32
 * The pool's pages of a staged user are neither read nor written (they must still be allotted
 * in the page table: mts_kv_unpack and the append fill them afterwards).  Served by the
 * streaming bf16 kernel only; MTS_ERR_UNSUPPORTED for fp32 caches and for the long new segments
 * the dense-prefill kernel serves (there, unpack first).  Rows of the onload buffer are loaded
 * 16 bytes per lane like pool tiles, V being transposed through LDS on the way, but only two
 * such tiles are in flight per wavefront: per token they stream about a third more slowly than
 * pool tiles, which is fine for the few restored users of a batch.
 */
int32_t mts_attn_incremental_staged(const mts_cache_desc* cache, int32_t layer, const void* q,
                                    const void* k_new, const void* v_new, const void* staged_rows,
                                    const int32_t* staged_first_run, const int64_t* staged_run_tok,
                                    int32_t chunk_tokens, void* out, const mts_batch_meta* meta,
                                    float sm_scale, void* workspace, int64_t workspace_bytes,
                                    void* stream);

/* Host<->device staging copies on `stream` (hipMemcpyAsync); `host` should be pinned for the
 * copy to be asynchronous (Sec. 4.2, DMA between pinned buffers and the onload / offload buffers). */
int32_t mts_stage_h2d_async(void* device_dst, const void* host_src, int64_t bytes, void* stream);
int32_t mts_stage_d2h_async(void* host_dst, const void* device_src, int64_t bytes, void* stream);

/*
 * ---- Transfer pipeline -------------------------------------------------------------------
 * The two background paths either side of the kernels (Sec. 4.2 "Pipelined Onload via Double
 * Buffering", "Transient Offload Pipeline", "Offload Capacity Control"; Sec. 4.4 four-stream
 * model and layer-wise synchronisation; Alg. 1 steps 2, 7, 8.3, 9).  An mts_xfer owns, on the
 * device that is current at creation: an onload stream, a scatter stream and an offload stream
 * (default priority, non-blocking), two pinned host buffers per direction, a device arena for
 * transient offload buffers, one host worker per direction and a pool of copy threads.  These
 * are the only functions of the library that allocate, create threads or block the host.
 *
 * Onload of a step: for every layer, each run is copied from the caller's host chunk into a
 * pinned buffer (host threads) while the other pinned buffer is in flight to the device
 * (onload stream); when a layer's runs have landed in `staging`, mts_kv_unpack of that layer
 * is enqueued on the scatter stream and an event is recorded.  mts_xfer_onload_wait_layer
 * makes a compute stream wait for exactly that event, so layer l's attention starts as soon
 * as layer l is scattered, while deeper layers are still on the bus.
 *
 * Offload of a step: after the work already enqueued on `after_stream` (the step's appends),
 * every layer's runs are gathered by one mts_kv_pack_layers launch into a transient buffer
 * from the arena (offload stream), copied to the pinned buffers in turn, and copied from there into the
 * caller's host chunks by the copy threads while the next buffer is in flight.  A task is
 * refused with MTS_ERR_BUSY, before anything is enqueued, if the tokens pending in transient
 * buffers would exceed the quota or the arena has no room.
 */
typedef struct mts_xfer mts_xfer;

typedef struct mts_xfer_config {
  int64_t pinned_bytes;         /* bytes of each pinned buffer: >= the largest run (one host chunk); a
                                   multiple of it lets several consecutive runs share one DMA */
  int64_t offload_arena_bytes;  /* device bytes for transient offload buffers (0: no offload path) */
  int64_t offload_quota_tokens; /* most run tokens that may be pending in transient buffers */
  int32_t num_layers;           /* layers a task covers (= cache->num_layers of every call) */
  int32_t copy_threads;         /* host threads per bulk copy and direction, >= 1; they poll between the
                                   copies of a task, so keep 2 * copy_threads below the core count */
} mts_xfer_config;

/* The runs of one task; the first five fields are exactly the arguments of mts_kv_unpack /
 * mts_kv_pack and stay valid until the task has finished. */
typedef struct mts_xfer_runs {
  int32_t        num_segs;
  const int32_t* seg_user;        /* device [num_segs] */
  const int32_t* seg_pos;         /* device [num_segs] */
  const int64_t* seg_tok_indptr;  /* device [num_segs+1] */
  int32_t        max_seg_tokens;
  const int64_t* host_tok_indptr; /* host copy of seg_tok_indptr; read during submit only */
  void* const*   host_runs;       /* host [num_layers * num_segs]: run s of layer l, contiguous layout
                                     [2][n_s][H][D], ordinary (pageable) memory; read (onload) or
                                     written (offload) until the task has finished; the array itself
                                     is read during submit only */
} mts_xfer_runs;

int32_t mts_xfer_create(const mts_xfer_config* config, mts_xfer** out);
/* Waits for all submitted work, then frees everything.  NULL is a no-op. */
int32_t mts_xfer_destroy(mts_xfer* x);

/* Starts the onload of one step and returns at once.  `staging` is the device onload buffer:
 * layer l's runs are laid out at staging + l * staging_layer_stride_bytes exactly as
 * mts_kv_unpack expects them.  One onload task at a time: a second submit waits for the first
 * to be fully enqueued.  cache and meta are copied; the arrays they point to must stay valid. */
int32_t mts_xfer_onload_submit(mts_xfer* x, const mts_cache_desc* cache, const mts_batch_meta* meta,
                               const mts_xfer_runs* runs, void* staging,
                               int64_t staging_layer_stride_bytes);
/* Blocks the calling host thread until layer `layer` of the current onload task has been
 * enqueued (bounded wait), then makes `compute_stream` wait for its scatter (Alg. 1 step 8.3). */
int32_t mts_xfer_onload_wait_layer(mts_xfer* x, int32_t layer, void* compute_stream);

/* Queues the offload of one step and returns at once, or refuses it (MTS_ERR_BUSY). */
int32_t mts_xfer_offload_submit(mts_xfer* x, const mts_cache_desc* cache, const mts_batch_meta* meta,
                                const mts_xfer_runs* runs, void* after_stream);
/* Run tokens currently pending in transient buffers (the quantity the quota bounds). */
int64_t mts_xfer_offload_pending_tokens(mts_xfer* x);
/* Blocks until every submitted task of both directions has finished (host data in place,
 * device work complete).  Returns the first error a background task met, if any. */
int32_t mts_xfer_drain(mts_xfer* x);

/*
 * ---- Cache manager (host only) -------------------------------------------------------------
 * The KVCacheManager of Sec. 3.1 / Sec. 4.3: per-user sequence lengths, the page table of the
 * GPU tier, page allocation from a free pool, LRU replacement with O(1) updates, eviction as a
 * pure metadata operation (the host tier is the backup; nothing is copied), and the registry
 * of locked users that victim selection skips.  It makes no device call: its output is the
 * host copy of the arrays mts_batch_meta points to.  Not thread-safe: one caller at a time.
 *
 * Per user the manager tracks total_len (tokens of history cached on either tier), host_len
 * (the prefix of those persisted in the host tier) and whether the GPU tier holds the user.
 * Evicting a user frees its pages and cuts total_len back to host_len: tokens the offload
 * path had not persisted yet are simply no longer cached (counted in tokens_dropped).
 */
typedef struct mts_cm mts_cm;

typedef struct mts_cm_stats {
  int64_t gpu_hits;       /* requests whose history was in the GPU tier */
  int64_t host_hits;      /* requests whose history had to come up from the host tier */
  int64_t cold_requests;  /* requests with no cached history at all */
  int64_t evictions;      /* users evicted from the GPU tier */
  int64_t tokens_dropped; /* tokens lost at eviction because they were not persisted yet */
  int64_t free_pages;
  int64_t users_tracked;
  int64_t users_on_gpu;
} mts_cm_stats;

int32_t mts_cm_create(int32_t num_pages, int32_t page_size, int32_t host_chunk_tokens, mts_cm** out);
int32_t mts_cm_destroy(mts_cm* m);

/* Tokens of history cached for `user` on either tier; 0 for an unknown user (Alg. 1 step 1). */
int32_t mts_cm_cached_length(mts_cm* m, int64_t user);

/* Registers a user whose history of total_len tokens lies, whole, in the host tier (e.g. at
 * start-up, from a persisted store).  The user must not be tracked yet. */
int32_t mts_cm_import_history(mts_cm* m, int64_t user, int32_t total_len);

/*
 * Page allocation and LRU for one batch (Alg. 1 steps 2 and 6).  For request i (users[i]
 * distinct, new_tokens[i] >= 0) the user is given ceil((total_len + new_tokens[i]) / page_size)
 * pages: missing ones come from the free pool, and when that runs dry whole users are evicted
 * from the least-recently-used end, skipping locked users and the users of this batch.
 * Outputs (host arrays): prefix_lens[i] = total_len; onload_lens[i] = tokens that must be
 * brought up from the host tier first (0 if the GPU tier holds the user; total_len otherwise);
 * page_indptr[batch+1] / page_indices = the users' page lists in CSR form, logical order.
 * MTS_ERR_BUSY: even after evicting every eligible victim the batch does not fit; MTS_ERR_SHAPE:
 * page_capacity (entries of page_indices) is too small.  On any error nothing has changed
 * (users first seen in a failed call are not tracked).
 */
int32_t mts_cm_prepare_batch(mts_cm* m, const int64_t* users, const int32_t* new_tokens, int32_t batch,
                             int32_t* prefix_lens, int32_t* onload_lens, int32_t* page_indptr,
                             int32_t* page_indices, int64_t page_capacity);
/* The prepared batch has run (Alg. 1 step 7): total_len += new_tokens, the users are on the
 * GPU tier and become the most recently used, in batch order. */
int32_t mts_cm_commit_batch(mts_cm* m);
/* The prepared batch will not run (the step failed before its commit): every user of it goes
 * back to the pages its cached tokens need (none for a user that is not on the GPU tier), the
 * pages prepare had added return to the free pool and the batch's requests are taken out of the
 * hit / cold counters.  Users that prepare evicted to make room stay evicted.  With no prepared
 * batch the call does nothing. */
int32_t mts_cm_abort_batch(mts_cm* m);

/* Offload trigger (Sec. 4.2): users on the GPU tier whose not-yet-persisted tokens amount to
 * at least one host chunk.  Returns how many were written (<= capacity), most recent first:
 * tokens [from_pos[k], from_pos[k] + count[k]) of users[k], count a multiple of the chunk.
 * Each returned user is locked until mts_cm_offload_done. */
int32_t mts_cm_offload_due(mts_cm* m, int64_t* users, int32_t* from_pos, int32_t* count, int32_t capacity);
/* The host tier now holds tokens [0, persisted_len) of `user`; unlocks the user. */
int32_t mts_cm_offload_done(mts_cm* m, int64_t user, int32_t persisted_len);
/* Puts `user` into (locked != 0) or takes it out of the locked registry by hand. */
int32_t mts_cm_set_locked(mts_cm* m, int64_t user, int32_t locked);

/* Users evicted since the last call, in eviction order; returns how many were written. */
int64_t mts_cm_take_evicted(mts_cm* m, int64_t* users, int64_t capacity);
int32_t mts_cm_get_stats(mts_cm* m, mts_cm_stats* out);

/*
 * Measurement yardstick (not part of the method): reads `bytes` bytes of device memory at `src`
 * once, 16 bytes per lane, and folds them into `sink` (device, 4096 bytes, any contents).  Timed
 * by the caller, it gives the rate a kernel that only streams reaches on this machine, which is
 * what the attention kernels' HBM fractions are to be read against.  src and bytes multiples of 16.
 */
int32_t mts_diag_stream_read(const void* src, int64_t bytes, void* sink, void* stream);

/* Text of the calling thread's last error ("" if none).  Never NULL. */
const char* mts_last_error(void);

/* Library version as major * 10000 + minor * 100 + patch. */
int32_t mts_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MTSERVE_H */
