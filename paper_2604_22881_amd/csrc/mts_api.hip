// C ABI of the library: argument validation on the host, then the launchers.
// Every entry point returns before launching anything if an argument is bad.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "../../include/mtserve.h"
#include "mts_internal.hpp"

namespace {

thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int elem_bytes(int32_t dtype) { return dtype == MTS_F32 ? 4 : (dtype == MTS_BF16 ? 2 : 0); }

// Validates the descriptor (and the layer, unless layer < -1 is passed as "not needed").
int32_t check_cache(const mts_cache_desc* c, int32_t layer, bool need_pool, mts::PoolGeom* g) {
  if (!c) return fail(MTS_ERR_INVALID_ARG, "cache descriptor is NULL");
  const int es = elem_bytes(c->dtype);
  if (!es) return fail(MTS_ERR_UNSUPPORTED, "dtype %d is neither MTS_F32 nor MTS_BF16", c->dtype);
  if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128)
    return fail(MTS_ERR_UNSUPPORTED, "head_dim %d not in {32, 64, 128}", c->head_dim);
  if (c->page_size != 16 && c->page_size != 32 && c->page_size != 64)
    return fail(MTS_ERR_UNSUPPORTED, "page_size %d not in {16, 32, 64}", c->page_size);
  if (c->num_heads < 1 || c->num_heads > 65535)
    return fail(MTS_ERR_INVALID_ARG, "num_heads %d out of range [1, 65535]", c->num_heads);
  if (c->num_layers < 1 || c->num_pages < 1)
    return fail(MTS_ERR_INVALID_ARG, "num_layers %d and num_pages %d must be >= 1", c->num_layers, c->num_pages);
  const int64_t page_bytes = 2ll * c->num_heads * c->page_size * c->head_dim * es;
  if (need_pool) {
    if (!c->pool) return fail(MTS_ERR_INVALID_ARG, "pool is NULL");
    if (!aligned(c->pool, 256)) return fail(MTS_ERR_INVALID_ARG, "pool is not 256-byte aligned");
    if (c->layer_stride_bytes < page_bytes * c->num_pages)
      return fail(MTS_ERR_SHAPE, "layer_stride_bytes %lld < num_pages * page_bytes %lld",
                  (long long)c->layer_stride_bytes, (long long)(page_bytes * c->num_pages));
    if (c->layer_stride_bytes % 256)
      return fail(MTS_ERR_INVALID_ARG, "layer_stride_bytes is not a multiple of 256");
    if (layer < 0 || layer >= c->num_layers)
      return fail(MTS_ERR_INVALID_ARG, "layer %d out of range [0, %d)", layer, c->num_layers);
  }
  if (g) {
    g->layer_base = need_pool ? static_cast<char*>(c->pool) + (int64_t)layer * c->layer_stride_bytes : nullptr;
    g->page_bytes = page_bytes;
    g->num_pages = c->num_pages;
    g->S = c->page_size;
    g->H = c->num_heads;
    g->D = c->head_dim;
    g->es = es;
    g->sub_shift = c->page_size == 16 ? 0 : (c->page_size == 32 ? 1 : 2);
  }
  return MTS_OK;
}

int32_t check_meta(const mts_batch_meta* m, bool need_new, bool need_ptrs, mts::BatchDev* b) {
  if (!m) return fail(MTS_ERR_INVALID_ARG, "batch metadata is NULL");
  if (m->batch < 0 || m->batch > 65535) return fail(MTS_ERR_INVALID_ARG, "batch %d out of range [0, 65535]", m->batch);
  if (m->total_pages < 0 || m->total_new < 0 || m->max_new < 0 || m->max_total_len < 0)
    return fail(MTS_ERR_INVALID_ARG, "negative count in batch metadata");
  if (need_ptrs && m->batch > 0) {
    if (!m->page_indptr || !m->page_indices)
      return fail(MTS_ERR_INVALID_ARG, "page_indptr / page_indices is NULL");
    if (need_new && (!m->prefix_lens || !m->new_indptr))
      return fail(MTS_ERR_INVALID_ARG, "prefix_lens / new_indptr is NULL");
  }
  if (need_new) {
    if ((int64_t)m->total_new > (int64_t)m->batch * m->max_new)
      return fail(MTS_ERR_SHAPE, "total_new %d exceeds batch %d * max_new %d", m->total_new, m->batch, m->max_new);
    if (m->max_new > m->max_total_len)
      return fail(MTS_ERR_SHAPE, "max_new %d exceeds max_total_len %d", m->max_new, m->max_total_len);
  }
  if (b) {
    b->batch = m->batch;
    b->page_indptr = m->page_indptr;
    b->page_indices = m->page_indices;
    b->prefix_lens = m->prefix_lens;
    b->new_indptr = m->new_indptr;
    b->total_new = m->total_new;
    b->max_new = m->max_new;
    b->max_total_len = m->max_total_len;
    b->total_pages = m->total_pages;
  }
  return MTS_OK;
}

int32_t check_segs(int32_t num_segs, const int32_t* seg_user, const int32_t* seg_pos,
                   const int64_t* seg_tok_indptr, int32_t max_seg_tokens, mts::SegDev* s) {
  if (num_segs < 0 || num_segs > 65535)
    return fail(MTS_ERR_INVALID_ARG, "num_segs %d out of range [0, 65535]", num_segs);
  if (max_seg_tokens < 0) return fail(MTS_ERR_INVALID_ARG, "max_seg_tokens is negative");
  if (num_segs > 0 && (!seg_user || !seg_pos || !seg_tok_indptr))
    return fail(MTS_ERR_INVALID_ARG, "segment array is NULL");
  s->num_segs = num_segs;
  s->seg_user = seg_user;
  s->seg_pos = seg_pos;
  s->seg_tok_indptr = seg_tok_indptr;
  s->max_seg_tokens = max_seg_tokens;
  return MTS_OK;
}

int32_t hip_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return MTS_OK;
  return fail(MTS_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

int64_t roundup(int64_t v, int m) { return (v + m - 1) / m * m; }

// ---- library-owned scratch of mts_attn_incremental_noalloc -----------------------------------
// One copy per GPU the library is loaded on, held until the process ends.  In host code the
// array's name is only a stand-in for the symbol: the memory's address on the current device is
// asked from the runtime once per device and kept.
constexpr int64_t kScratchBytes = MTS_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device; nullptr + error text on failure
void* scratch_on_current_device() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(MTS_ERR_HIP, "hipGetDevice: %s (device %d)", hipGetErrorString(e), dev);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      fail(MTS_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

namespace mts {

int32_t set_error(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// mts_attn_set_tuning: 0 = automatic
std::atomic<int> g_tune_min_tiles{0}, g_tune_max_waves{0}, g_tune_pair_cost{0}, g_tune_kernel{0};

AttnPlan plan_attention(const PoolGeom& g, const BatchDev& b) {
  AttnPlan p{};
  const int force = g_tune_kernel.load(std::memory_order_relaxed);
  p.use_mfma = (g.es == 2) && force != MTS_ATTN_KERNEL_PLAIN;
  p.q_tile = 16; p.q_tiles_max = 1; p.n_items = 0; p.min_tiles = 4; p.max_waves = 4;
  if (!p.use_mfma || b.total_new <= 0 || b.batch <= 0) return p;
  const int max_new = b.max_new > 0 ? b.max_new : 1;
  // Long new segments (a cache miss, Sec. 5.1's full prefill) are a dense contraction: the
  // workgroup-per-query-block kernel shares K/V tiles through LDS and needs no workspace.
  // Short ones with long prefixes need the split-kv schedule of the streaming kernel.
  bool prefill = max_new >= 256 && (int64_t)b.total_new >= 128ll * b.batch;
  if (force == MTS_ATTN_KERNEL_PREFILL) prefill = true;
  if (force == MTS_ATTN_KERNEL_STREAMING) prefill = false;
  if (prefill && attn_prefill_applicable(g, b)) { p.use_prefill = true; return p; }
  p.q_tile = roundup(max_new, 16) < 64 ? roundup(max_new, 16) : 64;
  p.q_tiles_max = (max_new + p.q_tile - 1) / p.q_tile;
  const int64_t items = (int64_t)b.batch * p.q_tiles_max;
  // Every (query tile, head) also counts an allowance for what it costs besides streaming its
  // tiles; measured optimum 6-12 tiles on three workloads (a flat one), worth 7 % of the launch
  // where a share holds several short pairs and 1-2 % where pairs are longer than shares.
  p.pair_cost = 8;
  if (const int v = g_tune_pair_cost.load(std::memory_order_relaxed); v > 0) p.pair_cost = v < 64 ? v : 64;
  const int64_t tiles_upper = items * ((b.max_total_len + 31) / 32 + 1 + p.pair_cost) * g.H;   // schedule units of the call
  if (items > 16384 || b.batch > 4096 || tiles_upper >= (1ll << 31)) { p.too_large = true; return p; }
  p.n_items = (int)items;
  // a wavefront's share is never shorter than this: below it, start-up and the partial
  // accumulators cost more than the share itself
  if (const int v = g_tune_min_tiles.load(std::memory_order_relaxed); v >= 1) p.min_tiles = v;
  int64_t waves = (tiles_upper + p.min_tiles - 1) / p.min_tiles;
  waves = (waves + 3) / 4 * 4;
  // 256 CUs x 4 SIMDs: one wavefront per SIMD.  A second one (the kernel is compiled to fit two)
  // measured 2-5 % slower on every shape tried, small or large: it doubles the cuts, and the
  // wavefront that starts second on a SIMD streams more slowly than the first.
  int64_t cap = kAttnMaxWaves;
  if (const int v = g_tune_max_waves.load(std::memory_order_relaxed); v >= 4 && v < cap) cap = v / 4 * 4;
  p.max_waves = (int)(waves < cap ? waves : cap);
  if (p.max_waves < 4) p.max_waves = 4;
  p.ws_desc_bytes = roundup((int64_t)p.max_waves * 32, 256);
  p.ws_bytes = p.ws_desc_bytes + (int64_t)p.max_waves * 2 * p.q_tile * (g.D + 2) * (int64_t)sizeof(float);
  return p;
}

}  // namespace mts

extern "C" {

const char* mts_last_error(void) { return g_err; }

int32_t mts_version(void) { return 100; }

int64_t mts_page_bytes(const mts_cache_desc* cache) {
  mts::PoolGeom g{};
  const int32_t st = check_cache(cache, 0, false, &g);
  return st != MTS_OK ? st : g.page_bytes;
}

int32_t mts_pages_for(int32_t len, int32_t page_size) {
  if (len < 0 || page_size <= 0) return fail(MTS_ERR_INVALID_ARG, "len >= 0 and page_size > 0 required");
  return (int32_t)(((int64_t)len + page_size - 1) / page_size);
}

int64_t mts_elem_offset(const mts_cache_desc* cache, int32_t kv, int32_t head, int32_t slot, int32_t dim) {
  mts::PoolGeom g{};
  const int32_t st = check_cache(cache, 0, false, &g);
  if (st != MTS_OK) return st;
  if (kv < 0 || kv > 1 || head < 0 || head >= g.H || slot < 0 || slot >= g.S || dim < 0 || dim >= g.D)
    return fail(MTS_ERR_INVALID_ARG, "element (kv %d, head %d, slot %d, dim %d) out of range", kv, head, slot, dim);
  return mts::elem_offset(kv, head, slot, dim, g.S, g.D, g.es);
}

int32_t mts_kv_unpack(const mts_cache_desc* cache, int32_t layer, const void* staging, int32_t num_segs,
                      const int32_t* seg_user, const int32_t* seg_pos, const int64_t* seg_tok_indptr,
                      int32_t max_seg_tokens, const mts_batch_meta* meta, void* stream) {
  mts::PoolGeom g{};
  mts::BatchDev b{};
  mts::SegDev s{};
  int32_t st;
  if ((st = check_cache(cache, layer, true, &g)) != MTS_OK) return st;
  if ((st = check_meta(meta, false, true, &b)) != MTS_OK) return st;
  if ((st = check_segs(num_segs, seg_user, seg_pos, seg_tok_indptr, max_seg_tokens, &s)) != MTS_OK) return st;
  if (num_segs == 0 || max_seg_tokens == 0) return MTS_OK;
  if (!staging) return fail(MTS_ERR_INVALID_ARG, "staging is NULL");
  if (!aligned(staging, 16)) return fail(MTS_ERR_INVALID_ARG, "staging is not 16-byte aligned");
  if (b.batch == 0) return fail(MTS_ERR_SHAPE, "segments given for an empty batch");
  return hip_status(mts::launch_unpack(g, staging, s, b, static_cast<hipStream_t>(stream)), "mts_kv_unpack launch");
}

int32_t mts_kv_pack(const mts_cache_desc* cache, int32_t layer, void* staging_out, int32_t num_segs,
                    const int32_t* seg_user, const int32_t* seg_pos, const int64_t* seg_tok_indptr,
                    int32_t max_seg_tokens, const mts_batch_meta* meta, void* stream) {
  mts::PoolGeom g{};
  mts::BatchDev b{};
  mts::SegDev s{};
  int32_t st;
  if ((st = check_cache(cache, layer, true, &g)) != MTS_OK) return st;
  if ((st = check_meta(meta, false, true, &b)) != MTS_OK) return st;
  if ((st = check_segs(num_segs, seg_user, seg_pos, seg_tok_indptr, max_seg_tokens, &s)) != MTS_OK) return st;
  if (num_segs == 0 || max_seg_tokens == 0) return MTS_OK;
  if (!staging_out) return fail(MTS_ERR_INVALID_ARG, "staging_out is NULL");
  if (!aligned(staging_out, 16)) return fail(MTS_ERR_INVALID_ARG, "staging_out is not 16-byte aligned");
  if (b.batch == 0) return fail(MTS_ERR_SHAPE, "segments given for an empty batch");
  return hip_status(mts::launch_pack(g, staging_out, s, b, static_cast<hipStream_t>(stream)), "mts_kv_pack launch");
}

// mts_kv_unpack_layers / mts_kv_pack_layers
static int32_t move_layers(bool pack, const mts_cache_desc* cache, int32_t layer_begin, int32_t layer_count, void* staging,
                    int64_t staging_layer_stride_bytes, int32_t num_segs, const int32_t* seg_user,
                    const int32_t* seg_pos, const int64_t* seg_tok_indptr, int32_t max_seg_tokens,
                    const mts_batch_meta* meta, void* stream) {
  mts::PoolGeom g{};
  mts::BatchDev b{};
  mts::SegDev s{};
  int32_t st;
  if (layer_count < 0) return fail(MTS_ERR_INVALID_ARG, "layer_count is negative");
  if ((st = check_cache(cache, layer_begin, true, &g)) != MTS_OK) return st;
  if (layer_count > cache->num_layers - layer_begin)
    return fail(MTS_ERR_INVALID_ARG, "layers [%d, %d) exceed the cache's %d layers", layer_begin,
                layer_begin + layer_count, cache->num_layers);
  if ((st = check_meta(meta, false, true, &b)) != MTS_OK) return st;
  if ((st = check_segs(num_segs, seg_user, seg_pos, seg_tok_indptr, max_seg_tokens, &s)) != MTS_OK) return st;
  if (num_segs == 0 || max_seg_tokens == 0 || layer_count == 0) return MTS_OK;
  if (!staging) return fail(MTS_ERR_INVALID_ARG, "staging is NULL");
  if (!aligned(staging, 16) || (staging_layer_stride_bytes & 15) || staging_layer_stride_bytes < 0)
    return fail(MTS_ERR_INVALID_ARG, "staging and its layer stride must be multiples of 16 bytes");
  if (b.batch == 0) return fail(MTS_ERR_SHAPE, "segments given for an empty batch");
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const hipError_t e = pack ? mts::launch_pack(g, staging, s, b, hs, layer_count, cache->layer_stride_bytes,
                                               staging_layer_stride_bytes)
                            : mts::launch_unpack(g, staging, s, b, hs, layer_count, cache->layer_stride_bytes,
                                                 staging_layer_stride_bytes);
  return hip_status(e, pack ? "mts_kv_pack_layers launch" : "mts_kv_unpack_layers launch");
}

int32_t mts_kv_unpack_layers(const mts_cache_desc* cache, int32_t layer_begin, int32_t layer_count,
                             const void* staging, int64_t staging_layer_stride_bytes, int32_t num_segs,
                             const int32_t* seg_user, const int32_t* seg_pos, const int64_t* seg_tok_indptr,
                             int32_t max_seg_tokens, const mts_batch_meta* meta, void* stream) {
  return move_layers(false, cache, layer_begin, layer_count, const_cast<void*>(staging), staging_layer_stride_bytes,
                     num_segs, seg_user, seg_pos, seg_tok_indptr, max_seg_tokens, meta, stream);
}

int32_t mts_kv_pack_layers(const mts_cache_desc* cache, int32_t layer_begin, int32_t layer_count,
                           void* staging_out, int64_t staging_layer_stride_bytes, int32_t num_segs,
                           const int32_t* seg_user, const int32_t* seg_pos, const int64_t* seg_tok_indptr,
                           int32_t max_seg_tokens, const mts_batch_meta* meta, void* stream) {
  return move_layers(true, cache, layer_begin, layer_count, staging_out, staging_layer_stride_bytes, num_segs,
                     seg_user, seg_pos, seg_tok_indptr, max_seg_tokens, meta, stream);
}

int32_t mts_kv_append(const mts_cache_desc* cache, int32_t layer, const void* k_new, const void* v_new,
                      const mts_batch_meta* meta, void* stream) {
  mts::PoolGeom g{};
  mts::BatchDev b{};
  int32_t st;
  if ((st = check_cache(cache, layer, true, &g)) != MTS_OK) return st;
  if ((st = check_meta(meta, true, true, &b)) != MTS_OK) return st;
  if (b.batch == 0 || b.total_new == 0) return MTS_OK;
  if (!k_new || !v_new) return fail(MTS_ERR_INVALID_ARG, "k_new / v_new is NULL");
  if (!aligned(k_new, 16) || !aligned(v_new, 16))
    return fail(MTS_ERR_INVALID_ARG, "k_new / v_new is not 16-byte aligned");
  return hip_status(mts::launch_append(g, k_new, v_new, b, static_cast<hipStream_t>(stream)), "mts_kv_append launch");
}

int32_t mts_kv_append_layers(const mts_cache_desc* cache, int32_t layer_begin, int32_t layer_count, const void* k_new,
                             const void* v_new, int64_t rows_layer_stride_bytes, const mts_batch_meta* meta,
                             void* stream) {
  mts::PoolGeom g{};
  mts::BatchDev b{};
  int32_t st;
  if (layer_count < 0) return fail(MTS_ERR_INVALID_ARG, "layer_count is negative");
  if ((st = check_cache(cache, layer_begin, true, &g)) != MTS_OK) return st;
  if (layer_count > cache->num_layers - layer_begin)
    return fail(MTS_ERR_INVALID_ARG, "layers [%d, %d) exceed the cache's %d layers", layer_begin,
                layer_begin + layer_count, cache->num_layers);
  if ((st = check_meta(meta, true, true, &b)) != MTS_OK) return st;
  if (b.batch == 0 || b.total_new == 0 || layer_count == 0) return MTS_OK;
  if (!k_new || !v_new) return fail(MTS_ERR_INVALID_ARG, "k_new / v_new is NULL");
  if (!aligned(k_new, 16) || !aligned(v_new, 16) || (rows_layer_stride_bytes & 15) || rows_layer_stride_bytes < 0)
    return fail(MTS_ERR_INVALID_ARG, "k_new / v_new and their layer stride must be multiples of 16 bytes");
  return hip_status(mts::launch_append(g, k_new, v_new, b, static_cast<hipStream_t>(stream), layer_count,
                                       cache->layer_stride_bytes, rows_layer_stride_bytes),
                    "mts_kv_append_layers launch");
}

int32_t mts_attn_set_tuning(const mts_attn_tuning* t) {
  const mts_attn_tuning none{0, 0, 0, 0};
  if (!t) t = &none;
  if (t->min_tiles < 0 || t->max_waves < 0 || t->pair_cost < 0 || t->kernel < 0 || t->kernel > MTS_ATTN_KERNEL_PLAIN)
    return fail(MTS_ERR_INVALID_ARG, "tuning fields must be >= 0 and kernel one of MTS_ATTN_KERNEL_*");
  mts::g_tune_min_tiles.store(t->min_tiles, std::memory_order_relaxed);
  mts::g_tune_max_waves.store(t->max_waves, std::memory_order_relaxed);
  mts::g_tune_pair_cost.store(t->pair_cost, std::memory_order_relaxed);
  mts::g_tune_kernel.store(t->kernel, std::memory_order_relaxed);
  return MTS_OK;
}

int64_t mts_attn_workspace_bytes(const mts_cache_desc* cache, const mts_batch_meta* meta) {
  mts::PoolGeom g{};
  mts::BatchDev b{};
  int32_t st;
  if ((st = check_cache(cache, 0, false, &g)) != MTS_OK) return st;
  if ((st = check_meta(meta, true, false, &b)) != MTS_OK) return st;
  const mts::AttnPlan plan = mts::plan_attention(g, b);
  if (plan.too_large) return fail(MTS_ERR_UNSUPPORTED, "too many query tiles or kv tiles for one call");
  return plan.ws_bytes;
}

}  // extern "C"

namespace {

// the streaming kernel addresses the elements of k_new / v_new with 32-bit offsets
bool rows_fit_32bit(const mts::PoolGeom& g, const mts::BatchDev& b) {
  return (int64_t)b.total_new * g.H * g.D < (1ll << 31);
}

// mts_attn_incremental (inv_norm == 0) and mts_attn_pointwise (inv_norm > 0); with `unappended`,
// the step's K/V rows come from k_new / v_new instead of the pool
int32_t attention_call(const char* name, const mts_cache_desc* cache, int32_t layer, const void* q, void* out,
                       const mts_batch_meta* meta, float sm_scale, float inv_norm, void* workspace,
                       int64_t workspace_bytes, void* stream, bool unappended = false,
                       const void* k_new = nullptr, const void* v_new = nullptr,
                       const mts::StagedHistories* hist = nullptr) {
  mts::PoolGeom g{};
  mts::BatchDev b{};
  int32_t st;
  if ((st = check_cache(cache, layer, true, &g)) != MTS_OK) return st;
  if ((st = check_meta(meta, true, true, &b)) != MTS_OK) return st;
  if (!(sm_scale >= 0.f) || sm_scale > 1e30f)
    return fail(MTS_ERR_INVALID_ARG, "sm_scale must be finite and >= 0 (0 selects 1/sqrt(D))");
  if (b.batch == 0 || b.total_new == 0) return MTS_OK;
  if (!q || !out) return fail(MTS_ERR_INVALID_ARG, "q / out is NULL");
  if (!aligned(q, 16) || !aligned(out, 16)) return fail(MTS_ERR_INVALID_ARG, "q / out is not 16-byte aligned");
  if (unappended) {
    if (!k_new || !v_new) return fail(MTS_ERR_INVALID_ARG, "k_new / v_new is NULL");
    if (!aligned(k_new, 16) || !aligned(v_new, 16))
      return fail(MTS_ERR_INVALID_ARG, "k_new / v_new is not 16-byte aligned");
  }
  const mts::AttnPlan plan = mts::plan_attention(g, b);
  if (plan.too_large)
    return fail(MTS_ERR_UNSUPPORTED, "batch %d exceeds 4096 users, batch x ceil(max_new %d / 64) exceeds 16384 "
                "query tiles, or the call has 2^31 or more kv tiles", b.batch, b.max_new);
  if (plan.ws_bytes > 0) {
    if (!workspace) return fail(MTS_ERR_WORKSPACE, "workspace is NULL but %lld bytes are needed", (long long)plan.ws_bytes);
    if (workspace_bytes < plan.ws_bytes)
      return fail(MTS_ERR_WORKSPACE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes,
                  (long long)plan.ws_bytes);
    if (!aligned(workspace, 256)) return fail(MTS_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  }
  const float scale = sm_scale > 0.f ? sm_scale : 1.0f / sqrtf((float)g.D);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (plan.use_mfma && !plan.use_prefill && !(unappended && !rows_fit_32bit(g, b)))
    return hip_status(mts::launch_attn_mfma(g, plan, q, out, b, scale, inv_norm, plan.ws_bytes > 0 ? workspace : nullptr, s,
                                            unappended ? k_new : nullptr, unappended ? v_new : nullptr, hist), name);
  if (hist)
    return fail(MTS_ERR_UNSUPPORTED, "histories in the onload buffer are read by the streaming bf16 kernel only "
                "(short new segments): unpack them first for this shape");
  // The other kernels read every key from the pool: an unappended call writes the rows there
  // first, on the same stream (a long new segment or fp32 elements; the copy is a small part
  // of such a call).
  if (unappended) {
    const hipError_t e = mts::launch_append(g, k_new, v_new, b, s);
    if (e != hipSuccess) return hip_status(e, name);
  }
  if (plan.use_mfma && plan.use_prefill)
    return hip_status(mts::launch_attn_prefill(g, q, out, b, scale, inv_norm, s), name);
  return hip_status(mts::launch_attn_generic(g, q, out, b, scale, inv_norm, s), name);
}

}  // namespace

extern "C" {

int32_t mts_attn_incremental(const mts_cache_desc* cache, int32_t layer, const void* q, void* out,
                             const mts_batch_meta* meta, float sm_scale, void* workspace,
                             int64_t workspace_bytes, void* stream) {
  return attention_call("mts_attn_incremental launch", cache, layer, q, out, meta, sm_scale, 0.f, workspace,
                        workspace_bytes, stream);
}

int32_t mts_attn_incremental_noalloc(const mts_cache_desc* cache, int32_t layer, const void* q, void* out,
                                     const mts_batch_meta* meta, float sm_scale, void* stream) {
  // the shape's needs are known from the host-side bounds alone: refuse before touching the device
  mts::PoolGeom g{};
  mts::BatchDev b{};
  int32_t st;
  if ((st = check_cache(cache, layer, true, &g)) != MTS_OK) return st;
  if ((st = check_meta(meta, true, true, &b)) != MTS_OK) return st;
  const mts::AttnPlan plan = mts::plan_attention(g, b);
  if (plan.too_large) return fail(MTS_ERR_UNSUPPORTED, "too many query tiles or kv tiles for one call");
  if (plan.ws_bytes > kScratchBytes)
    return fail(MTS_ERR_WORKSPACE, "this shape needs %lld bytes of scratch, the library-owned buffer of "
                "mts_attn_incremental_noalloc holds %lld: use mts_attn_incremental with a workspace",
                (long long)plan.ws_bytes, (long long)kScratchBytes);
  if (b.batch == 0 || b.total_new == 0) return MTS_OK;
  void* ws = scratch_on_current_device();
  if (!ws) return MTS_ERR_HIP;
  return attention_call("mts_attn_incremental_noalloc launch", cache, layer, q, out, meta, sm_scale, 0.f, ws,
                        kScratchBytes, stream);
}

int32_t mts_attn_pointwise(const mts_cache_desc* cache, int32_t layer, const void* q, void* out,
                           const mts_batch_meta* meta, float sm_scale, float inv_norm, void* workspace,
                           int64_t workspace_bytes, void* stream) {
  if (!(inv_norm > 0.f) || inv_norm > 1e30f)
    return fail(MTS_ERR_INVALID_ARG, "inv_norm must be finite and > 0");
  return attention_call("mts_attn_pointwise launch", cache, layer, q, out, meta, sm_scale, inv_norm, workspace,
                        workspace_bytes, stream);
}

int32_t mts_attn_unappended_appends(const mts_cache_desc* cache, const mts_batch_meta* meta) {
  mts::PoolGeom g{};
  mts::BatchDev b{};
  int32_t st;
  if ((st = check_cache(cache, 0, false, &g)) != MTS_OK) return st;
  if ((st = check_meta(meta, true, false, &b)) != MTS_OK) return st;
  if (b.batch == 0 || b.total_new == 0) return 0;
  const mts::AttnPlan plan = mts::plan_attention(g, b);
  return (plan.use_mfma && !plan.use_prefill && rows_fit_32bit(g, b)) ? 0 : 1;
}

int32_t mts_attn_incremental_unappended(const mts_cache_desc* cache, int32_t layer, const void* q, const void* k_new,
                                        const void* v_new, void* out, const mts_batch_meta* meta, float sm_scale,
                                        void* workspace, int64_t workspace_bytes, void* stream) {
  return attention_call("mts_attn_incremental_unappended launch", cache, layer, q, out, meta, sm_scale, 0.f, workspace,
                        workspace_bytes, stream, true, k_new, v_new);
}

int32_t mts_attn_pointwise_unappended(const mts_cache_desc* cache, int32_t layer, const void* q, const void* k_new,
                                      const void* v_new, void* out, const mts_batch_meta* meta, float sm_scale,
                                      float inv_norm, void* workspace, int64_t workspace_bytes, void* stream) {
  if (!(inv_norm > 0.f) || inv_norm > 1e30f)
    return fail(MTS_ERR_INVALID_ARG, "inv_norm must be finite and > 0");
  return attention_call("mts_attn_pointwise_unappended launch", cache, layer, q, out, meta, sm_scale, inv_norm,
                        workspace, workspace_bytes, stream, true, k_new, v_new);
}

int32_t mts_attn_incremental_staged(const mts_cache_desc* cache, int32_t layer, const void* q, const void* k_new,
                                    const void* v_new, const void* staged_rows, const int32_t* staged_first_run,
                                    const int64_t* staged_run_tok, int32_t chunk_tokens, void* out,
                                    const mts_batch_meta* meta, float sm_scale, void* workspace,
                                    int64_t workspace_bytes, void* stream) {
  if (!staged_rows || !staged_first_run || !staged_run_tok)
    return fail(MTS_ERR_INVALID_ARG, "staged_rows / staged_first_run / staged_run_tok is NULL");
  if (!aligned(staged_rows, 16)) return fail(MTS_ERR_INVALID_ARG, "staged_rows is not 16-byte aligned");
  if (chunk_tokens <= 0 || chunk_tokens % 32 != 0)
    return fail(MTS_ERR_INVALID_ARG, "chunk_tokens must be a positive multiple of 32");
  if (cache && (int64_t)chunk_tokens * cache->num_heads * cache->head_dim * 4 >= (1ll << 31))
    return fail(MTS_ERR_UNSUPPORTED, "a run of %d tokens exceeds 2 GiB", chunk_tokens);
  const mts::StagedHistories hist{staged_rows, staged_first_run, staged_run_tok, chunk_tokens};
  return attention_call("mts_attn_incremental_staged launch", cache, layer, q, out, meta, sm_scale, 0.f, workspace,
                        workspace_bytes, stream, true, k_new, v_new, &hist);
}

int32_t mts_stage_h2d_async(void* device_dst, const void* host_src, int64_t bytes, void* stream) {
  if (bytes < 0) return fail(MTS_ERR_INVALID_ARG, "negative byte count");
  if (bytes == 0) return MTS_OK;
  if (!device_dst || !host_src) return fail(MTS_ERR_INVALID_ARG, "NULL pointer");
  return hip_status(hipMemcpyAsync(device_dst, host_src, (size_t)bytes, hipMemcpyHostToDevice,
                                   static_cast<hipStream_t>(stream)), "host-to-device staging copy");
}

int32_t mts_stage_d2h_async(void* host_dst, const void* device_src, int64_t bytes, void* stream) {
  if (bytes < 0) return fail(MTS_ERR_INVALID_ARG, "negative byte count");
  if (bytes == 0) return MTS_OK;
  if (!host_dst || !device_src) return fail(MTS_ERR_INVALID_ARG, "NULL pointer");
  return hip_status(hipMemcpyAsync(host_dst, device_src, (size_t)bytes, hipMemcpyDeviceToHost,
                                   static_cast<hipStream_t>(stream)), "device-to-host staging copy");
}

}  // extern "C"
