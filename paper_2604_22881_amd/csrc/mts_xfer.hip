// Transfer pipeline: the background onload and offload paths either side of the kernels
// (Sec. 4.2 "Pipelined Onload via Double Buffering", "Transient Offload Pipeline", "Offload
// Capacity Control"; Sec. 4.4 four-stream model and layer-wise synchronisation; Alg. 1
// steps 2, 7, 8.3 and 9).  Host code only: it drives hipMemcpyAsync, events and the library's
// own mts_kv_unpack / mts_kv_pack.
//
// Onload worker, per layer and run:  host chunk --copy threads--> pinned[b]  --DMA, onload
// stream--> device onload buffer; the two pinned buffers alternate, so the host copy of run
// k+1 overlaps the DMA of run k.  After a layer's last run: event -> scatter stream waits ->
// mts_kv_unpack(layer) -> "layer ready" event, which mts_xfer_onload_wait_layer hands to the
// compute stream.  A stream may only be made to wait for an event that has already been
// recorded, so that call first blocks the host (bounded) until the worker has recorded it.
//
// Offload worker, per task:  offload stream waits for the caller's stream; per layer
// mts_kv_pack into a transient region of the arena; per run  DMA to pinned[b]  while the copy
// threads move pinned[b^1] into the host chunk.  Admission control (quota in tokens, arena
// space) happens in the submitting thread before anything is queued.
#include <hip/hip_runtime.h>
#include <string.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <mutex>
#include <thread>
#include <vector>

#include "../../include/mtserve.h"
#include "mts_copy_pool.hpp"
#include "mts_internal.hpp"

using mts::CopyPool;

namespace {

constexpr auto kHostWait = std::chrono::seconds(60);   // every host-side wait is bounded by this

struct Task {
  mts_cache_desc cache;
  mts_batch_meta meta;
  int32_t num_segs = 0;
  const int32_t* seg_user = nullptr;
  const int32_t* seg_pos = nullptr;
  const int64_t* seg_tok_indptr = nullptr;
  int32_t max_seg_tokens = 0;
  std::vector<int64_t> tok;      // host copy of seg_tok_indptr
  std::vector<void*> host;       // [layers * num_segs]
  int64_t row_bytes = 0;         // 2 * H * D * es: K and V of one token
  // onload
  char* staging = nullptr;
  int64_t stride = 0;
  // offload
  hipEvent_t after = nullptr;
  int64_t arena_off = 0, arena_bytes = 0, tokens = 0;
};

}  // namespace

struct mts_xfer {
  int dev = 0;
  mts_xfer_config cfg{};
  hipStream_t s_onload = nullptr, s_scatter = nullptr, s_offload = nullptr;
  void* pin_on[2] = {nullptr, nullptr};
  void* pin_off[2] = {nullptr, nullptr};
  hipEvent_t ev_on_dma[2] = {nullptr, nullptr};
  hipEvent_t ev_off_dma[2] = {nullptr, nullptr};
  bool on_dma_used[2] = {false, false};
  std::vector<hipEvent_t> ev_layer_dma, ev_layer_ready;
  bool had_onload = false;
  char* arena = nullptr;

  CopyPool* pool_on = nullptr;
  CopyPool* pool_off = nullptr;

  // onload worker state (mu_on)
  std::thread th_on;
  std::mutex mu_on;
  std::condition_variable cv_on;
  bool on_has_task = false, on_busy = false;
  std::atomic<bool> stop{false};
  Task on_task;
  int on_layers_enqueued = 0;
  int32_t on_err = MTS_OK;
  char on_err_text[256] = "";

  // offload worker state (mu_off)
  std::thread th_off;
  std::mutex mu_off;
  std::condition_variable cv_off;
  std::deque<Task> off_q;
  bool off_busy = false;
  int64_t pending_tokens = 0;
  int64_t arena_head = 0;      // ring allocator: regions are freed in the order they were taken
  int64_t arena_tail = 0;
  int arena_regions = 0;
  int32_t off_err = MTS_OK;
  char off_err_text[256] = "";
};

namespace {

#define XFER_HIP(call, errvar, textvar)                                              \
  do {                                                                               \
    hipError_t e_ = (call);                                                          \
    if (e_ != hipSuccess) {                                                          \
      errvar = MTS_ERR_HIP;                                                          \
      snprintf(textvar, sizeof(textvar), "%s: %s", #call, hipGetErrorString(e_));    \
      return false;                                                                  \
    }                                                                                \
  } while (0)

bool run_onload(mts_xfer* x, const Task& t, int32_t& err, char (&text)[256]) {
  const int L = x->cfg.num_layers;
  if (x->had_onload)   // the previous task's scatter kernels still read the onload buffer
    XFER_HIP(hipStreamWaitEvent(x->s_onload, x->ev_layer_ready[L - 1], 0), err, text);
  int k = 0;
  for (int l = 0; l < L; ++l) {
    // Consecutive runs of a layer are consecutive in the onload buffer: as many as fit one pinned
    // buffer travel in one DMA (a copy of a megabyte or two is dominated by its fixed cost).
    for (int s = 0; s < t.num_segs;) {
      int e = s;
      int64_t bytes = 0;
      while (e < t.num_segs && (e == s || bytes + (t.tok[e + 1] - t.tok[e]) * t.row_bytes <= x->cfg.pinned_bytes)) {
        bytes += (t.tok[e + 1] - t.tok[e]) * t.row_bytes;
        ++e;
      }
      if (bytes > 0) {
        const int b = k & 1;
        if (x->on_dma_used[b]) XFER_HIP(hipEventSynchronize(x->ev_on_dma[b]), err, text);   // pinned[b] has left for the device
        char* pin = static_cast<char*>(x->pin_on[b]);
        for (int r = s; r < e; ++r) {
          const int64_t rb = (t.tok[r + 1] - t.tok[r]) * t.row_bytes;
          if (rb > 0) x->pool_on->copy(pin + (t.tok[r] - t.tok[s]) * t.row_bytes, t.host[(size_t)l * t.num_segs + r], (size_t)rb);
        }
        XFER_HIP(hipMemcpyAsync(t.staging + l * t.stride + t.tok[s] * t.row_bytes, pin, (size_t)bytes,
                                hipMemcpyHostToDevice, x->s_onload), err, text);
        XFER_HIP(hipEventRecord(x->ev_on_dma[b], x->s_onload), err, text);
        x->on_dma_used[b] = true;
        ++k;
      }
      s = e;
    }
    XFER_HIP(hipEventRecord(x->ev_layer_dma[l], x->s_onload), err, text);
    XFER_HIP(hipStreamWaitEvent(x->s_scatter, x->ev_layer_dma[l], 0), err, text);
    const int32_t st = mts_kv_unpack(&t.cache, l, t.staging + l * t.stride, t.num_segs, t.seg_user, t.seg_pos,
                                     t.seg_tok_indptr, t.max_seg_tokens, &t.meta, x->s_scatter);
    if (st != MTS_OK) {
      err = st;
      snprintf(text, sizeof(text), "mts_kv_unpack of layer %d: %s", l, mts_last_error());
      return false;
    }
    XFER_HIP(hipEventRecord(x->ev_layer_ready[l], x->s_scatter), err, text);
    {
      std::lock_guard<std::mutex> g(x->mu_on);
      x->on_layers_enqueued = l + 1;
    }
    x->cv_on.notify_all();
  }
  x->had_onload = true;
  return true;
}

void onload_worker(mts_xfer* x) {
  (void)hipSetDevice(x->dev);
  for (;;) {
    Task t;
    {
      std::unique_lock<std::mutex> g(x->mu_on);
      x->cv_on.wait(g, [&] { return x->on_has_task || x->stop; });
      if (!x->on_has_task) return;
      t = std::move(x->on_task);
      x->on_has_task = false;
      x->on_busy = true;
    }
    int32_t err = MTS_OK;
    char text[256] = "";
    const bool ok = run_onload(x, t, err, text);
    {
      std::lock_guard<std::mutex> g(x->mu_on);
      if (!ok && x->on_err == MTS_OK) {
        x->on_err = err;
        memcpy(x->on_err_text, text, sizeof(text));
      }
      x->on_layers_enqueued = x->cfg.num_layers;   // nobody may be left waiting, failed or not
      x->on_busy = false;
    }
    x->cv_on.notify_all();
  }
}

bool run_offload(mts_xfer* x, const Task& t, int32_t& err, char (&text)[256]) {
  const int L = x->cfg.num_layers;
  XFER_HIP(hipStreamWaitEvent(x->s_offload, t.after, 0), err, text);
  const int64_t layer_bytes = t.tokens * t.row_bytes;
  char* region = x->arena + t.arena_off;
  int k = 0;
  bool have_prev = false;
  int prev_l = 0, prev_s = 0, prev_e = 0;
  auto drain_prev = [&](int b) -> bool {   // pinned[b] -> host chunks, once its DMA has landed
    XFER_HIP(hipEventSynchronize(x->ev_off_dma[b]), err, text);
    const char* pin = static_cast<const char*>(x->pin_off[b]);
    for (int r = prev_s; r < prev_e; ++r) {
      const int64_t rb = (t.tok[r + 1] - t.tok[r]) * t.row_bytes;
      if (rb > 0) x->pool_off->copy(t.host[(size_t)prev_l * t.num_segs + r], pin + (t.tok[r] - t.tok[prev_s]) * t.row_bytes, (size_t)rb);
    }
    return true;
  };
  // one gather launch for all layers (the region holds them layer after layer), then the DMAs
  const int32_t st = mts_kv_pack_layers(&t.cache, 0, L, region, layer_bytes, t.num_segs, t.seg_user, t.seg_pos,
                                        t.seg_tok_indptr, t.max_seg_tokens, &t.meta, x->s_offload);
  if (st != MTS_OK) {
    err = st;
    snprintf(text, sizeof(text), "mts_kv_pack_layers: %s", mts_last_error());
    return false;
  }
  for (int l = 0; l < L; ++l) {
    for (int s = 0; s < t.num_segs;) {      // consecutive runs, as many as fit one pinned buffer, per DMA
      int e = s;
      int64_t bytes = 0;
      while (e < t.num_segs && (e == s || bytes + (t.tok[e + 1] - t.tok[e]) * t.row_bytes <= x->cfg.pinned_bytes)) {
        bytes += (t.tok[e + 1] - t.tok[e]) * t.row_bytes;
        ++e;
      }
      if (bytes > 0) {
        const int b = k & 1;
        XFER_HIP(hipMemcpyAsync(x->pin_off[b], region + l * layer_bytes + t.tok[s] * t.row_bytes, (size_t)bytes,
                                hipMemcpyDeviceToHost, x->s_offload), err, text);
        XFER_HIP(hipEventRecord(x->ev_off_dma[b], x->s_offload), err, text);
        if (have_prev && !drain_prev(b ^ 1)) return false;      // overlaps the copy just enqueued
        prev_l = l; prev_s = s; prev_e = e;
        have_prev = true;
        ++k;
      }
      s = e;
    }
  }
  if (have_prev && !drain_prev((k - 1) & 1)) return false;
  return true;
}

void offload_worker(mts_xfer* x) {
  (void)hipSetDevice(x->dev);
  for (;;) {
    Task t;
    {
      std::unique_lock<std::mutex> g(x->mu_off);
      x->cv_off.wait(g, [&] { return !x->off_q.empty() || x->stop; });
      if (x->off_q.empty()) return;
      t = std::move(x->off_q.front());
      x->off_q.pop_front();
      x->off_busy = true;
    }
    int32_t err = MTS_OK;
    char text[256] = "";
    const bool ok = run_offload(x, t, err, text);
    if (!ok) (void)hipStreamSynchronize(x->s_offload);   // nothing may still read the region we free below
    (void)hipEventDestroy(t.after);
    {
      std::lock_guard<std::mutex> g(x->mu_off);
      if (!ok && x->off_err == MTS_OK) {
        x->off_err = err;
        memcpy(x->off_err_text, text, sizeof(text));
      }
      x->pending_tokens -= t.tokens;
      x->arena_tail = t.arena_off + t.arena_bytes;
      if (--x->arena_regions == 0) x->arena_head = x->arena_tail = 0;
      x->off_busy = false;
    }
    x->cv_off.notify_all();
  }
}

// Fills the parts of a task that both directions share; validates what the host can see.
int32_t make_task(const mts_xfer* x, const mts_cache_desc* cache, const mts_batch_meta* meta,
                  const mts_xfer_runs* runs, Task* t) {
  if (!x) return mts::set_error(MTS_ERR_INVALID_ARG, "mts_xfer is NULL");
  if (!cache || !meta || !runs) return mts::set_error(MTS_ERR_INVALID_ARG, "cache / meta / runs is NULL");
  const int64_t page_bytes = mts_page_bytes(cache);       // validates the descriptor
  if (page_bytes < 0) return (int32_t)page_bytes;
  if (cache->num_layers != x->cfg.num_layers)
    return mts::set_error(MTS_ERR_SHAPE, "cache has %d layers, the pipeline was created for %d", cache->num_layers,
                          x->cfg.num_layers);
  if (runs->num_segs < 0 || runs->num_segs > 65535) return mts::set_error(MTS_ERR_INVALID_ARG, "num_segs out of range");
  if (runs->num_segs > 0 && (!runs->seg_user || !runs->seg_pos || !runs->seg_tok_indptr || !runs->host_tok_indptr ||
                             !runs->host_runs))
    return mts::set_error(MTS_ERR_INVALID_ARG, "a run array is NULL");
  const int es = cache->dtype == MTS_F32 ? 4 : 2;
  t->cache = *cache;
  t->meta = *meta;
  t->num_segs = runs->num_segs;
  t->seg_user = runs->seg_user;
  t->seg_pos = runs->seg_pos;
  t->seg_tok_indptr = runs->seg_tok_indptr;
  t->max_seg_tokens = runs->max_seg_tokens;
  t->row_bytes = 2ll * cache->num_heads * cache->head_dim * es;
  t->tok.assign(runs->host_tok_indptr, runs->host_tok_indptr + (runs->num_segs > 0 ? runs->num_segs + 1 : 0));
  if (t->tok.empty()) t->tok.push_back(0);
  if (t->tok.front() != 0) return mts::set_error(MTS_ERR_SHAPE, "host_tok_indptr[0] must be 0");
  for (int s = 0; s < runs->num_segs; ++s) {
    const int64_t n = t->tok[s + 1] - t->tok[s];
    if (n < 0 || n > runs->max_seg_tokens)
      return mts::set_error(MTS_ERR_SHAPE, "run %d has %lld tokens, max_seg_tokens is %d", s, (long long)n,
                            runs->max_seg_tokens);
    if (n * t->row_bytes > x->cfg.pinned_bytes)
      return mts::set_error(MTS_ERR_SHAPE, "run %d (%lld bytes) does not fit a pinned buffer of %lld bytes", s,
                            (long long)(n * t->row_bytes), (long long)x->cfg.pinned_bytes);
  }
  t->tokens = t->tok.back() - t->tok.front();
  const size_t nptr = (size_t)x->cfg.num_layers * runs->num_segs;
  t->host.assign(runs->host_runs, runs->host_runs + nptr);
  for (size_t i = 0; i < nptr; ++i) {
    const int s = (int)(i % runs->num_segs);
    if (!t->host[i] && t->tok[s + 1] > t->tok[s]) return mts::set_error(MTS_ERR_INVALID_ARG, "host run %zu is NULL", i);
  }
  return MTS_OK;
}

}  // namespace

extern "C" {

int32_t mts_xfer_create(const mts_xfer_config* c, mts_xfer** out) {
  if (!c || !out) return mts::set_error(MTS_ERR_INVALID_ARG, "config / out is NULL");
  *out = nullptr;
  if (c->pinned_bytes < 16 || c->num_layers < 1 || c->copy_threads < 1 || c->copy_threads > 64 ||
      c->offload_arena_bytes < 0 || c->offload_quota_tokens < 0)
    return mts::set_error(MTS_ERR_INVALID_ARG, "pinned_bytes >= 16, num_layers >= 1, copy_threads in [1, 64], "
                          "arena and quota >= 0 required");
  mts_xfer* x = new mts_xfer;
  x->cfg = *c;
  hipError_t e = hipGetDevice(&x->dev);
  auto bail = [&](const char* what) {
    const int32_t st = mts::set_error(MTS_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    mts_xfer_destroy(x);
    return st;
  };
  if (e != hipSuccess) return bail("hipGetDevice");
  if ((e = hipStreamCreateWithFlags(&x->s_onload, hipStreamNonBlocking)) != hipSuccess) return bail("stream");
  if ((e = hipStreamCreateWithFlags(&x->s_scatter, hipStreamNonBlocking)) != hipSuccess) return bail("stream");
  if ((e = hipStreamCreateWithFlags(&x->s_offload, hipStreamNonBlocking)) != hipSuccess) return bail("stream");
  for (int b = 0; b < 2; ++b) {
    if ((e = hipHostMalloc(&x->pin_on[b], (size_t)c->pinned_bytes, hipHostMallocDefault)) != hipSuccess) return bail("hipHostMalloc");
    if ((e = hipHostMalloc(&x->pin_off[b], (size_t)c->pinned_bytes, hipHostMallocDefault)) != hipSuccess) return bail("hipHostMalloc");
    if ((e = hipEventCreateWithFlags(&x->ev_on_dma[b], hipEventDisableTiming)) != hipSuccess) return bail("event");
    if ((e = hipEventCreateWithFlags(&x->ev_off_dma[b], hipEventDisableTiming)) != hipSuccess) return bail("event");
  }
  x->ev_layer_dma.assign(c->num_layers, nullptr);
  x->ev_layer_ready.assign(c->num_layers, nullptr);
  for (int l = 0; l < c->num_layers; ++l) {
    if ((e = hipEventCreateWithFlags(&x->ev_layer_dma[l], hipEventDisableTiming)) != hipSuccess) return bail("event");
    if ((e = hipEventCreateWithFlags(&x->ev_layer_ready[l], hipEventDisableTiming)) != hipSuccess) return bail("event");
  }
  if (c->offload_arena_bytes > 0 &&
      (e = hipMalloc(reinterpret_cast<void**>(&x->arena), (size_t)c->offload_arena_bytes)) != hipSuccess)
    return bail("hipMalloc of the offload arena");
  x->pool_on = new CopyPool(c->copy_threads);
  x->pool_off = new CopyPool(c->copy_threads);
  x->th_on = std::thread(onload_worker, x);
  x->th_off = std::thread(offload_worker, x);
  *out = x;
  return MTS_OK;
}

int32_t mts_xfer_drain(mts_xfer* x) {
  if (!x) return mts::set_error(MTS_ERR_INVALID_ARG, "mts_xfer is NULL");
  int32_t st = MTS_OK;
  {
    std::unique_lock<std::mutex> g(x->mu_on);
    if (!x->cv_on.wait_for(g, kHostWait, [&] { return !x->on_has_task && !x->on_busy; }))
      return mts::set_error(MTS_ERR_HIP, "onload worker did not finish in time");
    if (x->on_err != MTS_OK) {
      st = mts::set_error(x->on_err, "onload: %s", x->on_err_text);
      x->on_err = MTS_OK;
    }
  }
  {
    std::unique_lock<std::mutex> g(x->mu_off);
    if (!x->cv_off.wait_for(g, kHostWait, [&] { return x->off_q.empty() && !x->off_busy; }))
      return mts::set_error(MTS_ERR_HIP, "offload worker did not finish in time");
    if (x->off_err != MTS_OK) {
      if (st == MTS_OK) st = mts::set_error(x->off_err, "offload: %s", x->off_err_text);
      x->off_err = MTS_OK;
    }
  }
  hipError_t e = hipSuccess;
  if (x->s_onload && (e = hipStreamSynchronize(x->s_onload)) != hipSuccess && st == MTS_OK)
    st = mts::set_error(MTS_ERR_HIP, "onload stream: %s", hipGetErrorString(e));
  if (x->s_scatter && (e = hipStreamSynchronize(x->s_scatter)) != hipSuccess && st == MTS_OK)
    st = mts::set_error(MTS_ERR_HIP, "scatter stream: %s", hipGetErrorString(e));
  if (x->s_offload && (e = hipStreamSynchronize(x->s_offload)) != hipSuccess && st == MTS_OK)
    st = mts::set_error(MTS_ERR_HIP, "offload stream: %s", hipGetErrorString(e));
  return st;
}

int32_t mts_xfer_destroy(mts_xfer* x) {
  if (!x) return MTS_OK;
  int32_t st = MTS_OK;
  if (x->th_on.joinable() || x->th_off.joinable()) {
    st = mts_xfer_drain(x);
    x->stop = true;
    { std::lock_guard<std::mutex> g(x->mu_on); }      // a worker about to wait has released its mutex by now
    { std::lock_guard<std::mutex> g(x->mu_off); }
    x->cv_on.notify_all();
    x->cv_off.notify_all();
    if (x->th_on.joinable()) x->th_on.join();
    if (x->th_off.joinable()) x->th_off.join();
  }
  delete x->pool_on;
  delete x->pool_off;
  for (int b = 0; b < 2; ++b) {
    if (x->ev_on_dma[b]) (void)hipEventDestroy(x->ev_on_dma[b]);
    if (x->ev_off_dma[b]) (void)hipEventDestroy(x->ev_off_dma[b]);
    if (x->pin_on[b]) (void)hipHostFree(x->pin_on[b]);
    if (x->pin_off[b]) (void)hipHostFree(x->pin_off[b]);
  }
  for (hipEvent_t ev : x->ev_layer_dma) if (ev) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : x->ev_layer_ready) if (ev) (void)hipEventDestroy(ev);
  if (x->arena) (void)hipFree(x->arena);
  if (x->s_onload) (void)hipStreamDestroy(x->s_onload);
  if (x->s_scatter) (void)hipStreamDestroy(x->s_scatter);
  if (x->s_offload) (void)hipStreamDestroy(x->s_offload);
  delete x;
  return st;
}

int32_t mts_xfer_onload_submit(mts_xfer* x, const mts_cache_desc* cache, const mts_batch_meta* meta,
                               const mts_xfer_runs* runs, void* staging, int64_t stride) {
  Task t;
  int32_t st = make_task(x, cache, meta, runs, &t);
  if (st != MTS_OK) return st;
  if (t.num_segs > 0 && !staging) return mts::set_error(MTS_ERR_INVALID_ARG, "staging is NULL");
  if ((reinterpret_cast<uintptr_t>(staging) & 15) || (stride & 15))
    return mts::set_error(MTS_ERR_INVALID_ARG, "staging and its layer stride must be multiples of 16 bytes");
  if (stride < t.tok.back() * t.row_bytes)
    return mts::set_error(MTS_ERR_SHAPE, "staging layer stride %lld < %lld bytes of runs per layer", (long long)stride,
                          (long long)(t.tok.back() * t.row_bytes));
  t.staging = static_cast<char*>(staging);
  t.stride = stride;
  std::unique_lock<std::mutex> g(x->mu_on);
  if (!x->cv_on.wait_for(g, kHostWait, [&] { return !x->on_has_task && !x->on_busy; }))
    return mts::set_error(MTS_ERR_HIP, "the previous onload task did not finish in time");
  if (x->on_err != MTS_OK) {
    st = mts::set_error(x->on_err, "earlier onload task: %s", x->on_err_text);
    x->on_err = MTS_OK;
    return st;
  }
  x->on_task = std::move(t);
  x->on_has_task = true;
  x->on_layers_enqueued = 0;
  g.unlock();
  x->cv_on.notify_all();
  return MTS_OK;
}

int32_t mts_xfer_onload_wait_layer(mts_xfer* x, int32_t layer, void* compute_stream) {
  if (!x) return mts::set_error(MTS_ERR_INVALID_ARG, "mts_xfer is NULL");
  if (layer < 0 || layer >= x->cfg.num_layers)
    return mts::set_error(MTS_ERR_INVALID_ARG, "layer %d out of range [0, %d)", layer, x->cfg.num_layers);
  {
    std::unique_lock<std::mutex> g(x->mu_on);
    if (!x->cv_on.wait_for(g, kHostWait, [&] { return x->on_layers_enqueued > layer || x->on_err != MTS_OK; }))
      return mts::set_error(MTS_ERR_HIP, "layer %d of the onload task was not enqueued in time", layer);
    if (x->on_err != MTS_OK) return mts::set_error(x->on_err, "onload: %s", x->on_err_text);
  }
  const hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(compute_stream), x->ev_layer_ready[layer], 0);
  if (e != hipSuccess) return mts::set_error(MTS_ERR_HIP, "hipStreamWaitEvent: %s", hipGetErrorString(e));
  return MTS_OK;
}

int32_t mts_xfer_offload_submit(mts_xfer* x, const mts_cache_desc* cache, const mts_batch_meta* meta,
                                const mts_xfer_runs* runs, void* after_stream) {
  Task t;
  int32_t st = make_task(x, cache, meta, runs, &t);
  if (st != MTS_OK) return st;
  if (t.tokens == 0) return MTS_OK;
  t.arena_bytes = (t.tokens * t.row_bytes * x->cfg.num_layers + 255) & ~255ll;
  if (t.arena_bytes > x->cfg.offload_arena_bytes)
    return mts::set_error(MTS_ERR_BUSY, "task needs %lld bytes of transient buffer, the arena has %lld",
                          (long long)t.arena_bytes, (long long)x->cfg.offload_arena_bytes);
  std::unique_lock<std::mutex> g(x->mu_off);
  if (x->pending_tokens + t.tokens > x->cfg.offload_quota_tokens)
    return mts::set_error(MTS_ERR_BUSY, "offload quota: %lld tokens pending + %lld new > %lld", (long long)x->pending_tokens,
                          (long long)t.tokens, (long long)x->cfg.offload_quota_tokens);
  // ring allocation; regions are freed in the order they were taken
  const int64_t size = x->cfg.offload_arena_bytes;
  int64_t off = -1;
  if (x->arena_regions == 0) {
    off = 0;
  } else if (x->arena_head > x->arena_tail) {            // free: [head, size) and [0, tail)
    if (size - x->arena_head >= t.arena_bytes) off = x->arena_head;
    else if (x->arena_tail >= t.arena_bytes) off = 0;
  } else if (x->arena_head < x->arena_tail) {            // free: [head, tail)
    if (x->arena_tail - x->arena_head >= t.arena_bytes) off = x->arena_head;
  }
  if (off < 0)
    return mts::set_error(MTS_ERR_BUSY, "no room for %lld bytes of transient buffer while earlier tasks are pending",
                          (long long)t.arena_bytes);
  hipError_t e = hipEventCreateWithFlags(&t.after, hipEventDisableTiming);
  if (e == hipSuccess) {
    e = hipEventRecord(t.after, static_cast<hipStream_t>(after_stream));
    if (e != hipSuccess) (void)hipEventDestroy(t.after);
  }
  if (e != hipSuccess) return mts::set_error(MTS_ERR_HIP, "event on after_stream: %s", hipGetErrorString(e));
  t.arena_off = off;
  x->arena_head = off + t.arena_bytes;
  ++x->arena_regions;
  x->pending_tokens += t.tokens;
  x->off_q.push_back(std::move(t));
  g.unlock();
  x->cv_off.notify_all();
  return MTS_OK;
}

int64_t mts_xfer_offload_pending_tokens(mts_xfer* x) {
  if (!x) return mts::set_error(MTS_ERR_INVALID_ARG, "mts_xfer is NULL");
  std::lock_guard<std::mutex> g(x->mu_off);
  return x->pending_tokens;
}

}  // extern "C"
