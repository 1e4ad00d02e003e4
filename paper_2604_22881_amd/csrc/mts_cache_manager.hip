// Host-side KVCacheManager (Sec. 3.1 "KVCacheManager", Sec. 4.3 "Cache Management"; Alg. 1
// steps 1, 2, 6, 7): sequence-length tracking, the page table of the GPU tier, page
// allocation, LRU replacement with O(1) updates (doubly-linked list + hash map), eviction as
// a pure metadata operation, and the locked-user registry that the LRU walk skips.  It
// produces the CSR metadata (prefix lengths, page_indptr / page_indices) the kernels consume.
// Host code only; no device call is made here.
#include <stdint.h>
#include <string.h>

#include <unordered_map>
#include <vector>

#include "../../include/mtserve.h"
#include "mts_internal.hpp"

namespace {

struct User {
  int64_t id = 0;
  int32_t total_len = 0;     // tokens of history the cache holds for this user (GPU or host)
  int32_t host_len = 0;      // of those, tokens persisted in the host tier: [0, host_len)
  bool on_gpu = false;       // pages hold tokens [0, total_len)
  bool locked = false;       // being read by the offload path: not a victim
  int32_t batch_new = -1;    // >= 0 while the user belongs to the batch being prepared
  std::vector<int32_t> pages;
  User* prev = nullptr;      // LRU list of users with on_gpu: head = most recent
  User* next = nullptr;
};

}  // namespace

struct mts_cm {
  int32_t num_pages = 0, page_size = 0, chunk = 0;
  std::unordered_map<int64_t, User*> users;
  std::vector<int32_t> free_pages;      // stack
  User* head = nullptr;
  User* tail = nullptr;
  std::vector<User*> batch;             // users of the prepared, not yet committed batch
  std::vector<int64_t> evicted;         // since the last mts_cm_take_evicted
  mts_cm_stats stats{};

  void unlink(User* u) {
    if (u->prev) u->prev->next = u->next; else if (head == u) head = u->next;
    if (u->next) u->next->prev = u->prev; else if (tail == u) tail = u->prev;
    u->prev = u->next = nullptr;
  }
  void push_front(User* u) {
    u->prev = nullptr;
    u->next = head;
    if (head) head->prev = u;
    head = u;
    if (!tail) tail = u;
  }
  // Zero-copy eviction: the pages go back to the pool, the host tier keeps what it has; tokens
  // the offload path had not persisted yet are no longer cached anywhere.
  void evict(User* u) {
    unlink(u);
    for (int32_t p : u->pages) free_pages.push_back(p);
    u->pages.clear();
    u->on_gpu = false;
    stats.tokens_dropped += u->total_len - u->host_len;
    u->total_len = u->host_len;
    evicted.push_back(u->id);
    ++stats.evictions;
  }
};

namespace {

int32_t pages_for(int32_t len, int32_t S) { return (int32_t)(((int64_t)len + S - 1) / S); }

}  // namespace

extern "C" {

int32_t mts_cm_create(int32_t num_pages, int32_t page_size, int32_t host_chunk_tokens, mts_cm** out) {
  if (!out) return mts::set_error(MTS_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  if (num_pages < 1 || page_size < 1 || host_chunk_tokens < 1)
    return mts::set_error(MTS_ERR_INVALID_ARG, "num_pages, page_size and host_chunk_tokens must be >= 1");
  mts_cm* m = new mts_cm;
  m->num_pages = num_pages;
  m->page_size = page_size;
  m->chunk = host_chunk_tokens;
  m->free_pages.reserve(num_pages);
  for (int32_t p = num_pages - 1; p >= 0; --p) m->free_pages.push_back(p);   // page 0 is handed out first
  *out = m;
  return MTS_OK;
}

int32_t mts_cm_destroy(mts_cm* m) {
  if (!m) return MTS_OK;
  for (auto& kv : m->users) delete kv.second;
  delete m;
  return MTS_OK;
}

int32_t mts_cm_cached_length(mts_cm* m, int64_t user) {
  if (!m) return mts::set_error(MTS_ERR_INVALID_ARG, "manager is NULL");
  auto it = m->users.find(user);
  return it == m->users.end() ? 0 : it->second->total_len;
}

int32_t mts_cm_import_history(mts_cm* m, int64_t user, int32_t total_len) {
  if (!m) return mts::set_error(MTS_ERR_INVALID_ARG, "manager is NULL");
  if (total_len < 0) return mts::set_error(MTS_ERR_INVALID_ARG, "total_len is negative");
  if (m->users.count(user)) return mts::set_error(MTS_ERR_INVALID_ARG, "user %lld is already tracked", (long long)user);
  User* u = new User;
  u->id = user;
  u->total_len = u->host_len = total_len;      // all of it persisted in the host tier, none on the GPU
  m->users.emplace(user, u);
  return MTS_OK;
}

int32_t mts_cm_prepare_batch(mts_cm* m, const int64_t* users, const int32_t* new_tokens, int32_t batch,
                             int32_t* prefix_lens, int32_t* onload_lens, int32_t* page_indptr,
                             int32_t* page_indices, int64_t page_capacity) {
  if (!m) return mts::set_error(MTS_ERR_INVALID_ARG, "manager is NULL");
  if (batch < 0 || (batch > 0 && (!users || !new_tokens || !prefix_lens || !onload_lens || !page_indptr)))
    return mts::set_error(MTS_ERR_INVALID_ARG, "batch < 0 or an array is NULL");
  if (!m->batch.empty()) return mts::set_error(MTS_ERR_INVALID_ARG, "the previous batch was not committed");
  // pass 1: validate, mark the batch (its users are never victims), count the pages it needs
  int64_t need = 0;
  std::vector<User*> us(batch);
  std::vector<User*> created;                    // users first seen in this call: forgotten again if it fails
  auto unmark = [&](int upto) {
    for (int i = 0; i < upto; ++i) us[i]->batch_new = -1;
    for (User* c : created) {
      m->users.erase(c->id);
      delete c;
    }
  };
  for (int i = 0; i < batch; ++i) {
    if (new_tokens[i] < 0) { unmark(i); return mts::set_error(MTS_ERR_INVALID_ARG, "new_tokens[%d] is negative", i); }
    User*& u = us[i];
    auto it = m->users.find(users[i]);
    if (it == m->users.end()) {
      u = new User;
      u->id = users[i];
      m->users.emplace(users[i], u);
      created.push_back(u);
    } else {
      u = it->second;
    }
    if (u->batch_new >= 0) { unmark(i); return mts::set_error(MTS_ERR_INVALID_ARG, "user %lld appears twice in the batch", (long long)users[i]); }
    if ((int64_t)u->total_len + new_tokens[i] > 0x7fffffffll) { unmark(i); return mts::set_error(MTS_ERR_SHAPE, "sequence too long"); }
    u->batch_new = new_tokens[i];
    need += pages_for(u->total_len + new_tokens[i], m->page_size) - (int64_t)u->pages.size();
  }
  if (page_indices == nullptr && need > 0) { unmark(batch); return mts::set_error(MTS_ERR_INVALID_ARG, "page_indices is NULL"); }
  // pass 2: can the pool, after evicting every eligible victim, hold the batch?  (nothing changes on refusal)
  int64_t reclaimable = (int64_t)m->free_pages.size();
  for (User* v = m->tail; v && reclaimable < need; v = v->prev)
    if (!v->locked && v->batch_new < 0) reclaimable += (int64_t)v->pages.size();
  int64_t total_pages = 0;
  for (int i = 0; i < batch; ++i) total_pages += pages_for(us[i]->total_len + new_tokens[i], m->page_size);
  if (reclaimable < need || total_pages > page_capacity) {
    unmark(batch);
    if (reclaimable < need)
      return mts::set_error(MTS_ERR_BUSY, "the batch needs %lld more pages; %lld are free or reclaimable", (long long)need,
                            (long long)reclaimable);
    return mts::set_error(MTS_ERR_SHAPE, "page_indices holds %lld entries, the batch needs %lld", (long long)page_capacity,
                          (long long)total_pages);
  }
  // pass 3: reclaim from the LRU tail (skipping locked users and the batch itself), then allocate
  for (User* v = m->tail; v && (int64_t)m->free_pages.size() < need;) {
    User* prev = v->prev;
    if (!v->locked && v->batch_new < 0) m->evict(v);
    v = prev;
  }
  page_indptr[0] = 0;
  for (int i = 0; i < batch; ++i) {
    User* u = us[i];
    const bool cold = (u->total_len == 0);
    prefix_lens[i] = u->total_len;
    onload_lens[i] = u->on_gpu ? 0 : u->total_len;     // history held by the host tier only must come up
    if (cold) ++m->stats.cold_requests;
    else if (u->on_gpu) ++m->stats.gpu_hits;
    else ++m->stats.host_hits;
    const int32_t want = pages_for(u->total_len + new_tokens[i], m->page_size);
    while ((int32_t)u->pages.size() < want) {
      u->pages.push_back(m->free_pages.back());
      m->free_pages.pop_back();
    }
    memcpy(page_indices + page_indptr[i], u->pages.data(), sizeof(int32_t) * u->pages.size());
    page_indptr[i + 1] = page_indptr[i] + (int32_t)u->pages.size();
    m->batch.push_back(u);
  }
  return MTS_OK;
}

int32_t mts_cm_commit_batch(mts_cm* m) {
  if (!m) return mts::set_error(MTS_ERR_INVALID_ARG, "manager is NULL");
  for (User* u : m->batch) {          // in batch order: the last user of the batch ends up most recent
    u->total_len += u->batch_new;
    u->batch_new = -1;
    if (u->on_gpu) m->unlink(u);
    if (u->total_len > 0) {
      u->on_gpu = true;
      m->push_front(u);
    } else {                          // nothing cached: holds no pages (pages_for(0) == 0)
      u->on_gpu = false;
    }
  }
  m->batch.clear();
  return MTS_OK;
}

int32_t mts_cm_abort_batch(mts_cm* m) {
  if (!m) return mts::set_error(MTS_ERR_INVALID_ARG, "manager is NULL");
  for (User* u : m->batch) {
    // back to the pages the cached tokens need in the GPU tier; a user that is not there holds none
    const size_t keep = u->on_gpu ? (size_t)pages_for(u->total_len, m->page_size) : 0;
    while (u->pages.size() > keep) {
      m->free_pages.push_back(u->pages.back());
      u->pages.pop_back();
    }
    if (u->total_len == 0) --m->stats.cold_requests;
    else if (u->on_gpu) --m->stats.gpu_hits;
    else --m->stats.host_hits;
    u->batch_new = -1;
  }
  m->batch.clear();
  return MTS_OK;
}

int32_t mts_cm_offload_due(mts_cm* m, int64_t* users, int32_t* from_pos, int32_t* count, int32_t capacity) {
  if (!m) return mts::set_error(MTS_ERR_INVALID_ARG, "manager is NULL");
  if (capacity < 0 || (capacity > 0 && (!users || !from_pos || !count)))
    return mts::set_error(MTS_ERR_INVALID_ARG, "capacity < 0 or an array is NULL");
  int32_t n = 0;
  for (User* u = m->head; u && n < capacity; u = u->next) {   // most recent first
    const int32_t fresh = u->total_len - u->host_len;
    if (u->locked || u->batch_new >= 0 || fresh < m->chunk) continue;
    users[n] = u->id;
    from_pos[n] = u->host_len;
    count[n] = fresh / m->chunk * m->chunk;                    // whole host chunks only
    u->locked = true;
    ++n;
  }
  return n;
}

int32_t mts_cm_offload_done(mts_cm* m, int64_t user, int32_t persisted_len) {
  if (!m) return mts::set_error(MTS_ERR_INVALID_ARG, "manager is NULL");
  auto it = m->users.find(user);
  if (it == m->users.end()) return mts::set_error(MTS_ERR_INVALID_ARG, "unknown user %lld", (long long)user);
  User* u = it->second;
  if (persisted_len < u->host_len || persisted_len > u->total_len)
    return mts::set_error(MTS_ERR_SHAPE, "persisted_len %d outside [%d, %d]", persisted_len, u->host_len, u->total_len);
  u->host_len = persisted_len;
  u->locked = false;
  return MTS_OK;
}

int32_t mts_cm_set_locked(mts_cm* m, int64_t user, int32_t locked) {
  if (!m) return mts::set_error(MTS_ERR_INVALID_ARG, "manager is NULL");
  auto it = m->users.find(user);
  if (it == m->users.end()) return mts::set_error(MTS_ERR_INVALID_ARG, "unknown user %lld", (long long)user);
  it->second->locked = locked != 0;
  return MTS_OK;
}

int64_t mts_cm_take_evicted(mts_cm* m, int64_t* users, int64_t capacity) {
  if (!m) return mts::set_error(MTS_ERR_INVALID_ARG, "manager is NULL");
  if (capacity < 0 || (capacity > 0 && !users)) return mts::set_error(MTS_ERR_INVALID_ARG, "bad output array");
  const int64_t n = (int64_t)m->evicted.size() < capacity ? (int64_t)m->evicted.size() : capacity;
  for (int64_t i = 0; i < n; ++i) users[i] = m->evicted[i];
  m->evicted.erase(m->evicted.begin(), m->evicted.begin() + n);
  return n;
}

int32_t mts_cm_get_stats(mts_cm* m, mts_cm_stats* out) {
  if (!m || !out) return mts::set_error(MTS_ERR_INVALID_ARG, "manager / out is NULL");
  *out = m->stats;
  out->free_pages = (int64_t)m->free_pages.size();
  out->users_tracked = (int64_t)m->users.size();
  int64_t on = 0;
  for (User* u = m->head; u; u = u->next) ++on;
  out->users_on_gpu = on;
  return MTS_OK;
}

}  // extern "C"
