// Host side of include/synera_sched.h: the verification-aware scheduler (Section 4.5, Algorithm 1)
// as a request pool, two arrival queues, a page pool and a small state machine that hands out one
// engine call at a time.  No device code: this file forms the arrays synera_verify takes.
#include <chrono>
#include <cstdint>
#include <deque>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/synera.h"
#include "../../include/synera_sched.h"

namespace {

struct Request {
  int64_t id = 0;
  int64_t cached = 0;              // L
  std::vector<int32_t> pages;
  bool active = false;             // member of the algorithm's batch B
  bool completed = false;
  bool waiting = false;            // a submission of this request sits in a queue
  bool running = false;            // a submission of this request is being executed
  int32_t u = 0, k = 0;            // the waiting submission: prompt (u = n_prompt, k = 0) or verification
};

struct Work {                      // one submission in the iteration being executed
  Request* r;
  int32_t u, k;
  bool verify;
  int32_t done;                    // tokens already forwarded
  int32_t total() const { return u + k; }
};

struct Item {                      // one request's part of the outstanding engine call
  Work* w;
  int32_t n;                       // tokens forwarded
  bool final_verify;
};

struct Clock {
  explicit Clock(int64_t* acc) : acc_(acc), t0_(std::chrono::steady_clock::now()) {}
  ~Clock() { *acc_ += std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t0_).count(); }
  int64_t* acc_;
  std::chrono::steady_clock::time_point t0_;
};

}  // namespace

struct synera_sched {
  int32_t n_pages = 0, max_pages = 0, max_batch = 0, max_tokens = 0;
  std::vector<int32_t> free_pages;                   // stack
  std::unordered_map<int64_t, Request> pool;
  std::deque<int64_t> prefill_queue, verify_queue;
  std::vector<int64_t> B;                            // active batch, in the algorithm's order
  // iteration in progress
  std::vector<Work> batch;
  int32_t batch_kind = SYNERA_SCHED_IDLE;
  std::vector<Item> outstanding;                     // non-empty between next and commit
  synera_sched_stats stats{};

  static int32_t pages_for(int64_t tokens) { return (int32_t)((tokens + SYNERA_PAGE_SIZE - 1) / SYNERA_PAGE_SIZE); }
  int32_t page_limit() const { return max_pages < n_pages ? max_pages : n_pages; }

  // Gathers the head of `queue` into the batch while requests fit (batch, token and page limits); a
  // request that joins gets the pages for its whole new length.  No overtaking.
  void gather(std::deque<int64_t>& queue, bool verify) {
    int32_t tokens = 0;
    while (!queue.empty()) {
      Request& r = pool.at(queue.front());
      const int32_t total = r.u + r.k;
      const int32_t chunk = total < SYNERA_MAX_CHUNK ? total : SYNERA_MAX_CHUNK;
      if ((int32_t)batch.size() + 1 > max_batch) break;
      if (tokens + chunk > max_tokens) break;
      const int32_t need = pages_for(r.cached + total) - (int32_t)r.pages.size();
      if (need > (int32_t)free_pages.size()) break;
      for (int32_t i = 0; i < need; ++i) {
        r.pages.push_back(free_pages.back());
        free_pages.pop_back();
      }
      tokens += chunk;
      batch.push_back(Work{&r, r.u, r.k, verify, 0});
      r.waiting = false;
      r.running = true;
      r.u = r.k = 0;
      queue.pop_front();
    }
  }

  void remove_completed() {
    size_t keep = 0;
    for (size_t i = 0; i < B.size(); ++i) {
      auto it = pool.find(B[i]);
      if (it->second.completed) {
        for (int32_t p : it->second.pages) free_pages.push_back(p);
        pool.erase(it);
      } else {
        B[keep++] = B[i];
      }
    }
    B.resize(keep);
  }

  // End of an iteration: B <- B_prefill U B (prefill, and the iteration ends there), or
  // B <- B U B_verify followed by remove_completed.
  void close_iteration() {
    if (batch_kind == SYNERA_SCHED_PREFILL) {
      std::vector<int64_t> joined;
      joined.reserve(batch.size() + B.size());
      for (const Work& w : batch) {
        w.r->active = true;
        joined.push_back(w.r->id);
      }
      joined.insert(joined.end(), B.begin(), B.end());
      B.swap(joined);
    } else {
      remove_completed();          // verification requests are members of B already
    }
    batch.clear();
    batch_kind = SYNERA_SCHED_IDLE;
  }
};

extern "C" int32_t synera_sched_create(synera_sched** out, int32_t n_pages_in_pool, int32_t max_pages,
                                       int32_t max_batch, int32_t max_tokens) {
  if (!out) return SYNERA_EINVAL;
  *out = nullptr;
  if (n_pages_in_pool < 1 || max_pages < 1 || max_batch < 1 || max_tokens < 1) return SYNERA_EINVAL;
  synera_sched* s = new (std::nothrow) synera_sched;
  if (!s) return SYNERA_ENOMEM;
  s->n_pages = n_pages_in_pool;
  s->max_pages = max_pages;
  s->max_batch = max_batch;
  s->max_tokens = max_tokens;
  s->free_pages.resize(n_pages_in_pool);
  for (int32_t i = 0; i < n_pages_in_pool; ++i) s->free_pages[i] = n_pages_in_pool - 1 - i;   // page 0 on top
  *out = s;
  return SYNERA_OK;
}

extern "C" int32_t synera_sched_destroy(synera_sched* s) {
  delete s;
  return SYNERA_OK;
}

extern "C" int32_t synera_sched_submit_prefill(synera_sched* s, int64_t request_id, int32_t n_prompt) {
  if (!s || n_prompt < 1 || s->pool.count(request_id)) return SYNERA_EINVAL;
  if (synera_sched::pages_for(n_prompt) > s->page_limit()) return SYNERA_ENOSPC;
  Request& r = s->pool[request_id];
  r.id = request_id;
  r.u = n_prompt;
  r.k = 0;
  r.waiting = true;
  s->prefill_queue.push_back(request_id);
  return SYNERA_OK;
}

extern "C" int32_t synera_sched_submit_verify(synera_sched* s, int64_t request_id, int32_t n_uncached,
                                              int32_t n_draft) {
  if (!s || n_uncached < 0 || n_draft < 1 || n_draft > SYNERA_MAX_CHUNK) return SYNERA_EINVAL;
  auto it = s->pool.find(request_id);
  if (it == s->pool.end()) return SYNERA_EINVAL;
  Request& r = it->second;
  if (!r.active || r.completed || r.waiting || r.running) return SYNERA_EINVAL;
  if (synera_sched::pages_for(r.cached + n_uncached + n_draft) > s->page_limit()) return SYNERA_ENOSPC;
  r.u = n_uncached;
  r.k = n_draft;
  r.waiting = true;
  s->verify_queue.push_back(request_id);
  return SYNERA_OK;
}

extern "C" int32_t synera_sched_finish(synera_sched* s, int64_t request_id) {
  if (!s) return SYNERA_EINVAL;
  auto it = s->pool.find(request_id);
  if (it == s->pool.end() || !it->second.active || it->second.waiting || it->second.running) return SYNERA_EINVAL;
  it->second.completed = true;
  return SYNERA_OK;
}

extern "C" int32_t synera_sched_next(synera_sched* s, int32_t* kind, int32_t* B, int64_t* h_request_id,
                                     int32_t* h_ctx_len, int32_t* h_n_uncached, int32_t* h_n_draft,
                                     int32_t* h_token_begin, int32_t* h_final_verify, int32_t* h_block_table) {
  if (!s || !kind || !B || !h_request_id || !h_ctx_len || !h_n_uncached || !h_n_draft || !h_token_begin ||
      !h_final_verify || !h_block_table)
    return SYNERA_EINVAL;
  if (!s->outstanding.empty()) return SYNERA_EINVAL;
  Clock clock(&s->stats.host_ns);

  if (s->batch.empty()) {          // a new iteration: prefills first and alone, else the verifications
    s->gather(s->prefill_queue, false);
    if (!s->batch.empty()) {
      s->batch_kind = SYNERA_SCHED_PREFILL;
      ++s->stats.iterations_prefill;
    } else {
      s->gather(s->verify_queue, true);
      if (!s->batch.empty()) {
        s->batch_kind = SYNERA_SCHED_VERIFY;
        ++s->stats.iterations_verify;
      } else {
        ++s->stats.iterations_idle;
        s->remove_completed();
        *kind = SYNERA_SCHED_IDLE;
        *B = 0;
        return SYNERA_OK;
      }
    }
  }

  int32_t b = 0;
  for (Work& w : s->batch) {
    const int32_t remaining = w.total() - w.done;
    if (remaining <= 0) continue;
    int32_t n, k;
    bool final_verify;
    if (w.verify && remaining <= SYNERA_MAX_CHUNK) {   // the rest of the uncached tokens and all drafts
      n = remaining;
      k = w.k;
      final_verify = true;
    } else {                                           // tokens forwarded for their KV only
      const int32_t kv_only = remaining - w.k;
      n = kv_only < SYNERA_MAX_CHUNK ? kv_only : SYNERA_MAX_CHUNK;
      k = 1;
      final_verify = false;
    }
    const Request& r = *w.r;
    h_request_id[b] = r.id;
    h_ctx_len[b] = (int32_t)(r.cached + w.done);
    h_n_uncached[b] = n - k;
    h_n_draft[b] = k;
    h_token_begin[b] = w.done;
    h_final_verify[b] = final_verify ? 1 : 0;
    int32_t* row = h_block_table + (size_t)b * s->max_pages;
    const int32_t have = (int32_t)r.pages.size();
    for (int32_t p = 0; p < s->max_pages; ++p) row[p] = p < have ? r.pages[p] : -1;
    s->outstanding.push_back(Item{&w, n, final_verify});
    s->stats.tokens_forwarded += n;
    ++b;
  }
  ++s->stats.engine_calls;
  *kind = s->batch_kind;
  *B = b;
  return SYNERA_OK;
}

extern "C" int32_t synera_sched_commit(synera_sched* s, const int32_t* h_accept_len) {
  if (!s || s->outstanding.empty()) return SYNERA_EINVAL;
  Clock clock(&s->stats.host_ns);
  for (size_t i = 0; i < s->outstanding.size(); ++i) {
    const Item& it = s->outstanding[i];
    if (it.final_verify && (!h_accept_len || h_accept_len[i] < 0 || h_accept_len[i] > it.w->k)) return SYNERA_EINVAL;
  }
  for (size_t i = 0; i < s->outstanding.size(); ++i) {
    const Item& it = s->outstanding[i];
    Work& w = *it.w;
    w.done += it.n;
    if (w.done == w.total()) {                         // submission consumed
      // after a verification L + u + a: the rejected drafts' entries are dead
      w.r->cached += w.u + (it.final_verify ? h_accept_len[i] : 0);
      w.r->running = false;
    }
  }
  s->outstanding.clear();
  bool all_done = true;
  for (const Work& w : s->batch) all_done = all_done && w.done == w.total();
  if (all_done) s->close_iteration();
  return SYNERA_OK;
}

extern "C" int64_t synera_sched_cached_len(const synera_sched* s, int64_t request_id) {
  if (!s) return -1;
  auto it = s->pool.find(request_id);
  return it == s->pool.end() ? -1 : it->second.cached;
}

extern "C" int32_t synera_sched_get_stats(const synera_sched* s, synera_sched_stats* out) {
  if (!s || !out) return SYNERA_EINVAL;
  *out = s->stats;
  out->active_requests = (int32_t)s->B.size();
  out->waiting_prefill = (int32_t)s->prefill_queue.size();
  out->waiting_verify = (int32_t)s->verify_queue.size();
  out->free_pages = (int32_t)s->free_pages.size();
  return SYNERA_OK;
}
