// Batch-level scheduling policy (host only).
//
// Paper Section 3.4, Algorithm 2, run after every decode iteration: release
// the HBM of completed requests; if the next iteration does not fit, evict a
// victim to the candidate-requests buffer (the longest request, or -- while
// two original batches coexist -- the longest request of the old batch);
// otherwise admit from the candidate-requests buffer if it holds anything,
// else from the candidate-batch buffer (which starts a batch switch).
//
// Block accounting: a request holds ceil(kv_len / block_size) blocks; the next
// iteration needs one fresh block per running request whose kv_len is a
// multiple of block_size.  Eviction repeats until the next iteration fits;
// admission takes requests in buffer order while the batch is below
// max_batch and the request's blocks plus next-iteration growth fit, and
// stops at the first that does not.
#include <algorithm>
#include <cstdint>
#include <memory>
#include <vector>

#include "common.h"

namespace {
struct SReq {
  int32_t id, kv_len, remaining, origin;
};

// First-in first-out buffer over one vector.  Unlike std::deque it can reserve
// room ahead of time, so that a scheduling pass does all its allocation before
// it changes anything and cannot fail half way.
struct Fifo {
  std::vector<SReq> v;
  size_t head = 0;
  bool empty() const { return head == v.size(); }
  size_t size() const { return v.size() - head; }
  const SReq& front() const { return v[head]; }
  void pop_front() {
    if (++head == v.size()) { v.clear(); head = 0; }
  }
  void push_back(const SReq& r) { v.push_back(r); }
  void pop_back() { v.pop_back(); }
  // room for `extra` more entries without a further allocation (may throw; changes no content)
  void reserve_extra(size_t extra) {
    if (head > 0 && v.size() + extra > v.capacity()) {
      v.erase(v.begin(), v.begin() + static_cast<std::ptrdiff_t>(head));  // moves only, no allocation
      head = 0;
    }
    v.reserve(v.size() + extra);
  }
};
}  // namespace

struct as_sched {
  int64_t total, free_;
  int32_t bs, max_batch;
  std::vector<SReq> running;
  Fifo r_cand, b_cand;

  int64_t blocks(const SReq& r) const { return (static_cast<int64_t>(r.kv_len) + bs - 1) / bs; }
  int64_t growth() const {
    int64_t g = 0;
    for (const SReq& r : running) g += (r.kv_len % bs == 0);
    return g;
  }
};

extern "C" as_status as_sched_create(as_sched** out, int64_t total_blocks, int32_t block_size,
                                     int32_t max_batch) {
  if (!out) return als::fail(AS_EINVAL, "as_sched_create: out is null");
  if (total_blocks < 1 || block_size < 1 || max_batch < 1)
    return als::fail(AS_EINVAL, "as_sched_create: total_blocks, block_size and max_batch must be positive");
  ALS_TRY
  std::unique_ptr<as_sched> s(new as_sched());
  s->total = s->free_ = total_blocks;
  s->bs = block_size;
  s->max_batch = max_batch;
  s->running.reserve(static_cast<size_t>(max_batch));
  *out = s.release();
  ALS_CATCH("as_sched_create")
  return AS_OK;
}

extern "C" as_status as_sched_destroy(as_sched* s) {
  if (!s) return als::fail(AS_EINVAL, "as_sched_destroy: scheduler is null");
  delete s;
  return AS_OK;
}

extern "C" as_status as_sched_push_candidate_batch(as_sched* s, int32_t origin, const int32_t* ids,
                                                   const int32_t* kv_lens, const int32_t* remaining,
                                                   int32_t n) {
  if (!s || n < 0 || (n > 0 && (!ids || !kv_lens || !remaining)))
    return als::fail(AS_EINVAL, "as_sched_push_candidate_batch: null argument or negative n");
  for (int32_t i = 0; i < n; ++i)
    if (kv_lens[i] < 1 || remaining[i] < 1)
      return als::fail(AS_EINVAL, "as_sched_push_candidate_batch: request %d has kv_len %d, remaining %d", ids[i],
                       kv_lens[i], remaining[i]);
  ALS_TRY
  s->b_cand.reserve_extra(static_cast<size_t>(n));   // all or nothing
  ALS_CATCH("as_sched_push_candidate_batch")
  for (int32_t i = 0; i < n; ++i) s->b_cand.push_back(SReq{ids[i], kv_lens[i], remaining[i], origin});
  return AS_OK;
}

extern "C" as_status as_sched_push_candidate_request(as_sched* s, int32_t origin, int32_t id, int32_t kv_len,
                                                     int32_t remaining) {
  if (!s) return als::fail(AS_EINVAL, "as_sched_push_candidate_request: scheduler is null");
  if (kv_len < 1 || remaining < 1)
    return als::fail(AS_EINVAL, "as_sched_push_candidate_request: kv_len and remaining must be positive");
  ALS_TRY
  s->r_cand.reserve_extra(1);
  ALS_CATCH("as_sched_push_candidate_request")
  s->r_cand.push_back(SReq{id, kv_len, remaining, origin});
  return AS_OK;
}

extern "C" as_status as_sched_step(as_sched* s, int32_t advance, int32_t* completed, int32_t* n_completed,
                                   int32_t* evicted, int32_t* n_evicted, int32_t* admitted,
                                   int32_t* n_admitted, int32_t capacity, int32_t* which_case) {
  if (!s || !completed || !n_completed || !evicted || !n_evicted || !admitted || !n_admitted || !which_case)
    return als::fail(AS_EINVAL, "as_sched_step: null argument");
  // every list is bounded by the running batch before the step plus what can be admitted
  if (capacity < static_cast<int32_t>(s->running.size()) || capacity < s->max_batch)
    return als::fail(AS_ERANGE, "as_sched_step: capacity %d is below the running batch / max_batch", capacity);
  // every victim of this pass fits the candidate-requests buffer and every admission fits the running
  // batch without a further allocation: past this point nothing can fail
  ALS_TRY
  s->r_cand.reserve_extra(s->running.size());
  s->running.reserve(std::max(s->running.size(), static_cast<size_t>(s->max_batch)));
  ALS_CATCH("as_sched_step")
  if (advance) {
    for (SReq& r : s->running) {
      const int64_t before = s->blocks(r);
      r.kv_len += 1;
      r.remaining -= 1;
      s->free_ -= s->blocks(r) - before;
    }
  }
  int32_t nc = 0, ne = 0, na = 0;
  {
    size_t keep = 0;
    for (size_t i = 0; i < s->running.size(); ++i) {
      const SReq r = s->running[i];
      if (r.remaining <= 0) {
        s->free_ += s->blocks(r);
        completed[nc++] = r.id;
      } else {
        s->running[keep++] = r;
      }
    }
    s->running.resize(keep);
  }
  int32_t which = 0;
  if (s->growth() > s->free_) {  // case 3
    which = 3;
    while (!s->running.empty() && s->growth() > s->free_) {
      int32_t lo = s->running[0].origin, hi = lo;
      for (const SReq& r : s->running) { lo = r.origin < lo ? r.origin : lo; hi = r.origin > hi ? r.origin : hi; }
      const bool switching = lo != hi;
      size_t v = s->running.size();
      for (size_t i = 0; i < s->running.size(); ++i) {
        if (switching && s->running[i].origin != lo) continue;
        if (v == s->running.size() || s->running[i].kv_len > s->running[v].kv_len) v = i;
      }
      const SReq victim = s->running[v];
      s->running.erase(s->running.begin() + static_cast<std::ptrdiff_t>(v));
      s->free_ += s->blocks(victim);
      s->r_cand.push_back(victim);
      evicted[ne++] = victim.id;
    }
  } else {
    Fifo* src = nullptr;
    if (!s->r_cand.empty()) { src = &s->r_cand; which = 1; }
    else if (!s->b_cand.empty()) { src = &s->b_cand; which = 2; }
    if (src) {
      while (!src->empty() && static_cast<int32_t>(s->running.size()) < s->max_batch) {
        const SReq r = src->front();
        const int64_t need = s->blocks(r) + s->growth() + (r.kv_len % s->bs == 0);
        if (need > s->free_) break;
        src->pop_front();
        s->free_ -= s->blocks(r);
        s->running.push_back(r);
        admitted[na++] = r.id;
      }
      if (na == 0) which = 0;
    }
  }
  *n_completed = nc;
  *n_evicted = ne;
  *n_admitted = na;
  *which_case = which;
  return AS_OK;
}

extern "C" as_status as_sched_state(const as_sched* s, int64_t* free_blocks, int32_t* n_running,
                                    int32_t* n_candidate_requests, int32_t* n_candidate_batch) {
  if (!s || !free_blocks || !n_running || !n_candidate_requests || !n_candidate_batch)
    return als::fail(AS_EINVAL, "as_sched_state: null argument");
  *free_blocks = s->free_;
  *n_running = static_cast<int32_t>(s->running.size());
  *n_candidate_requests = static_cast<int32_t>(s->r_cand.size());
  *n_candidate_batch = static_cast<int32_t>(s->b_cand.size());
  return AS_OK;
}

extern "C" as_status as_sched_running(const as_sched* s, int32_t* ids, int32_t* kv_lens, int32_t* origins,
                                      int32_t capacity, int32_t* n) {
  if (!s || !n) return als::fail(AS_EINVAL, "as_sched_running: null argument");
  const int32_t m = static_cast<int32_t>(s->running.size());
  if (m > capacity) return als::fail(AS_ERANGE, "as_sched_running: %d running requests exceed capacity %d", m, capacity);
  for (int32_t i = 0; i < m; ++i) {
    if (ids) ids[i] = s->running[i].id;
    if (kv_lens) kv_lens[i] = s->running[i].kv_len;
    if (origins) origins[i] = s->running[i].origin;
  }
  *n = m;
  return AS_OK;
}
