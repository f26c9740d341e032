// Quad-tree + Density First Search batch generator (host only).
//
// Paper Section 3.3, Algorithm 1: in-flight requests sit in the leaves of a
// quad-tree keyed on prefix length; every internal node carries the request
// and block counters of its sub-tree.  One batch is produced by a search from
// the root: a sub-tree that fits the block budget B_max and holds at least
// K_min requests is taken whole (case 1); one that exceeds B_max sends the
// search into its child with the largest request counter (case 2); one that
// fits but is too small is widened with requests of its nearest siblings
// (case 3; left siblings if present, else right ones, nearest request first,
// stopping at the first that does not fit, at most K_min - |batch| of them).
// Section 4.1: range [1, 65536] with longer prefixes clamped; Section 3.5:
// per-node time stamps let a sub-tree that has not produced a batch for too
// long be served first.
//
// The tree is implicit: level l is an array of 4^l counters, node i of level
// l covers lengths [1 + i*w_l, (i+1)*w_l] with w_l = max_len / 4^l, so a
// node's children are 4i..4i+3 and counters of a level fit consecutive cache
// lines.  Leaves keep their requests sorted by (length, id).
#include <algorithm>
#include <cstdint>
#include <memory>
#include <unordered_map>
#include <vector>

#include "common.h"

namespace {

struct Req {
  int32_t len;
  int32_t id;
  int32_t blocks;
  bool operator<(const Req& o) const { return len != o.len ? len < o.len : id < o.id; }
};

}  // namespace

struct as_qtree {
  int32_t max_len;
  int32_t leaf_width;
  int levels;                                   // leaf level index (root = 0)
  std::vector<std::vector<int64_t>> req_count;  // [level][node]
  std::vector<std::vector<int64_t>> blk_count;
  std::vector<std::vector<double>> stamp;
  std::vector<std::vector<Req>> leaves;
  std::unordered_map<int32_t, Req> by_id;
  int32_t last_case;

  int64_t width(int level) const { return static_cast<int64_t>(max_len) >> (2 * level); }
  int64_t node_of(int level, int32_t key) const { return (key - 1) / width(level); }

  void collect(int level, int64_t idx, std::vector<Req>* out) const {
    const int64_t span = int64_t{1} << (2 * (levels - level));
    for (int64_t l = idx * span; l < (idx + 1) * span; ++l)
      out->insert(out->end(), leaves[l].begin(), leaves[l].end());
  }

  void erase(const Req& r) {
    auto& leaf = leaves[node_of(levels, r.len)];
    leaf.erase(std::lower_bound(leaf.begin(), leaf.end(), r));
    for (int l = 0; l <= levels; ++l) {
      const int64_t i = node_of(l, r.len);
      req_count[l][i] -= 1;
      blk_count[l][i] -= r.blocks;
    }
    by_id.erase(r.id);
  }
};

extern "C" as_status as_qtree_create(as_qtree** out, int32_t max_len, int32_t leaf_width) {
  if (!out) return als::fail(AS_EINVAL, "as_qtree_create: out is null");
  if (leaf_width < 1 || max_len < leaf_width)
    return als::fail(AS_EINVAL, "as_qtree_create: need 1 <= leaf_width <= max_len");
  int levels = 0;
  int64_t span = max_len;
  while (span > leaf_width) {
    if (span % 4) return als::fail(AS_EINVAL, "as_qtree_create: max_len / leaf_width must be a power of four");
    span /= 4;
    ++levels;
  }
  if (span != leaf_width || levels > 12)
    return als::fail(AS_EINVAL, "as_qtree_create: max_len / leaf_width must be a power of four (at most 4^12)");
  ALS_TRY
  std::unique_ptr<as_qtree> t(new as_qtree());
  t->max_len = max_len;
  t->leaf_width = leaf_width;
  t->levels = levels;
  t->last_case = 0;
  for (int l = 0; l <= levels; ++l) {
    const size_t n = size_t{1} << (2 * l);
    t->req_count.emplace_back(n, 0);
    t->blk_count.emplace_back(n, 0);
    t->stamp.emplace_back(n, 0.0);
  }
  t->leaves.resize(size_t{1} << (2 * levels));
  *out = t.release();
  ALS_CATCH("as_qtree_create")
  return AS_OK;
}

extern "C" as_status as_qtree_destroy(as_qtree* t) {
  if (!t) return als::fail(AS_EINVAL, "as_qtree_destroy: tree is null");
  delete t;
  return AS_OK;
}

extern "C" as_status as_qtree_insert(as_qtree* t, int32_t request_id, int32_t prefix_len, int32_t blocks,
                                     double now) {
  if (!t) return als::fail(AS_EINVAL, "as_qtree_insert: tree is null");
  if (prefix_len < 1 || blocks < 1)
    return als::fail(AS_EINVAL, "as_qtree_insert: prefix_len %d and blocks %d must be positive", prefix_len, blocks);
  if (t->by_id.count(request_id))
    return als::fail(AS_EINVAL, "as_qtree_insert: request %d is already in the tree", request_id);
  const Req r{std::min(prefix_len, t->max_len), request_id, blocks};
  // the two steps that allocate come first; the counters change only once both have succeeded
  ALS_TRY
  t->by_id.emplace(request_id, r);
  try {
    auto& leaf = t->leaves[t->node_of(t->levels, r.len)];
    leaf.insert(std::lower_bound(leaf.begin(), leaf.end(), r), r);
  } catch (...) {
    t->by_id.erase(request_id);
    throw;
  }
  ALS_CATCH("as_qtree_insert")
  for (int l = 0; l <= t->levels; ++l) {
    const int64_t i = t->node_of(l, r.len);
    if (t->req_count[l][i] == 0) t->stamp[l][i] = now;  // age counts from the first arrival
    t->req_count[l][i] += 1;
    t->blk_count[l][i] += blocks;
  }
  return AS_OK;
}

extern "C" as_status as_qtree_remove(as_qtree* t, int32_t request_id) {
  if (!t) return als::fail(AS_EINVAL, "as_qtree_remove: tree is null");
  auto it = t->by_id.find(request_id);
  if (it == t->by_id.end()) return als::fail(AS_EINVAL, "as_qtree_remove: request %d is not in the tree", request_id);
  const Req r = it->second;
  t->erase(r);
  return AS_OK;
}

extern "C" as_status as_qtree_size(const as_qtree* t, int64_t* requests, int64_t* blocks) {
  if (!t || !requests || !blocks) return als::fail(AS_EINVAL, "as_qtree_size: null argument");
  *requests = t->req_count[0][0];
  *blocks = t->blk_count[0][0];
  return AS_OK;
}

extern "C" as_status as_qtree_next_batch(as_qtree* t, int64_t b_max, int32_t k_min, double now,
                                         double starve_after, int32_t* out_ids, int32_t capacity,
                                         int32_t* out_n, int32_t* out_case) {
  if (!t || !out_n) return als::fail(AS_EINVAL, "as_qtree_next_batch: null argument");
  if (b_max < 1 || k_min < 1) return als::fail(AS_EINVAL, "as_qtree_next_batch: b_max and k_min must be positive");
  *out_n = 0;
  if (t->req_count[0][0] == 0) return AS_OK;
  if (!out_ids) return als::fail(AS_EINVAL, "as_qtree_next_batch: out_ids is null");

  // starting node: the root, or the starving internal node with the largest age
  int level = 0;
  int64_t idx = 0;
  if (starve_after >= 0.0) {
    double best_age = 0.0;
    bool found = false;
    for (int l = 0; l < t->levels; ++l) {
      for (int64_t i = 0; i < static_cast<int64_t>(t->req_count[l].size()); ++i) {
        if (t->req_count[l][i] == 0) continue;
        const double age = now - t->stamp[l][i];
        if (age <= starve_after) continue;
        // largest age, then deeper, then leftmost: levels and indices ascend, so
        // a later candidate wins only if older, or as old and deeper
        if (!found || age > best_age || (age == best_age && l > level)) {
          found = true; best_age = age; level = l; idx = i;
        }
      }
    }
  }

  // the batch is gathered into local storage (the only part that allocates); the tree changes after it
  std::vector<Req> batch;
  int which = 0;
  ALS_TRY
  for (;;) {
    const int64_t used = t->blk_count[level][idx];
    const int64_t count = t->req_count[level][idx];
    if (used <= b_max && count >= k_min) {  // case 1
      t->collect(level, idx, &batch);
      which = 1;
      break;
    }
    if (used > b_max) {  // case 2
      if (level == t->levels) {
        int64_t acc = 0;
        for (const Req& r : t->leaves[idx]) {  // the first request is always taken
          if (!batch.empty() && acc + r.blocks > b_max) break;
          batch.push_back(r);
          acc += r.blocks;
        }
        which = 2;
        break;
      }
      int64_t best = 4 * idx;
      for (int64_t c = 4 * idx + 1; c < 4 * idx + 4; ++c)
        if (t->req_count[level + 1][c] > t->req_count[level + 1][best]) best = c;  // leftmost on ties
      level += 1;
      idx = best;
      continue;
    }
    // case 3
    t->collect(level, idx, &batch);
    const int64_t b_left = b_max - used;
    const int64_t k_left = k_min - count;
    if (level > 0) {
      const int64_t first = idx & ~int64_t{3};
      std::vector<Req> addition, tmp;
      int64_t acc = 0;
      bool stop = false;
      if (idx > first) {  // left siblings, nearest first, longest request first
        for (int64_t s = idx - 1; s >= first && !stop; --s) {
          tmp.clear();
          t->collect(level, s, &tmp);
          for (auto it = tmp.rbegin(); it != tmp.rend(); ++it) {
            if (it->blocks + acc <= b_left) { addition.push_back(*it); acc += it->blocks; }
            else { stop = true; break; }
          }
        }
      } else {            // right siblings, nearest first, shortest request first
        for (int64_t s = idx + 1; s < first + 4 && !stop; ++s) {
          tmp.clear();
          t->collect(level, s, &tmp);
          for (const Req& r : tmp) {
            if (r.blocks + acc <= b_left) { addition.push_back(r); acc += r.blocks; }
            else { stop = true; break; }
          }
        }
      }
      const int64_t keep = std::min<int64_t>(k_left, static_cast<int64_t>(addition.size()));
      batch.insert(batch.end(), addition.begin(), addition.begin() + keep);
    }
    which = 3;
    break;
  }
  ALS_CATCH("as_qtree_next_batch")

  if (static_cast<int64_t>(batch.size()) > capacity)
    return als::fail(AS_ERANGE, "as_qtree_next_batch: batch of %zu requests exceeds capacity %d", batch.size(), capacity);
  // stamp the node where the search ended and its ancestors
  for (int l = level; l >= 0; --l) t->stamp[l][idx >> (2 * (level - l))] = now;
  for (size_t i = 0; i < batch.size(); ++i) out_ids[i] = batch[i].id;
  for (const Req& r : batch) t->erase(r);
  *out_n = static_cast<int32_t>(batch.size());
  if (out_case) *out_case = which;
  t->last_case = which;
  return AS_OK;
}

extern "C" as_status as_dfs_batches(const int32_t* kv_lens, const int32_t* blocks, int32_t n, int64_t b_max,
                                    int32_t k_min, int32_t max_len, int32_t leaf_width, int32_t* order,
                                    int32_t* batch_offsets, int32_t* num_batches) {
  if (n < 0) return als::fail(AS_EINVAL, "as_dfs_batches: n is negative");
  if (!batch_offsets || !num_batches || (n > 0 && (!kv_lens || !blocks || !order)))
    return als::fail(AS_EINVAL, "as_dfs_batches: null argument");
  as_qtree* t = nullptr;
  as_status st = as_qtree_create(&t, max_len, leaf_width);
  if (st != AS_OK) return st;
  for (int32_t i = 0; i < n && st == AS_OK; ++i) st = as_qtree_insert(t, i, kv_lens[i], blocks[i], 0.0);
  int32_t nb = 0, done = 0;
  batch_offsets[0] = 0;
  while (st == AS_OK && done < n) {
    int32_t got = 0;
    st = as_qtree_next_batch(t, b_max, k_min, 0.0, -1.0, order + done, n - done, &got, nullptr);
    if (st != AS_OK) break;
    done += got;
    batch_offsets[++nb] = done;
  }
  as_qtree_destroy(t);
  if (st != AS_OK) return st;
  *num_batches = nb;
  return AS_OK;
}
