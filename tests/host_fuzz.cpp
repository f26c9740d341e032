// Host-only driver for the sanitizer test: random call sequences against the
// batcher, the quad-tree generator and the scheduler, built with
// -fsanitize=address,undefined by tests/test_host_sanitizers.py.  It checks
// only memory safety and status codes; values are checked elsewhere.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "alignedserve.h"

#define REQUIRE(x) do { if (!(x)) { std::fprintf(stderr, "REQUIRE failed: %s (line %d): %s\n", #x, __LINE__, as_last_error()); return 1; } } while (0)

int main() {
  std::mt19937 rng(12345);
  auto uni = [&](int lo, int hi) { return std::uniform_int_distribution<int>(lo, hi)(rng); };

  // --- sort-and-chunk batcher
  for (int trial = 0; trial < 300; ++trial) {
    const int n = uni(0, 500), B = uni(1, 70);
    std::vector<int32_t> lens(n), order(n + 1), offs(n / B + 3);
    for (auto& l : lens) l = trial % 3 ? uni(1, 100000) : uni(1, 3);
    int32_t nb = -1;
    REQUIRE(as_aligned_batch(lens.data(), n, B, order.data(), offs.data(), &nb) == AS_OK);
    REQUIRE(nb == (n + B - 1) / B && offs[nb] == n);
  }
  int32_t nb = 0, off1[2];
  REQUIRE(as_aligned_batch(nullptr, 3, 2, nullptr, off1, &nb) == AS_EINVAL);

  // --- quad-tree generator: inserts, removes, batches, interleaved
  for (int trial = 0; trial < 40; ++trial) {
    as_qtree* t = nullptr;
    REQUIRE(as_qtree_create(&t, trial % 2 ? 65536 : 4096, trial % 2 ? 16 : 4) == AS_OK);
    std::vector<int32_t> live;
    int32_t next_id = 0;
    std::vector<int32_t> ids(4096);
    for (int step = 0; step < 300; ++step) {
      const int op = uni(0, 3);
      if (op <= 1) {
        const int L = uni(1, 80000);
        REQUIRE(as_qtree_insert(t, next_id, L, (L > 65536 ? 65536 : L) / 16 + 1, step) == AS_OK);
        REQUIRE(as_qtree_insert(t, next_id, L, 1, step) == AS_EINVAL);  // duplicate id
        live.push_back(next_id++);
      } else if (op == 2 && !live.empty()) {
        const int k = uni(0, static_cast<int>(live.size()) - 1);
        REQUIRE(as_qtree_remove(t, live[k]) == AS_OK);
        REQUIRE(as_qtree_remove(t, live[k]) == AS_EINVAL);
        live.erase(live.begin() + k);
      } else {
        int32_t n = 0, which = 0;
        REQUIRE(as_qtree_next_batch(t, uni(1, 20000), uni(1, 50), step, uni(0, 1) ? -1.0 : 10.0, ids.data(),
                                    static_cast<int32_t>(ids.size()), &n, &which) == AS_OK);
        for (int i = 0; i < n; ++i)
          for (size_t j = 0; j < live.size(); ++j)
            if (live[j] == ids[i]) { live.erase(live.begin() + static_cast<long>(j)); break; }
        int64_t r = 0, b = 0;
        REQUIRE(as_qtree_size(t, &r, &b) == AS_OK && r == static_cast<int64_t>(live.size()));
      }
    }
    if (!live.empty()) {  // capacity too small: nothing may be removed
      int32_t n = 0;
      int64_t r0 = 0, r1 = 0, b = 0;
      as_qtree_size(t, &r0, &b);
      as_status st = as_qtree_next_batch(t, 1 << 30, 1, 0.0, -1.0, ids.data(), 0, &n, nullptr);
      as_qtree_size(t, &r1, &b);
      REQUIRE(st == AS_ERANGE && r0 == r1);
    }
    REQUIRE(as_qtree_destroy(t) == AS_OK);
  }

  // --- scheduler
  for (int trial = 0; trial < 60; ++trial) {
    as_sched* s = nullptr;
    const int max_batch = uni(1, 32);
    REQUIRE(as_sched_create(&s, uni(4, 400), 16, max_batch) == AS_OK);
    int32_t next_id = 0, origin = 0;
    for (int it = 0; it < 300; ++it) {
      if (uni(0, 2) == 0) {
        const int n = uni(1, 12);
        std::vector<int32_t> ids(n), L(n), R(n);
        for (int i = 0; i < n; ++i) { ids[i] = next_id++; L[i] = uni(1, 1500); R[i] = uni(1, 60); }
        REQUIRE(as_sched_push_candidate_batch(s, origin++, ids.data(), L.data(), R.data(), n) == AS_OK);
      }
      if (uni(0, 9) == 0) REQUIRE(as_sched_push_candidate_request(s, origin, next_id++, uni(1, 300), uni(1, 20)) == AS_OK);
      int64_t free_blocks = 0;
      int32_t nr = 0, nrc = 0, nbc = 0;
      REQUIRE(as_sched_state(s, &free_blocks, &nr, &nrc, &nbc) == AS_OK && free_blocks >= 0);
      const int cap = nr > max_batch ? nr : max_batch;
      std::vector<int32_t> c(cap), e(cap), a(cap);
      int32_t nc = 0, ne = 0, na = 0, which = 0;
      REQUIRE(as_sched_step(s, it > 0, c.data(), &nc, e.data(), &ne, a.data(), &na, cap, &which) == AS_OK);
      REQUIRE(nc <= cap && ne <= cap && na <= cap);
      REQUIRE(as_sched_step(s, 0, c.data(), &nc, e.data(), &ne, a.data(), &na, 0, &which) == AS_ERANGE);
    }
    REQUIRE(as_sched_destroy(s) == AS_OK);
  }
  std::puts("host fuzz ok");
  return 0;
}
