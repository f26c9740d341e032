// Host-only driver for the sanitizer test: random call sequences against the
// batcher, the quad-tree generator and the scheduler, built with
// -fsanitize=address,undefined by tests/test_host_sanitizers.py.  It checks
// only memory safety and status codes; values are checked elsewhere.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <new>
#include <random>
#include <vector>

#include "alignedserve.h"

// Allocation-failure injection: while armed, the k-th allocation from now
// throws std::bad_alloc.  Armed only around a single library call.
static long g_fail_in = -1;
void* operator new(std::size_t n) {
  if (g_fail_in >= 0 && g_fail_in-- == 0) throw std::bad_alloc();
  if (void* p = std::malloc(n ? n : 1)) return p;
  throw std::bad_alloc();
}
void* operator new(std::size_t n, const std::nothrow_t&) noexcept {
  if (g_fail_in >= 0 && g_fail_in-- == 0) return nullptr;
  return std::malloc(n ? n : 1);
}
void operator delete(void* p) noexcept { std::free(p); }
void operator delete(void* p, std::size_t) noexcept { std::free(p); }

// Runs `call` with the k-th allocation failing, k = 0, 1, 2, ...: every outcome must be AS_OK or
// AS_ENOMEM (no exception may escape), `unchanged` must hold after an AS_ENOMEM, and the first
// AS_OK ends the sweep.  Returns the number of injected failures that surfaced as AS_ENOMEM.
template <typename Call, typename Check>
static int sweep_failures(Call call, Check unchanged, bool* ok) {
  int seen = 0;
  for (long k = 0; k < 100000; k += 1 + k / 8) {   // every early allocation, then a thinning sample of later ones
    g_fail_in = k;
    as_status st;
    try {
      st = call();
    } catch (...) {
      g_fail_in = -1;
      std::fprintf(stderr, "an exception crossed the C ABI (allocation %ld)\n", k);
      *ok = false;
      return seen;
    }
    const bool fired = g_fail_in < 0;
    g_fail_in = -1;
    if (st == AS_OK) { *ok = true; return seen; }
    if (st != AS_ENOMEM || !fired || !unchanged()) {
      std::fprintf(stderr, "allocation %ld failing: status %d, fired %d: %s\n", k, int(st), int(fired), as_last_error());
      *ok = false;
      return seen;
    }
    ++seen;
  }
  *ok = false;
  return seen;
}

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
  // --- allocation failures: AS_ENOMEM, the object unchanged, nothing thrown across the ABI
  {
    bool ok = false;
    int enomem = 0;
    auto always = [] { return true; };
    // batch formation
    std::vector<int32_t> lens(300), order(300), offs(40);
    for (int i = 0; i < 300; ++i) lens[i] = 1 + (i * 7919) % 5000;
    int32_t nbat = 0;
    enomem += sweep_failures([&] { return as_aligned_batch(lens.data(), 300, 8, order.data(), offs.data(), &nbat); }, always, &ok);
    REQUIRE(ok && nbat == 38);
    // quad-tree: create, insert, search
    as_qtree* t = nullptr;
    enomem += sweep_failures([&] { return as_qtree_create(&t, 65536, 16); }, [&] { return t == nullptr; }, &ok);
    REQUIRE(ok && t != nullptr);
    for (int i = 0; i < 200; ++i) {
      int64_t r0 = 0, b0 = 0;
      REQUIRE(as_qtree_size(t, &r0, &b0) == AS_OK);
      auto same = [&] { int64_t r = 0, b = 0; return as_qtree_size(t, &r, &b) == AS_OK && r == r0 && b == b0; };
      const int L = 1 + (i * 104729) % 60000;
      enomem += sweep_failures([&] { return as_qtree_insert(t, i, L, L / 16 + 1, 0.0); }, same, &ok);
      REQUIRE(ok);
      // a failed insert must not have left the id behind: the same id can still be removed exactly once
      int64_t r1 = 0, b1 = 0;
      REQUIRE(as_qtree_size(t, &r1, &b1) == AS_OK && r1 == r0 + 1 && b1 == b0 + L / 16 + 1);
    }
    std::vector<int32_t> ids(256);
    for (int round = 0; round < 6; ++round) {
      int64_t r0 = 0, b0 = 0;
      REQUIRE(as_qtree_size(t, &r0, &b0) == AS_OK);
      auto same = [&] { int64_t r = 0, b = 0; return as_qtree_size(t, &r, &b) == AS_OK && r == r0 && b == b0; };
      int32_t got = 0, which = 0;
      enomem += sweep_failures([&] { return as_qtree_next_batch(t, 20000, 36, 1.0, -1.0, ids.data(), 256, &got, &which); }, same, &ok);
      REQUIRE(ok);
      int64_t r1 = 0, b1 = 0;
      REQUIRE(as_qtree_size(t, &r1, &b1) == AS_OK && r1 == r0 - got);
    }
    REQUIRE(as_qtree_destroy(t) == AS_OK);
    std::vector<int32_t> blocks(300);
    for (int i = 0; i < 300; ++i) blocks[i] = lens[i] / 16 + 1;
    std::vector<int32_t> offs2(301);
    enomem += sweep_failures([&] { return as_dfs_batches(lens.data(), blocks.data(), 300, 4000, 36, 65536, 16, order.data(), offs2.data(), &nbat); }, always, &ok);
    REQUIRE(ok && offs2[nbat] == 300);
    // scheduler: create, push, step
    as_sched* sc = nullptr;
    enomem += sweep_failures([&] { return as_sched_create(&sc, 300, 16, 8); }, [&] { return sc == nullptr; }, &ok);
    REQUIRE(ok && sc != nullptr);
    int32_t next = 0;
    for (int it = 0; it < 120; ++it) {
      int64_t f0 = 0; int32_t a0 = 0, rc0 = 0, bc0 = 0;
      REQUIRE(as_sched_state(sc, &f0, &a0, &rc0, &bc0) == AS_OK);
      auto same = [&] { int64_t f = 0; int32_t a = 0, rc = 0, bc = 0;
                        return as_sched_state(sc, &f, &a, &rc, &bc) == AS_OK && f == f0 && a == a0 && rc == rc0 && bc == bc0; };
      if (bc0 == 0) {
        int32_t bid[5], bl[5], br[5];
        for (int i = 0; i < 5; ++i) { bid[i] = next++; bl[i] = 1 + (next * 37) % 700; br[i] = 1 + next % 30; }
        enomem += sweep_failures([&] { return as_sched_push_candidate_batch(sc, it, bid, bl, br, 5); }, same, &ok);
        REQUIRE(ok);
        REQUIRE(as_sched_state(sc, &f0, &a0, &rc0, &bc0) == AS_OK && bc0 == 5);
      }
      if (it % 17 == 3) {
        enomem += sweep_failures([&] { return as_sched_push_candidate_request(sc, it, next++, 40, 5); }, same, &ok);
        REQUIRE(ok);
        REQUIRE(as_sched_state(sc, &f0, &a0, &rc0, &bc0) == AS_OK);
      }
      int32_t c[64], e[64], a[64], nc = 0, ne = 0, na = 0, which = 0;
      enomem += sweep_failures([&] { return as_sched_step(sc, it > 0, c, &nc, e, &ne, a, &na, 64, &which); }, same, &ok);
      REQUIRE(ok);
    }
    REQUIRE(as_sched_destroy(sc) == AS_OK);
    REQUIRE(enomem > 50);   // the injection really reached the library's allocations
    std::printf("allocation failures surfaced as AS_ENOMEM: %d\n", enomem);
  }
  std::puts("host fuzz ok");
  return 0;
}
