// Length-aligned batch formation (host only).
//
// Paper Sections 2.4 / 3.3: requests with similar prefix length share a batch
// so that no decode iteration waits for a straggler (Section 2.3).  For a
// fixed batch size the partition that minimises the sum of per-batch maximum
// lengths is reached by sorting on length and cutting consecutive chunks; the
// canonical order is (length descending, request index ascending), which
// leaves the short remainder batch with the shortest requests.
//
// Implementation: LSD radix sort on the key ~length (so that ascending key
// order is descending length); radix passes are stable, which yields the
// index-ascending tie order for free.  Passes whose digit is constant over
// the input (the high bytes of realistic lengths) are skipped.
#include <cstdint>
#include <cstring>
#include <vector>

#include "common.h"

namespace als {
char* error_buffer() {
  static thread_local char buf[512] = {0};
  return buf;
}
}  // namespace als

extern "C" int32_t as_version(void) { return 100; }

extern "C" const char* as_last_error(void) { return als::error_buffer(); }

extern "C" as_status as_aligned_batch(const int32_t* kv_lens, int32_t n, int32_t batch_size,
                                      int32_t* order, int32_t* batch_offsets,
                                      int32_t* num_batches) {
  if (n < 0) return als::fail(AS_EINVAL, "as_aligned_batch: n = %d is negative", n);
  if (batch_size <= 0)
    return als::fail(AS_EINVAL, "as_aligned_batch: batch_size = %d must be positive", batch_size);
  if (!batch_offsets || !num_batches)
    return als::fail(AS_EINVAL, "as_aligned_batch: batch_offsets / num_batches is null");
  if (n > 0 && (!kv_lens || !order))
    return als::fail(AS_EINVAL, "as_aligned_batch: kv_lens / order is null with n > 0");
  for (int32_t i = 0; i < n; ++i)
    if (kv_lens[i] < 1)
      return als::fail(AS_EINVAL, "as_aligned_batch: kv_lens[%d] = %d, must be >= 1", i,
                       kv_lens[i]);

  const int64_t nb = (static_cast<int64_t>(n) + batch_size - 1) / batch_size;
  ALS_TRY
  if (n > 0) {
    // key = bitwise complement of the (positive) length: ascending key <=> descending length
    std::vector<uint32_t> key_a(n), key_b(n);
    std::vector<int32_t> idx_b(n);
    int32_t* idx_a = order;
    uint32_t all_or = 0, all_and = ~0u;
    for (int32_t i = 0; i < n; ++i) {
      key_a[i] = ~static_cast<uint32_t>(kv_lens[i]);
      idx_a[i] = i;
      all_or |= key_a[i];
      all_and &= key_a[i];
    }
    uint32_t* ka = key_a.data();
    uint32_t* kb = key_b.data();
    int32_t* ia = idx_a;
    int32_t* ib = idx_b.data();
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 8 * pass;
      if ((((all_or ^ all_and) >> shift) & 0xFFu) == 0) continue;  // digit constant: no-op pass
      uint32_t count[257];
      std::memset(count, 0, sizeof(count));
      for (int32_t i = 0; i < n; ++i) ++count[((ka[i] >> shift) & 0xFFu) + 1];
      for (int d = 0; d < 256; ++d) count[d + 1] += count[d];
      for (int32_t i = 0; i < n; ++i) {
        const uint32_t pos = count[(ka[i] >> shift) & 0xFFu]++;
        kb[pos] = ka[i];
        ib[pos] = ia[i];
      }
      uint32_t* tk = ka; ka = kb; kb = tk;
      int32_t* ti = ia; ia = ib; ib = ti;
    }
    if (ia != order) std::memcpy(order, ia, sizeof(int32_t) * static_cast<size_t>(n));
  }
  ALS_CATCH("as_aligned_batch")
  for (int64_t j = 0; j <= nb; ++j) {
    const int64_t off = j * batch_size;
    batch_offsets[j] = static_cast<int32_t>(off < n ? off : n);
  }
  *num_batches = static_cast<int32_t>(nb);
  als::error_buffer()[0] = 0;
  return AS_OK;
}
