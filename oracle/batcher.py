"""Oracle for length-aligned ("prefix-aware") batch formation.

TEST INFRASTRUCTURE ONLY: pure Python; shares no code with the C++ library.

The paper's policy (Sections 2.4 and 3.3) is to put requests whose prefixes
have similar length into the same batch, because a decode iteration lasts as
long as its longest member (Section 2.3).  With a fixed batch size B that is
formalised here as: partition the n in-flight requests into ceil(n/B) batches
of at most B so that the sum over batches of the largest KV length is minimal.
Sorting by length and cutting consecutive chunks reaches that minimum; the
canonical form (the one bit-exactness is defined against) is

    order   = request indices sorted by (length descending, index ascending)
    batch j = order[j*B : (j+1)*B]        (the last batch may be short and
                                           then holds the shortest requests)

Parity pins (tests/test_oracle_batcher.py): brute force over every partition
on tiny inputs confirms the objective value is the minimum; the closed form
sum_k d[k*B] (d = lengths sorted descending); structural invariants
(permutation, monotone offsets, stable ties); a hand-written golden case.
"""
from __future__ import annotations


def aligned_batch(kv_lens, batch_size: int):
    """Returns (order, batch_offsets): plain Python lists of ints.
    Batch j is order[batch_offsets[j] : batch_offsets[j+1]]."""
    n = len(kv_lens)
    if batch_size <= 0:
        raise ValueError("batch_size must be positive")
    order = sorted(range(n), key=lambda i: (-int(kv_lens[i]), i))
    offsets = [0]
    while offsets[-1] < n:
        offsets.append(min(offsets[-1] + batch_size, n))
    return order, offsets


def sum_of_batch_max(kv_lens, order, batch_offsets) -> int:
    """The straggler objective: sum over batches of the longest member."""
    total = 0
    for j in range(len(batch_offsets) - 1):
        members = order[batch_offsets[j]:batch_offsets[j + 1]]
        total += max(int(kv_lens[i]) for i in members)
    return total
