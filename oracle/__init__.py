"""CPU oracle for the decode-attention hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 NumPy / pure-Python restatements of what the path computes,
written from the paper.  Nothing here is tuned, and nothing here shares code
with the HIP library or imports it.  Only the tests, the smoke check and the
benchmark's `cpu_baseline` leg may import this package; the product path
never does.
"""
from .attention import decode_attention, gather_kv, merge_partials, attention_single  # noqa: F401
from .batcher import aligned_batch, sum_of_batch_max  # noqa: F401
