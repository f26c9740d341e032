"""Integration test of the decode loop on the GPU: batch generation,
Algorithm 2 scheduling, candidate-buffer prefetch on the side stream,
eviction round trips behind events, KV append and attention driven together;
after EVERY iteration the device KV of each running request is compared byte
by byte with a host mirror (initial host-pool blocks + appended rows).  The
seeds and pool sizes are chosen (on the CPU, with the dry back end) so that a
request is evicted while a single token sits in its last block, the case in
which a block count derived from a stale length loses that block."""
import numpy as np
import pytest

from paper_2605_23389_amd import decode_sim
from paper_2605_23389_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _inputs(seed, n=40):
    rng = np.random.default_rng(seed)
    prefix = wl.lognormal_lengths(rng, n, 200.0, 0.9, 8, 1500)
    outs = rng.integers(3, 40, n).astype(np.int32)
    return prefix, outs


@pytest.mark.parametrize("prefetch", [True, False])
@pytest.mark.parametrize("policy,seed,hbm_blocks", [("aligned", 10, 100), ("fcfs", 0, 120)])
def test_decode_loop_keeps_kv_consistent_and_finishes_everyone(lib, policy, seed, hbm_blocks, prefetch):
    prefix, outs = _inputs(seed)
    cfg = decode_sim.SimConfig(num_q_heads=8, num_kv_heads=2, head_dim=128, max_batch=8, hbm_blocks=hbm_blocks,
                               policy=policy, k_min=4, verify_every=1, seed=seed, prefetch=prefetch)
    sim = decode_sim.DecodeSim(prefix, outs, cfg)
    stats = sim.run(max_iters=5000)
    s = decode_sim.summarize(stats)
    assert s["completed"] == len(outs)
    assert s["generated_tokens"] == int(outs.sum())
    assert s["evictions"] > 0                                  # the eviction path really ran ...
    assert any(L % 16 == 1 for L in stats["eviction_lens"])    # ... with a lone token in the last block
    assert stats["restored_blocks"] == stats["evicted_blocks"]
    assert sorted(sim.free_blocks) == list(range(sim.pool_blocks))   # every block returned
    assert not sim.blocks_of and not sim.evicted and not sim.prefetched
    if prefetch:
        assert s["admitted_staged_ahead"] > 0 and s["staged_ahead_GB"] > 0
    else:
        assert s["admitted_staged_ahead"] == 0 and s["staged_ahead_GB"] == 0
    assert s["unstaged_GB"] > 0


def test_prefetch_takes_the_copies_off_the_critical_path(lib):
    """Same requests, same schedule: with prefetch on, (almost) nothing is staged at admission
    time; with prefetch off, everything is."""
    prefix, outs = _inputs(3, n=64)
    res = {}
    for prefetch in (True, False):
        # prefetch never pauses for unfinished copy groups here, so that what is staged ahead does
        # not depend on how fast this machine copies
        cfg = decode_sim.SimConfig(num_q_heads=8, num_kv_heads=2, head_dim=128, max_batch=8, hbm_blocks=400,
                                   policy="aligned", k_min=4, seed=3, prefetch=prefetch, prefetch_groups_in_flight=7)
        res[prefetch] = decode_sim.summarize(decode_sim.DecodeSim(prefix, outs, cfg).run(max_iters=5000))
    on, off = res[True], res[False]
    assert on["iterations"] == off["iterations"] and on["generated_tokens"] == off["generated_tokens"]
    assert off["staged_ahead_GB"] == 0 and off["staged_at_admission_GB"] > 0
    # the very first batch cannot be staged ahead of its own admission; the rest is
    assert on["staged_ahead_GB"] > 0.5 * off["staged_at_admission_GB"]
    assert on["staged_at_admission_GB"] < 0.5 * off["staged_at_admission_GB"]
