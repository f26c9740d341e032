"""Integration test of the decode loop on the GPU: batch generation,
Algorithm 2 scheduling, staging, eviction round trips, attention and KV append
driven together; every few iterations the device KV of each running request is
compared byte by byte with a host mirror (initial host-pool blocks + appended
rows)."""
import numpy as np
import pytest

from paper_2605_23389_amd import decode_sim
from paper_2605_23389_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("policy", ["aligned", "fcfs"])
def test_decode_loop_keeps_kv_consistent_and_finishes_everyone(lib, policy):
    rng = np.random.default_rng(3)
    n = 40
    prefix = wl.lognormal_lengths(rng, n, 200.0, 0.9, 8, 1500)
    outs = rng.integers(3, 40, n).astype(np.int32)
    # a pool tight enough to force evictions
    cfg = decode_sim.SimConfig(num_q_heads=8, num_kv_heads=2, head_dim=128, max_batch=8, hbm_blocks=150,
                               policy=policy, k_min=4, verify_every=3, seed=1)
    sim = decode_sim.DecodeSim(prefix, outs, cfg)
    stats = sim.run(max_iters=5000)
    s = decode_sim.summarize(stats)
    assert s["completed"] == n
    assert s["generated_tokens"] == int(outs.sum())
    assert s["evictions"] > 0                       # the eviction path really ran
    assert len(sim.free_blocks) == cfg.hbm_blocks   # every block returned
    assert sorted(sim.free_blocks) == list(range(cfg.hbm_blocks))
    assert not sim.blocks_of and not sim.evict_slot
