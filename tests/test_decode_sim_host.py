"""Host-only checks of the decode loop's bookkeeping (paper Section 3.4,
Algorithm 2 driven through the C ABI; no GPU: data movement is recorded, not
executed): every request finishes, every block comes back, a re-admitted
request gets back exactly the blocks it was evicted with -- including
evictions at kv_len % 16 == 1, where one token sits alone in the last block --
and prefetched requests are admitted without a copy."""
import numpy as np
import pytest

from paper_2605_23389_amd import decode_sim
from paper_2605_23389_amd import workloads as wl


def _run(seed, policy, prefetch, n=40, max_batch=8, hbm_blocks=120):
    rng = np.random.default_rng(seed)
    prefix = wl.lognormal_lengths(rng, n, 200.0, 0.9, 8, 1500)
    outs = rng.integers(3, 40, n).astype(np.int32)
    need = int((prefix.max() + outs.max() + 15) // 16 + 2)
    cfg = decode_sim.SimConfig(num_q_heads=8, num_kv_heads=2, head_dim=128, max_batch=max_batch,
                               hbm_blocks=max(hbm_blocks, need), policy=policy, k_min=4, seed=seed,
                               prefetch=prefetch, dry=True)
    sim = decode_sim.DecodeSim(prefix, outs, cfg)
    stats = sim.run(max_iters=20000)
    return sim, stats, outs


def test_bookkeeping_over_many_seeds(lib):
    seen_mod1 = 0
    evictions = 0
    for seed, policy, prefetch in [(s, p, f) for s in range(25) for p in ("aligned", "fcfs") for f in (True, False)]:
        sim, stats, outs = _run(seed, policy, prefetch, hbm_blocks=100)
        assert stats["completed"] == len(outs)
        assert int(np.sum(stats["batch_size"])) == int(outs.sum())
        # every block is back and owned by nobody; no request is left anywhere
        assert sorted(sim.free_blocks) == list(range(sim.pool_blocks))
        assert (sim.owner == -1).all()
        assert not sim.blocks_of and not sim.evicted and not sim.prefetched and not sim.pending_free
        assert sim.cand_used == 0 and not sim.b_cand and not sim.r_cand
        assert len(sim.evict_free) == sim.evict_slots
        # a request comes back with exactly the blocks it left with
        assert stats["restored_blocks"] == stats["evicted_blocks"]
        evictions += stats["evictions"]
        seen_mod1 += sum(1 for L in stats["eviction_lens"] if L % 16 == 1)
        if prefetch:
            assert stats["admitted_prefetched"] > 0
        else:
            assert stats["admitted_prefetched"] == 0
    assert evictions > 100
    assert seen_mod1 >= 4, "no eviction with a lone token in the last block: the seeds no longer cover the case"


def test_unused_block_table_columns_hold_an_invalid_id(lib):
    sim, stats, outs = _run(6, "fcfs", True)
    # after the run every row was released; rows are rewritten with -1 beyond the request's blocks
    rng = np.random.default_rng(0)
    sim2 = decode_sim.DecodeSim(np.array([40, 17], dtype=np.int32), np.array([3, 3], dtype=np.int32),
                                decode_sim.SimConfig(num_q_heads=2, num_kv_heads=2, head_dim=64, max_batch=2,
                                                     hbm_blocks=16, policy="fcfs", dry=True))
    sim2._next_candidate_batch()
    done, ev, ad, case = sim2.sched.step(advance=False)
    sim2._admit(ad)
    for rid in ad:
        row = sim2.bt_all[sim2.row_of[rid]]
        nb = len(sim2.blocks_of[rid])
        assert (row[:nb] >= 0).all() and (row[nb:] == -1).all()
