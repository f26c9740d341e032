#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

Workload (named in config.workload): the prefix-aware-vs-random case --
1024 in-flight requests, KV lengths lognormal(median 1024, sigma 1.2) clipped
to [64, 32768], 7B-shaped layer (32 MHA heads x 128, bf16), KV resident in a
paged HBM pool with random physical block placement.  One step = one pass of
the path over all requests: as_aligned_batch on the 1024 lengths, then one
as_decode_attention per length-aligned batch of 64 (16 batches).  `value` is
the algorithmic KV bandwidth of that pass (bytes the method must move / time).
The same pass over a seeded random grouping, per-batch times, the 7B-shaped
single ragged batch, the GQA long-context batch, the streaming-read ceiling,
the host-to-HBM staging pipeline and the CPU oracle are reported beside it.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def time_region(fn, iters, torch):
    """GPU time of `iters` calls of fn() on the current stream, by HIP events."""
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--chunk-tokens", type=int, default=0)
    ap.add_argument("--skip-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--skip-extra", action="store_true",
                    help="only the headline pass (used for profiling runs)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 2 GiB device-to-device copies (a kernel of known "
                         "traffic, for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_23389_amd import binding as als
    from paper_2605_23389_amd import harness, traffic
    from paper_2605_23389_amd import workloads as wl

    als.load()
    torch.cuda.set_device(0)
    dev_name = torch.cuda.get_device_name(0)
    shape = wl.CONFIG_SHAPES[2]
    Hq, Hkv, D = shape["num_q_heads"], shape["num_kv_heads"], shape["head_dim"]
    B = 64
    lens = wl.config_lengths(2, args.seed)
    n = len(lens)
    log(f"device {dev_name}; building pool for {n} requests, {int(lens.sum())} tokens")
    t0 = time.perf_counter()
    pool = harness.make_device_pool(lens, Hq, Hkv, D, dtype="bf16", seed=args.seed)
    torch.cuda.synchronize()
    log(f"pool: {pool.k.shape[0]} blocks, {2 * pool.k.numel() * 2 / 1e9:.1f} GB in {time.perf_counter() - t0:.1f}s")

    order_a, offs_a = als.aligned_batch(lens, B)
    order_r, offs_r = wl.random_grouping(n, B, seed=args.seed)
    batches_a = harness.make_device_batches(pool, order_a, offs_a, seed=args.seed)
    batches_r = harness.make_device_batches(pool, order_r, offs_r, seed=args.seed)

    def params_for(b):
        return als.attn_params(b.q, pool.k, b.block_table, b.out, chunk_tokens=args.chunk_tokens)

    # one workspace big enough for any batch of either grouping
    ws_bytes = max(als.decode_attention_workspace(params_for(b), b.tokens) for b in batches_a + batches_r)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    for b in batches_a + batches_r:
        b.params = params_for(b)
        b.bytes = traffic.attention_bytes(b.kv_lens_host, Hq, Hkv, D, 2, 2)

    def attend(b):
        als.decode_attention(b.q, pool.k, pool.v, b.block_table, b.kv_lens, b.out,
                             kv_lens_host=b.kv_lens_host, workspace=ws, params=b.params)

    def step_aligned():
        o, f = als.aligned_batch(lens, B)          # batch formation is part of the step
        for b in batches_a:
            attend(b)

    def step_random():
        for b in batches_r:
            attend(b)

    if args.copy_calibration:
        src = torch.empty(1 << 31, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- headline: K timed steps over the aligned batches
    for _ in range(args.warmup):
        step_aligned()
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    gpu_s = time_region(step_aligned, args.steps, torch)
    wall_s = time.perf_counter() - w0
    bytes_a = sum(b.bytes for b in batches_a)
    ms_per_step = wall_s / args.steps * 1e3
    value = bytes_a * args.steps / wall_s / 1e9
    launches = len(batches_a) * args.steps
    avg_launch_s = gpu_s / launches
    achieved = bytes_a / len(batches_a) / avg_launch_s / 1e9
    log(f"aligned: {ms_per_step:.3f} ms/step wall, {gpu_s / args.steps * 1e3:.3f} ms/step GPU, {value:.0f} GB/s")

    traffic_gb = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic_gb = json.load(open(tpath)).get("attn_cfg2_aligned_bytes_per_launch")
        except Exception:
            traffic_gb = None

    result = {
        "metric": "decode attention HBM GB/s (% of peak) + per-iteration us, aligned vs random",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "configs[2] aligned: 1024 requests, lognormal(1024, s1.2) clip [64,32768], "
                        "32 MHA heads x 128 bf16, block 16, 16 length-aligned batches of 64 per step",
            "device": dev_name, "seed": args.seed, "tokens_per_step": int(lens.sum()),
            "bytes_per_step": int(bytes_a), "chunk_tokens": args.chunk_tokens,
        },
        "pct_of_peak": round(100 * value / HBM_PEAK_GBS, 1),
        "roofline": {
            "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic_gb,
            "kernel": "attn_kernel<bf16,128,1>",
            "avg_launch_us": round(avg_launch_s * 1e6, 2),
            "alg_bytes_per_launch": int(bytes_a / len(batches_a)),
            "note": "launch duration = HIP-event time of the timed region / attention launches; "
                    "it includes the small plan and combine kernels of each call",
        },
    }

    if not args.skip_extra:
        # ---------------- per-batch times, aligned vs random
        def per_batch(batches, reps=5):
            rows = []
            for b in batches:
                attend(b)
                s = time_region(lambda: attend(b), reps, torch) / reps
                rows.append({"tokens": b.tokens, "max_len": int(b.kv_lens_host.max()),
                             "us": round(s * 1e6, 1), "GBs": round(b.bytes / s / 1e9, 0)})
            return rows

        rows_a = per_batch(batches_a)
        for _ in range(2):
            step_random()
        gpu_r = time_region(step_random, max(args.steps // 2, 3), torch) / max(args.steps // 2, 3)
        rows_r = per_batch(batches_r)
        bytes_r = sum(b.bytes for b in batches_r)
        result["aligned_vs_random"] = {
            "aligned": {"ms_per_pass": round(gpu_s / args.steps * 1e3, 3),
                        "GBs": round(bytes_a / (gpu_s / args.steps) / 1e9, 0),
                        "tokens_per_s": round(n / (gpu_s / args.steps), 0),
                        "sum_batch_max": int(sum(r["max_len"] for r in rows_a)), "batches": rows_a},
            "random": {"ms_per_pass": round(gpu_r * 1e3, 3), "GBs": round(bytes_r / gpu_r / 1e9, 0),
                       "tokens_per_s": round(n / gpu_r, 0),
                       "sum_batch_max": int(sum(r["max_len"] for r in rows_r)), "batches": rows_r},
            "note": "tokens_per_s = requests decoded per second by this one layer's attention",
        }
        log(f"random: {gpu_r * 1e3:.3f} ms/pass vs aligned {gpu_s / args.steps * 1e3:.3f}")

        # ---------------- streaming-read ceiling on the largest aligned batches
        cks = torch.zeros(256, dtype=torch.int32, device="cuda")

        def sweep_all():
            for b in batches_a:
                als.kv_read_sweep(pool.k, pool.v, b.block_table, b.kv_lens, cks, b.params, ws,
                                  kv_lens_host=b.kv_lens_host)
        sweep_all()
        sw = time_region(sweep_all, 5, torch) / 5
        result["read_ceiling"] = {"GBs": round(bytes_a / sw / 1e9, 0), "ms_per_pass": round(sw * 1e3, 3),
                                  "note": "same blocks, same work split, loads + XOR only"}
        log(f"read sweep: {bytes_a / sw / 1e9:.0f} GB/s")

        # ---------------- configs[1]: one ragged 7B-shaped batch of 64
        lens1 = wl.config_lengths(1, args.seed)
        pool1 = harness.make_device_pool(lens1, Hq, Hkv, D, dtype="bf16", seed=args.seed + 11)
        b1 = harness.make_device_batches(pool1, np.arange(64), np.array([0, 64]), seed=7)[0]
        b1.params = als.attn_params(b1.q, pool1.k, b1.block_table, b1.out, chunk_tokens=args.chunk_tokens)
        b1.bytes = traffic.attention_bytes(b1.kv_lens_host, Hq, Hkv, D, 2, 2)

        def attend1():
            als.decode_attention(b1.q, pool1.k, pool1.v, b1.block_table, b1.kv_lens, b1.out,
                                 kv_lens_host=b1.kv_lens_host, workspace=ws, params=b1.params)
        attend1()
        s1 = time_region(attend1, 20, torch) / 20
        result["cfg1_ragged_batch"] = {"tokens": b1.tokens, "us": round(s1 * 1e6, 1),
                                       "GBs": round(b1.bytes / s1 / 1e9, 0),
                                       "note": "configs[1]: 64 requests, lognormal(1024, s0.8) clip [128,8192]; "
                                               "its 1.5 GB working set is re-read back to back"}
        log(f"cfg1: {s1 * 1e6:.1f} us, {b1.bytes / s1 / 1e9:.0f} GB/s")

    # ---------------- CPU oracle baseline (bounded sample of the same workload)
    if not args.skip_cpu:
        from oracle import attention as oa
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = 1
        # batches from the middle outwards until the CPU-time budget is used
        mid = len(batches_a) // 2
        visit = sorted(range(len(batches_a)), key=lambda j: (abs(j - mid), j))
        done_bytes, done_tok, reqs, cpu_s, nb_done = 0, 0, 0, 0.0, 0
        for j in visit:
            bj = batches_a[j]
            for i, r in enumerate(bj.members):
                k, v, row = harness.fetch_request_kv(pool, int(r))
                q = bj.q[i].float().cpu().numpy()[None]
                L = np.array([int(pool.kv_lens[r])], dtype=np.int32)
                t1 = time.perf_counter()
                oa.decode_attention(q, k, v, row[None], L)
                cpu_s += time.perf_counter() - t1
                done_bytes += traffic.attention_bytes(L, Hq, Hkv, D, 2, 2)
                done_tok += int(L[0])
                reqs += 1
                if cpu_s > args.cpu_seconds:
                    break
            nb_done += 1
            if cpu_s > args.cpu_seconds:
                break
        result["cpu_baseline"] = {
            "value": round(done_bytes / cpu_s / 1e9, 3), "unit": "GB/s", "cores": int(cores),
            "kind": "oracle",
            "sample": f"{reqs} requests ({done_tok} tokens) from {nb_done} aligned batches taken from the "
                      f"middle of the length order outwards, fp64 NumPy oracle, {cpu_s:.1f} s of CPU time; "
                      f"bytes counted as bf16 like the GPU",
        }
        log(f"cpu oracle: {done_bytes / cpu_s / 1e9:.3f} GB/s on {cores} threads")

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
