"""The host-resident KV pipeline at its own shape, reduced in request count
only (paper Sections 3.2 and 4.4): 64 query / 8 KV heads, head_dim 128, bf16,
KV of two layers per token in pinned host pools with UNIQUE blocks (no
aliasing), length-aligned batches of 128 out of 384 requests drawn like the
full configuration, staged by as_stage_kv through the as_pipeline_* handshake
into a double-buffered HBM pool while the previous batch is attended, the
work plan built for layer 0 and reused (AS_ATTN_REUSE_PLAN) for layer 1.
Sampled (request, KV head) outputs of every batch and layer are compared with
the oracle on the host pool's own bytes, fp32 output, at the matrix-core
kernel's bound; a buffer is poisoned after its attention so that a copy or an
attention that does not wait would show."""
import math

import numpy as np
import pytest

from oracle import attention as oa
from paper_2605_23389_amd import workloads as wl
from tests import parity_bounds as pbnd

pytestmark = pytest.mark.gpu


def test_two_layer_gqa_batches_through_the_double_buffered_pipeline(lib):
    import torch
    from paper_2605_23389_amd import binding as als
    sh = wl.CONFIG_SHAPES[4]
    Hq, Hkv, D = sh["num_q_heads"], sh["num_kv_heads"], sh["head_dim"]
    assert (Hq, Hkv, D) == (64, 8, 128)
    layers, n, Bsz = 2, 384, 128
    lens = wl.config_lengths(4)[:n]
    order, offs = lib.aligned_batch(lens, Bsz)
    nblk = (lens.astype(np.int64) + 15) // 16
    starts = np.concatenate([[0], np.cumsum(nblk)[:-1]])
    total = int(nblk.sum())
    block_bytes = Hkv * 16 * D * 2
    # unique host blocks, drawn on the device and copied into pinned memory
    g = torch.Generator(device="cuda").manual_seed(4)
    host_k, host_v = [], []
    for l in range(layers):
        for dst in (host_k, host_v):
            t = torch.empty((total, Hkv, 16, D), dtype=torch.bfloat16, pin_memory=True)
            for i in range(0, total, 8192):
                m = min(8192, total - i)
                t[i:i + m].copy_(torch.empty((m, Hkv, 16, D), dtype=torch.bfloat16, device="cuda").normal_(generator=g))
            dst.append(t)
    torch.cuda.synchronize()
    batches = []
    for j in range(len(offs) - 1):
        members = order[offs[j]:offs[j + 1]]
        L = np.ascontiguousarray(lens[members])
        nb = nblk[members]
        src = np.concatenate([starts[r] + np.arange(nblk[r]) for r in members]).astype(np.int64)
        bt = np.zeros((len(members), int(nb.max())), dtype=np.int32)
        cur = 0
        for i, n_i in enumerate(nb):
            bt[i, :n_i] = np.arange(cur, cur + n_i)
            cur += int(n_i)
        batches.append(dict(members=members, lens=L, src=src, nblocks=cur, bt=bt))
    cap = max(b["nblocks"] for b in batches)
    dev_k = [torch.full((2 * cap, Hkv, 16, D), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(layers)]
    dev_v = [torch.full((2 * cap, Hkv, 16, D), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(layers)]
    gq = torch.Generator(device="cuda").manual_seed(5)
    for j, b in enumerate(batches):
        b["buf"] = j % 2
        b["dst"] = (np.arange(b["nblocks"]) + b["buf"] * cap).astype(np.int32)
        b["dbt"] = torch.from_numpy(b["bt"] + b["buf"] * cap).cuda()
        b["dlens"] = torch.from_numpy(b["lens"]).cuda()
        b["q"] = [torch.empty((len(b["lens"]), Hq, D), dtype=torch.bfloat16, device="cuda").normal_(generator=gq)
                  for _ in range(layers)]
        b["out"] = [torch.full((len(b["lens"]), Hq, D), float("nan"), dtype=torch.float32, device="cuda")
                    for _ in range(layers)]
    prm0 = als.attn_params(batches[0]["q"][0], dev_k[0], batches[0]["dbt"], batches[0]["out"][0])
    ws = torch.empty(max(als.decode_attention_workspace(
        als.attn_params(b["q"][0], dev_k[0], b["dbt"], b["out"][0]), int(b["lens"].sum())) for b in batches),
        dtype=torch.uint8, device="cuda")
    pipe = als.Pipeline(2)
    compute = torch.cuda.Stream()

    def stage(b):
        pipe.begin_stage(b["buf"])
        for l in range(layers):
            lib.stage_kv(host_k[l], host_v[l], b["src"], dev_k[l], dev_v[l], b["dst"], block_bytes, stream=pipe.stream)
        pipe.end_stage(b["buf"])

    def attend(b):
        pipe.acquire(b["buf"], stream=compute)
        with torch.cuda.stream(compute):
            prm = als.attn_params(b["q"][0], dev_k[0], b["dbt"], b["out"][0])
            for l in range(layers):
                prm.flags = 0 if l == 0 else als.ATTN_REUSE_PLAN
                lib.decode_attention(b["q"][l], dev_k[l], dev_v[l], b["dbt"], b["dlens"], b["out"][l],
                                     kv_lens_host=b["lens"], workspace=ws, params=prm, stream=compute)
            lo, hi = b["buf"] * cap, (b["buf"] + 1) * cap
            for l in range(layers):               # poison after use: the next copy into this buffer must wait
                dev_k[l][lo:hi].fill_(float("nan"))
                dev_v[l][lo:hi].fill_(float("nan"))
        pipe.release(b["buf"], stream=compute)

    stage(batches[0])
    for j, b in enumerate(batches):
        if j + 1 < len(batches):
            stage(batches[j + 1])                 # overlaps with the attention of batch j
        attend(b)
    torch.cuda.synchronize()
    pipe.destroy()

    assert pbnd.uses_matrix_core("bf16", D, Hq, Hkv)
    rng = np.random.default_rng(6)
    G = Hq // Hkv
    worst = 0.0
    for j, b in enumerate(batches):
        for l in range(layers):
            assert torch.isfinite(b["out"][l]).all(), f"batch {j} layer {l}: non-finite output"
        picks = [(int(i), int(h)) for i, h in zip(rng.integers(0, len(b["lens"]), 3), rng.integers(0, Hkv, 3))]
        picks += [(int(np.argmax(b["lens"])), 0), (int(np.argmin(b["lens"])), Hkv - 1)]
        for i, h in picks:
            r = int(b["members"][i])
            L = int(lens[r])
            s, e = int(starts[r]), int(starts[r] + nblk[r])
            for l in range(layers):
                K = host_k[l][s:e, h].reshape(-1, D)[:L].float().numpy()
                V = host_v[l][s:e, h].reshape(-1, D)[:L].float().numpy()
                for gq_ in range(G):
                    hq = h * G + gq_
                    ref = oa.attention_single(b["q"][l][i, hq].float().cpu().numpy(), K, V, 1.0 / math.sqrt(D))
                    got = b["out"][l][i, hq].double().cpu().numpy()
                    worst = max(worst, pbnd.assert_parity(got, ref, "bf16", "fp32", True,
                                                          what=f"batch {j} layer {l} request {r} head {hq}"))
    assert worst > 0.0
