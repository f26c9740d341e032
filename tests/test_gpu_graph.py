"""The attention call is graph-capturable (kernel launches only, no memset
nodes, no allocation when a workspace is passed): a captured decode step is
replayed several times with changing inputs and eager work in between, and
every replay must equal the eager result."""
import numpy as np
import pytest

from paper_2605_23389_amd import workloads as wl
from tests.gpu_util import check_parity, oracle_out, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("Hq,Hkv,lens", [(8, 8, [40, 700, 1300, 17]), (16, 2, [5000, 300, 2049])])
def test_captured_attention_replays_match_eager(lib, Hq, Hkv, lens):
    import torch
    from paper_2605_23389_amd import binding as als
    lens = np.asarray(lens, dtype=np.int32)
    pb = wl.make_paged_batch(lens, Hq, Hkv, 128, dtype="bf16", seed=4, poison="nan", spare_blocks=1)
    d = to_device(pb)
    out = torch.zeros(d["q"].shape, dtype=torch.float32, device="cuda")
    params = als.attn_params(d["q"], d["k"], d["bt"], out, chunk_tokens=256)    # forces plan + combine
    ws = torch.empty(lib.decode_attention_workspace(params, int(lens.sum())), dtype=torch.uint8, device="cuda")

    def call():
        lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out, kv_lens_host=lens,
                             workspace=ws, params=params)
    call()
    torch.cuda.synchronize()
    ref0 = oracle_out(pb)
    check_parity(out.double().cpu().numpy(), ref0, pb, out_dtype="fp32")

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            call()
    torch.cuda.current_stream().wait_stream(side)
    rng = np.random.default_rng(0)
    for rep in range(4):
        newq = wl.f32_to_bf16_bits(rng.standard_normal(pb.q.shape, dtype=np.float32))
        d["q"].copy_(torch.from_numpy(newq.view(np.int16)).cuda().view(torch.bfloat16))
        out.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        got = out.clone()
        out.fill_(float("nan"))
        call()                                    # eager, between replays
        torch.cuda.synchronize()
        assert torch.equal(got, out), f"replay {rep} differs from eager"
        pb.q = newq
        check_parity(got.double().cpu().numpy(), oracle_out(pb), pb, out_dtype="fp32", what=f"replay {rep}")


def test_captured_decode_step_follows_growing_lengths(lib):
    """One decode step (KV append + attention planned on the device, no host
    lengths) captured once and replayed while every request grows by a token
    per replay, across block and chunk boundaries; each replay is checked
    against the oracle for the lengths of that moment."""
    import torch
    from oracle import attention as oa
    from paper_2605_23389_amd import binding as als
    L0 = np.array([60, 126, 15, 255, 1], dtype=np.int32)
    R = 6
    pb = wl.make_paged_batch(L0 + R, 4, 2, 128, dtype="bf16", seed=31, poison="nan", spare_blocks=1)
    d = to_device(pb)
    B = len(L0)
    # the rows the replays will append: keep them aside, poison them in the pool
    rows_k = torch.empty((R, B, 2, 128), dtype=torch.bfloat16, device="cuda")
    rows_v = torch.empty_like(rows_k)
    for r in range(R):
        for b in range(B):
            t = int(L0[b]) + r
            blk, row = int(pb.block_table[b, t // 16]), t % 16
            rows_k[r, b] = d["k"][blk, :, row]
            rows_v[r, b] = d["v"][blk, :, row]
            d["k"][blk, :, row] = float("nan")
            d["v"][blk, :, row] = float("nan")
    dl = torch.from_numpy(L0.copy()).cuda()
    k_new = torch.empty((B, 2, 128), dtype=torch.bfloat16, device="cuda")
    v_new = torch.empty_like(k_new)
    out = torch.zeros(d["q"].shape, dtype=torch.float32, device="cuda")
    params = als.attn_params(d["q"], d["k"], d["bt"], out, chunk_tokens=64)
    ws = torch.empty(lib.decode_attention_workspace(params, -1), dtype=torch.uint8, device="cuda")

    def step():
        lib.kv_append(k_new, v_new, d["k"], d["v"], d["bt"], dl)
        lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], dl, out, workspace=ws, params=params)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    k_new.copy_(rows_k[0]); v_new.copy_(rows_v[0])
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()                                  # capture only: nothing runs
    torch.cuda.current_stream().wait_stream(side)
    rng = np.random.default_rng(1)
    kf, vf, qshape = pb.as_float("k_blocks"), pb.as_float("v_blocks"), pb.q.shape
    for r in range(R):
        newq = wl.f32_to_bf16_bits(rng.standard_normal(qshape, dtype=np.float32))
        d["q"].copy_(torch.from_numpy(newq.view(np.int16)).cuda().view(torch.bfloat16))
        k_new.copy_(rows_k[r]); v_new.copy_(rows_v[r])
        out.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert dl.cpu().numpy().tolist() == (L0 + r + 1).tolist()
        ref = oa.decode_attention(wl.bf16_bits_to_f32(newq), kf, vf, pb.block_table, L0 + r + 1)
        got = out.double().cpu().numpy()
        check_parity(got, ref, pb, out_dtype="fp32", what=f"replay {r}")
