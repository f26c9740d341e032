"""The attention call is graph-capturable (kernel launches only, no memset
nodes, no allocation when a workspace is passed): a captured decode step is
replayed several times with changing inputs and eager work in between, and
every replay must equal the eager result."""
import numpy as np
import pytest

from paper_2605_23389_amd import workloads as wl
from tests.gpu_util import oracle_out, to_device

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
    assert np.abs(out.double().cpu().numpy() - ref0).max() <= 1.5e-2

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
        assert np.abs(got.double().cpu().numpy() - oracle_out(pb)).max() <= 1.5e-2
