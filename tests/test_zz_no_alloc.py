"""The entry point for callers that cannot allocate (as_decode_attention_static:
plan and split-KV partials in the library's static device array) against
as_decode_attention on the same inputs, through the C ABI.  Same kernels, same
plan, so the results must agree bit for bit, and both must meet the parity
bounds against the oracle.  Two calls in a row share the array, the second on
a smaller input, so stale contents of the first must not matter."""
import numpy as np
import pytest

from paper_2605_23389_amd import workloads as wl
from tests.gpu_util import check_parity, oracle_out, to_device

pytestmark = pytest.mark.gpu


def _both(lib, pb, d, host_lens, chunk, flags=0):
    import torch
    out_ws = torch.full(d["q"].shape, float("nan"), dtype=torch.float32, device="cuda")
    out_st = torch.full_like(out_ws, float("nan"))
    host = pb.kv_lens if host_lens else None
    lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out_ws, kv_lens_host=host,
                         chunk_tokens=chunk, flags=flags)
    before = torch.cuda.memory_allocated()
    lib.decode_attention_static(d["q"], d["k"], d["v"], d["bt"], d["lens"], out_st, kv_lens_host=host,
                                chunk_tokens=chunk, flags=flags)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return out_ws, out_st


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2)])          # vector-ALU and matrix-core kernels
@pytest.mark.parametrize("host_lens", [True, False])
def test_static_scratch_call_equals_workspace_call_twice_in_a_row(lib, Hq, Hkv, host_lens):
    import torch
    rng = np.random.default_rng(17)
    big = np.concatenate([rng.integers(1, 3000, 20), [4097, 1, 16]]).astype(np.int32)
    small = rng.integers(1, 300, 5).astype(np.int32)
    for i, lens in enumerate((big, small)):                   # second call: smaller input
        pb = wl.make_paged_batch(lens, Hq, Hkv, 128, dtype="bf16", seed=40 + i, poison="nan", spare_blocks=1)
        ref = oracle_out(pb)
        d = to_device(pb)
        for chunk in (64, 0):                                 # split (plan + combine) and the library's choice
            out_ws, out_st = _both(lib, pb, d, host_lens, chunk)
            assert torch.equal(out_ws, out_st), f"call {i}, chunk {chunk}: static-scratch result differs"
            check_parity(out_st.double().cpu().numpy(), ref, pb, out_dtype="fp32", what=f"call {i} chunk {chunk}")


def test_static_scratch_rejects_what_does_not_fit(lib):
    """A plan + partials beyond the array: AS_EWORKSPACE before anything is enqueued."""
    import torch
    from paper_2605_23389_amd import binding as als
    cap = lib.decode_attention_static_capacity()
    assert cap == 32 << 20
    # 64 requests x 64 heads x 128 dims, 16-token chunks over 4096 tokens each: ~0.5 GB of partials
    B, Hq, Hkv, D, L = 64, 64, 8, 128, 4096
    q = torch.zeros((B, Hq, D), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((4, Hkv, 16, D), dtype=torch.bfloat16, device="cuda")
    bt = torch.zeros((B, L // 16), dtype=torch.int32, device="cuda")
    dl = torch.full((B,), L, dtype=torch.int32, device="cuda")
    out = torch.full((B, Hq, D), 7.0, dtype=torch.float32, device="cuda")
    params = als.attn_params(q, k, bt, out, chunk_tokens=16)
    assert lib.decode_attention_workspace(params, B * L) > cap
    with pytest.raises(als.AlignedServeError) as e:
        lib.decode_attention_static(q, k, k, bt, dl, out, kv_lens_host=np.full(B, L, dtype=np.int32),
                                    params=params)
    assert e.value.status == als.AS_EWORKSPACE
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)                              # nothing ran
    # the same shape with the library's own chunking fits and runs
    params = als.attn_params(q, k, bt, out)
    lib.decode_attention_static(q, k, k, bt, dl, out, kv_lens_host=np.full(B, L, dtype=np.int32), params=params)
    torch.cuda.synchronize()
    assert torch.all(out == 0.0)                              # V is all zeros


def test_static_scratch_call_under_graph_capture(lib):
    """The callers it exists for: one decode step (append + attention planned on the device, no
    host lengths, no workspace) captured once and replayed while the lengths grow; every replay is
    checked against the workspace entry point run eagerly on the same state."""
    import torch
    L0 = np.array([60, 126, 15, 255, 1, 700], dtype=np.int32)
    R = 4
    pb = wl.make_paged_batch(L0 + R, 8, 2, 128, dtype="bf16", seed=77, spare_blocks=1)
    d = to_device(pb)
    B = len(L0)
    dl = torch.from_numpy(L0.copy()).cuda()
    k_new = torch.empty((B, 2, 128), dtype=torch.bfloat16, device="cuda").normal_()
    v_new = torch.empty_like(k_new).normal_()
    out = torch.zeros(d["q"].shape, dtype=torch.float32, device="cuda")
    ref = torch.zeros_like(out)
    lib.decode_attention_static(d["q"], d["k"], d["v"], d["bt"], dl, out, chunk_tokens=64)   # looks the array up
    torch.cuda.synchronize()

    def step():
        lib.kv_append(k_new, v_new, d["k"], d["v"], d["bt"], dl)
        lib.decode_attention_static(d["q"], d["k"], d["v"], d["bt"], dl, out, chunk_tokens=64)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for r in range(R):
        d["q"].normal_()
        k_new.normal_()
        v_new.normal_()
        out.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert dl.cpu().numpy().tolist() == (L0 + r + 1).tolist()
        lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], dl, ref, chunk_tokens=64)      # eager, workspace
        torch.cuda.synchronize()
        assert torch.equal(out, ref), f"replay {r}"
        assert torch.isfinite(out).all()
