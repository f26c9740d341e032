"""GPU parity of the KV append kernel and of a short decode loop (append +
attention over several iterations) against the oracles."""
import numpy as np
import pytest

from oracle import attention as oa
from oracle import decode_loop as od
from paper_2605_23389_amd import workloads as wl
from tests.gpu_util import check_parity, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,D,Hkv", [("bf16", 128, 8), ("fp32", 64, 4), ("bf16", 64, 2), ("fp32", 128, 1)])
def test_append_is_bit_exact_and_touches_nothing_else(lib, dtype, D, Hkv):
    import torch
    rng = np.random.default_rng(1)
    lens = np.array([1, 15, 16, 17, 31, 32, 100], dtype=np.int32)
    steps = 20
    pb = wl.make_paged_batch(lens + steps, Hkv, Hkv, D, dtype=dtype, seed=2, spare_blocks=2)
    cur = lens.copy()
    d = to_device(pb)
    d["lens"].copy_(torch.from_numpy(cur))
    for it in range(steps):
        if dtype == "bf16":
            kn = wl.f32_to_bf16_bits(rng.standard_normal((7, Hkv, D), dtype=np.float32))
            vn = wl.f32_to_bf16_bits(rng.standard_normal((7, Hkv, D), dtype=np.float32))
            kd = torch.from_numpy(kn.view(np.int16)).cuda().view(torch.bfloat16)
            vd = torch.from_numpy(vn.view(np.int16)).cuda().view(torch.bfloat16)
        else:
            kn = rng.standard_normal((7, Hkv, D), dtype=np.float32)
            vn = rng.standard_normal((7, Hkv, D), dtype=np.float32)
            kd, vd = torch.from_numpy(kn).cuda(), torch.from_numpy(vn).cuda()
        od.kv_append(pb.k_blocks, pb.v_blocks, pb.block_table, cur, kn, vn)
        lib.kv_append(kd, vd, d["k"], d["v"], d["bt"], d["lens"])
    torch.cuda.synchronize()
    assert d["lens"].cpu().numpy().tolist() == cur.tolist()

    def host(t):
        return t.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else t.cpu().numpy()
    assert np.array_equal(host(d["k"]), pb.k_blocks)     # every byte of the pool, spare blocks included
    assert np.array_equal(host(d["v"]), pb.v_blocks)


def test_full_row_is_left_untouched(lib):
    import torch
    pb = wl.make_paged_batch(np.array([16, 5], dtype=np.int32), 2, 2, 64, dtype="fp32", seed=3)
    d = to_device(pb)
    before = d["k"].clone()
    kn = torch.ones((2, 2, 64), device="cuda")
    lib.kv_append(kn, kn, d["k"], d["v"], d["bt"], d["lens"])   # request 0's single-block row is full
    torch.cuda.synchronize()
    assert d["lens"].cpu().tolist() == [16, 6]
    blk0 = int(pb.block_table[0, 0])
    assert torch.equal(d["k"][blk0], before[blk0])
    assert torch.all(d["k"][int(pb.block_table[1, 0]), :, 5, :] == 1)


def test_decode_loop_append_then_attend(lib):
    """Five iterations of (attention, append) on the GPU against the oracles."""
    import torch
    rng = np.random.default_rng(5)
    lens = np.array([14, 30, 63, 200], dtype=np.int32)
    iters = 5
    pb = wl.make_paged_batch(lens + iters, 8, 2, 128, dtype="bf16", seed=6)
    cur = lens.copy()
    d = to_device(pb)
    d["lens"].copy_(torch.from_numpy(cur))
    for it in range(iters):
        out = torch.empty(d["q"].shape, dtype=torch.float32, device="cuda")
        lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out, kv_lens_host=cur)
        ref = oa.decode_attention(pb.as_float("q"), pb.as_float("k_blocks"), pb.as_float("v_blocks"),
                                  pb.block_table, cur)
        torch.cuda.synchronize()
        check_parity(out.double().cpu().numpy(), ref, pb, out_dtype="fp32", what=f"iteration {it}")
        kn = wl.f32_to_bf16_bits(rng.standard_normal((4, 2, 128), dtype=np.float32))
        vn = wl.f32_to_bf16_bits(rng.standard_normal((4, 2, 128), dtype=np.float32))
        od.kv_append(pb.k_blocks, pb.v_blocks, pb.block_table, cur, kn, vn)
        lib.kv_append(torch.from_numpy(kn.view(np.int16)).cuda().view(torch.bfloat16),
                      torch.from_numpy(vn.view(np.int16)).cuda().view(torch.bfloat16),
                      d["k"], d["v"], d["bt"], d["lens"])
    torch.cuda.synchronize()
    assert d["lens"].cpu().numpy().tolist() == cur.tolist()
