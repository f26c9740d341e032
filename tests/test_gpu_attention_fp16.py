"""GPU parity for IEEE binary16 inputs (the precision the paper runs its models
in, Section 4.1) against the fp64 oracle on the same seeded, fp16-rounded
inputs.

Tolerances (max-abs over all elements; no figure is given for fp16 by the
build's target, so they follow from the arithmetic):
  * vector-ALU kernel, fp32 output: fp16 values widen exactly and every
    product of two of them is exact in fp32, so the arithmetic is that of the
    fp32 path -> 1e-5;
  * matrix-core kernel, fp32 output: probabilities enter the second
    contraction as two fp16 terms (22 significant bits) -> 2e-5;
  * fp16 output adds the output rounding 2^-11 * |out| with |out| < 4 for
    N(0,1) values -> 3e-3 in all.
"""
import numpy as np
import pytest

from paper_2605_23389_amd import workloads as wl
from tests.gpu_util import oracle_out, run_attention, to_device

pytestmark = pytest.mark.gpu

TOL_VALU = 1e-5
TOL_MFMA = 2e-5
TOL_OUT16 = 3e-3

LENS = np.array([1, 2, 15, 16, 17, 31, 33, 63, 64, 65, 100, 255, 256, 257, 300, 511, 513, 777, 1037],
                dtype=np.int32)


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 4), (8, 1), (6, 2), (3, 1)])
def test_fp16_vector_kernel_matches_oracle(lib, D, Hq, Hkv):
    from paper_2605_23389_amd import binding as als
    for poison in ("nan", "big"):
        pb = wl.make_paged_batch(LENS, Hq, Hkv, D, dtype="fp16", seed=7 * D + Hq, spare_blocks=2,
                                 poison=poison, extra_table_cols=3)
        ref = oracle_out(pb)
        dev = to_device(pb)
        for chunk in (0, 128):
            got = run_attention(lib, pb, out_dtype="fp32", chunk_tokens=chunk, dev=dev, flags=als.ATTN_NO_MFMA)
            assert np.isfinite(got).all()
            err = np.abs(got - ref).max()
            assert err <= TOL_VALU, f"max-abs err {err:.3e}"


@pytest.mark.parametrize("Hq,Hkv", [(4, 1), (8, 2), (16, 1), (32, 2), (24, 1), (5, 1), (12, 1), (32, 1), (64, 1), (29, 1)])
def test_fp16_matrix_core_kernel_matches_oracle(lib, Hq, Hkv):
    for poison in ("nan", "big"):
        pb = wl.make_paged_batch(LENS, Hq, Hkv, 128, dtype="fp16", seed=Hq * 5 + Hkv, spare_blocks=2,
                                 poison=poison, extra_table_cols=2)
        ref = oracle_out(pb)
        dev = to_device(pb)
        for chunk in (0, 64, 512):
            got = run_attention(lib, pb, out_dtype="fp32", chunk_tokens=chunk, dev=dev)
            assert np.isfinite(got).all()
            err = np.abs(got - ref).max()
            assert err <= TOL_MFMA, f"max-abs err {err:.3e} (chunk {chunk})"
        got16 = run_attention(lib, pb, out_dtype="fp16", dev=dev)
        assert np.abs(got16 - ref).max() <= TOL_OUT16


def test_fp16_single_token_returns_v_bitwise_and_mean_limit(lib):
    for Hq, Hkv in ((4, 2), (8, 1)):   # vector-ALU and matrix-core kernels
        pb = wl.make_paged_batch(np.ones(3, dtype=np.int32), Hq, Hkv, 128, dtype="fp16", seed=2, poison="nan")
        got = run_attention(lib, pb)   # fp16 out: v itself is representable
        v = pb.as_float("v_blocks").astype(np.float64)
        G = Hq // Hkv
        for b in range(3):
            for h in range(Hq):
                assert np.array_equal(got[b, h], v[pb.block_table[b, 0], h // G, 0])
        pb = wl.make_paged_batch(np.array([128], dtype=np.int32), Hq, Hkv, 128, dtype="fp16", seed=13)
        k0 = pb.k_blocks[pb.block_table[0, 0], :, 0, :].copy()
        for j in range(8):
            pb.k_blocks[pb.block_table[0, j]] = k0[:, None, :]
        got = run_attention(lib, pb, out_dtype="fp32", chunk_tokens=64)
        rows = np.concatenate([pb.as_float("v_blocks")[pb.block_table[0, j]] for j in range(8)], axis=1)
        mean = rows.astype(np.float64).mean(axis=1)          # [Hkv][D]
        assert np.abs(got[0] - np.repeat(mean, G, axis=0)).max() <= 1e-5


def test_fp16_reduced_7b_shape_and_gqa_long_context(lib):
    """The paper's own setting: a 7B-shaped MHA layer in fp16 (12 requests of
    the configs[1] length draw), and the long-context grouped-query shape."""
    lens = wl.config_lengths(1)[:12]
    pb = wl.make_paged_batch(lens, 32, 32, 128, dtype="fp16", seed=1, poison="nan", spare_blocks=2)
    ref = oracle_out(pb)
    assert np.abs(run_attention(lib, pb, out_dtype="fp32") - ref).max() <= TOL_VALU
    assert np.abs(run_attention(lib, pb, out_dtype="fp16") - ref).max() <= TOL_OUT16
    lens = np.array([4096, 9000, 20011], dtype=np.int32)
    pb = wl.make_paged_batch(lens, 64, 8, 128, dtype="fp16", seed=3, poison="nan", spare_blocks=1)
    assert np.abs(run_attention(lib, pb, out_dtype="fp32") - oracle_out(pb)).max() <= TOL_MFMA


def test_fp16_kv_append_then_attention(lib):
    """as_kv_append moves 16-bit rows whatever their format: append one token
    per request in fp16 and attend over the grown cache."""
    import torch
    lens = np.array([15, 16, 40, 1], dtype=np.int32)
    grown = lens + 1
    pb = wl.make_paged_batch(grown, 4, 2, 128, dtype="fp16", seed=21, poison="nan", spare_blocks=1)
    ref = oracle_out(pb)
    d = to_device(pb)
    # take the last token of every request out of the pool, then append it back
    k_new = torch.empty((4, 2, 128), dtype=torch.float16, device="cuda")
    v_new = torch.empty_like(k_new)
    for b in range(4):
        blk, row = int(pb.block_table[b, lens[b] // 16]), int(lens[b] % 16)
        k_new[b] = d["k"][blk, :, row]
        v_new[b] = d["v"][blk, :, row]
        d["k"][blk, :, row] = float("nan")
        d["v"][blk, :, row] = float("nan")
    dl = torch.from_numpy(lens).cuda()
    out = torch.empty(d["q"].shape, dtype=torch.float32, device="cuda")
    lib.kv_append(k_new, v_new, d["k"], d["v"], d["bt"], dl)
    lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], dl, out)
    torch.cuda.synchronize()
    assert dl.cpu().numpy().tolist() == grown.tolist()
    assert np.abs(out.double().cpu().numpy() - ref).max() <= TOL_VALU
