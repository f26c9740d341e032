"""GPU parity: the HIP decode attention (through the C ABI) against the fp64
oracle, element by element on the same seeded inputs.

Tolerances: the contract is a max-abs error of 1e-5 for fp32 inputs and 1.5e-2
for bf16 inputs with fp32 accumulation; every comparison here also asserts the
bound the kernels' arithmetic gives (tests/parity_bounds.py: 1e-5 for the
vector-ALU kernel and 1e-4 for the matrix-core kernel with fp32 output, plus
half an ulp of the output format for 16-bit output), because the absolute
1.5e-2 cannot fail on long requests."""
import numpy as np
import pytest

from paper_2605_23389_amd import workloads as wl
from tests.gpu_util import check_parity, oracle_out, run_attention, to_device

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-5, "bf16": 1.5e-2}


def _check(lib, pb, **kw):
    ref = oracle_out(pb, scale=kw.get("scale") or None)
    got = run_attention(lib, pb, **kw)
    return check_parity(got, ref, pb, out_dtype=kw.get("out_dtype"), flags=kw.get("flags", 0))


def test_tiny_config_fp32(lib):
    """configs[0]: 8 requests, 4 heads, D=64, fp32, U{16..256}, random block table."""
    for seed in (0, 1, 2):
        lens = wl.config_lengths(0, seed)
        pb = wl.make_paged_batch(lens, dtype="fp32", seed=seed, spare_blocks=3, poison="nan",
                                 num_q_heads=4, num_kv_heads=4, head_dim=64)
        _check(lib, pb)
        _check(lib, pb, chunk_tokens=64)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 4), (8, 2), (8, 1), (6, 2), (3, 1)])
def test_shapes_ragged_tails_and_poison(lib, dtype, D, Hq, Hkv):
    # lengths span several tiles, waves and chunks, every tail residue class
    lens = np.array([1, 2, 15, 16, 17, 31, 33, 63, 64, 65, 100, 255, 256, 257, 300, 511, 513, 777],
                    dtype=np.int32)
    for poison in ("nan", "big"):
        pb = wl.make_paged_batch(lens, Hq, Hkv, D, dtype=dtype, seed=D + Hq, spare_blocks=2,
                                 poison=poison, extra_table_cols=3)
        _check(lib, pb, chunk_tokens=128, out_dtype="fp32")
        _check(lib, pb, out_dtype="fp32")


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_result_independent_of_split(lib, dtype):
    rng = np.random.default_rng(5)
    lens = wl.uniform_lengths(rng, 12, 1, 1500)
    pb = wl.make_paged_batch(lens, 8, 2, 128, dtype=dtype, seed=5, poison="nan", spare_blocks=1)
    ref = oracle_out(pb)
    dev = to_device(pb)
    from paper_2605_23389_amd import binding as als
    # the vector-ALU kernel keeps probabilities in fp32: the split only changes
    # the summation order.  The matrix-core kernel (bf16, group of 4 here)
    # carries probabilities as two bf16 terms relative to each chunk's own
    # maximum, so different splits differ by that (16-bit) rounding.
    for flags, bound in ((als.ATTN_NO_MFMA, 2e-6 if dtype == "fp32" else 1e-5), (0, 5e-5)):
        outs = []
        for chunk in (16, 48, 112, 256, 1024, 4096, 0):
            got = run_attention(lib, pb, out_dtype="fp32", chunk_tokens=chunk, dev=dev, flags=flags)
            check_parity(got, ref, pb, out_dtype="fp32", flags=flags)
            outs.append(got)
        spread = max(np.abs(o - outs[0]).max() for o in outs)
        assert spread <= bound, f"spread {spread:.3e} (flags {flags})"


def test_without_host_lens_and_plan_reuse(lib):
    from paper_2605_23389_amd import binding as als
    lens = np.array([5, 600, 17, 1025, 64], dtype=np.int32)
    pb = wl.make_paged_batch(lens, 4, 4, 128, dtype="bf16", seed=8, poison="nan", spare_blocks=1)
    ref = oracle_out(pb)
    got = run_attention(lib, pb, out_dtype="fp32", host_lens=False, chunk_tokens=256)
    check_parity(got, ref, pb, out_dtype="fp32")
    # second "layer" with the plan reused from a shared workspace
    import torch
    d = to_device(pb)
    out = torch.empty_like(d["q"], dtype=torch.float32)
    params = als.attn_params(d["q"], d["k"], d["bt"], out, chunk_tokens=256)
    ws = torch.empty(lib.decode_attention_workspace(params, int(lens.sum())), dtype=torch.uint8, device="cuda")
    lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out, kv_lens_host=lens,
                         workspace=ws, params=params)
    first = out.clone()
    out.fill_(float("nan"))
    params.flags = als.ATTN_REUSE_PLAN
    lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out, kv_lens_host=lens,
                         workspace=ws, params=params)
    torch.cuda.synchronize()
    assert torch.equal(first, out)
    check_parity(out.double().cpu().numpy(), ref, pb, out_dtype="fp32")


def test_single_token_returns_v_bitwise(lib):
    for dtype in ("fp32", "bf16"):
        pb = wl.make_paged_batch(np.ones(3, dtype=np.int32), 4, 2, 64, dtype=dtype, seed=2, poison="nan")
        got = run_attention(lib, pb)
        v = pb.as_float("v_blocks").astype(np.float64)
        for b in range(3):
            blk = pb.block_table[b, 0]
            for h in range(4):
                assert np.array_equal(got[b, h], v[blk, h // 2, 0])


def test_identical_keys_give_mean_of_v_and_large_offset(lib):
    lens = np.array([200], dtype=np.int32)
    pb = wl.make_paged_batch(lens, 2, 2, 64, dtype="fp32", seed=3)
    # all keys of the request identical, with a huge common score offset
    k0 = pb.k_blocks[pb.block_table[0, 0], :, 0, :].copy()
    k0 += 40.0 * pb.q[0] / np.linalg.norm(pb.q[0], axis=-1, keepdims=True)
    for j in range(13):
        pb.k_blocks[pb.block_table[0, j]] = k0[:, None, :]
    got = run_attention(lib, pb, chunk_tokens=64)
    rows = np.concatenate([pb.v_blocks[pb.block_table[0, j]] for j in range(13)], axis=1)[:, :200]
    mean = rows.astype(np.float64).mean(axis=1)
    assert np.isfinite(got).all()
    assert np.abs(got[0] - mean).max() <= 1e-5


def test_explicit_scale_and_bf16_output(lib):
    lens = wl.uniform_lengths(np.random.default_rng(4), 6, 10, 400)
    pb = wl.make_paged_batch(lens, 4, 4, 128, dtype="bf16", seed=4, poison="inf")
    _check(lib, pb, scale=0.25, out_dtype="fp32")
    _check(lib, pb, out_dtype="bf16")


def test_reduced_7b_shape_matches_oracle(lib):
    """configs[1] shape (32 MHA heads, D=128, bf16) on the first 12 requests of
    its length draw -- sized so that the oracle finishes in seconds."""
    lens = wl.config_lengths(1)[:12]
    pb = wl.make_paged_batch(lens, 32, 32, 128, dtype="bf16", seed=1, poison="nan", spare_blocks=2)
    _check(lib, pb, out_dtype="fp32")
    _check(lib, pb, out_dtype="bf16")


def test_reduced_gqa_long_context_matches_oracle(lib):
    """configs[3] shape (64 q heads / 8 kv heads, D=128, bf16), 3 long requests."""
    lens = np.array([4096, 9000, 20011], dtype=np.int32)
    pb = wl.make_paged_batch(lens, 64, 8, 128, dtype="bf16", seed=3, poison="nan", spare_blocks=1)
    _check(lib, pb, out_dtype="fp32")


def test_zero_length_request_gets_zeros_on_device_path(lib):
    import torch
    lens = np.array([40, 7], dtype=np.int32)
    pb = wl.make_paged_batch(lens, 2, 2, 64, dtype="fp32", seed=6)
    d = to_device(pb)
    d["lens"][1] = 0
    out = torch.full(d["q"].shape, float("nan"), device="cuda")
    lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out)   # no host lens: not validated
    torch.cuda.synchronize()
    assert torch.all(out[1] == 0)
    ref = oracle_out(pb)
    assert np.abs(out[0].double().cpu().numpy() - ref[0]).max() <= 1e-5


def test_read_sweep_checksum_is_xor_of_referenced_blocks(lib):
    import torch
    from paper_2605_23389_amd import binding as als
    lens = np.array([33, 500, 16], dtype=np.int32)
    pb = wl.make_paged_batch(lens, 4, 4, 128, dtype="bf16", seed=9, spare_blocks=2)
    d = to_device(pb)
    out = torch.empty_like(d["q"])
    params = als.attn_params(d["q"], d["k"], d["bt"], out, chunk_tokens=128)
    ws = torch.empty(lib.decode_attention_workspace(params, -1), dtype=torch.uint8, device="cuda")
    cks = torch.zeros(256, dtype=torch.int32, device="cuda")
    lib.kv_read_sweep(d["k"], d["v"], d["bt"], d["lens"], cks, params, ws, kv_lens_host=lens)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(cks.cpu().numpy().view(np.uint32))
    want = np.uint32(0)
    for b in range(3):
        for j in range((lens[b] + 15) // 16):
            blk = pb.block_table[b, j]
            want ^= np.bitwise_xor.reduce(pb.k_blocks[blk].reshape(-1).view(np.uint32))
            want ^= np.bitwise_xor.reduce(pb.v_blocks[blk].reshape(-1).view(np.uint32))
    assert got == want


@pytest.mark.parametrize("Hq,Hkv", [(4, 1), (8, 2), (8, 1), (16, 1), (32, 2), (32, 1), (24, 1), (5, 1), (12, 1),
                                    (17, 1), (64, 2), (64, 1), (40, 1), (96, 1), (48, 1)])
def test_matrix_core_path_matches_oracle_and_vector_path(lib, Hq, Hkv):
    """bf16, D=128 grouped-query shapes: the MFMA kernel (default for groups
    >= 4) and the vector-ALU kernel (forced) both meet the bf16 tolerance."""
    from paper_2605_23389_amd import binding as als
    lens = np.array([1, 3, 16, 17, 31, 64, 65, 100, 255, 256, 257, 300, 513, 1000, 1037], dtype=np.int32)
    for poison in ("nan", "big"):
        pb = wl.make_paged_batch(lens, Hq, Hkv, 128, dtype="bf16", seed=Hq * 3 + Hkv, spare_blocks=2,
                                 poison=poison, extra_table_cols=2)
        ref = oracle_out(pb)
        dev = to_device(pb)
        for chunk in (0, 64, 512):
            got = run_attention(lib, pb, out_dtype="fp32", chunk_tokens=chunk, dev=dev)
            # far inside the bf16 budget: the kernel's own error is that of
            # 16-bit weights and fp32 accumulation
            check_parity(got, ref, pb, out_dtype="fp32")
        valu = run_attention(lib, pb, out_dtype="fp32", dev=dev, flags=als.ATTN_NO_MFMA)
        check_parity(valu, ref, pb, out_dtype="fp32", flags=als.ATTN_NO_MFMA)


def test_matrix_core_path_one_hot_and_mean_limits(lib):
    """Single-token requests return v exactly and identical keys give the mean
    of V also through the MFMA kernel (bf16 probabilities)."""
    pb = wl.make_paged_batch(np.ones(2, dtype=np.int32), 8, 1, 128, dtype="bf16", seed=12, poison="nan")
    got = run_attention(lib, pb, out_dtype="fp32")
    v = pb.as_float("v_blocks").astype(np.float64)
    for b in range(2):
        for h in range(8):
            assert np.array_equal(got[b, h], v[pb.block_table[b, 0], 0, 0])
    pb = wl.make_paged_batch(np.array([128], dtype=np.int32), 8, 1, 128, dtype="bf16", seed=13)
    k0 = pb.k_blocks[pb.block_table[0, 0], :, 0, :].copy()
    for j in range(8):
        pb.k_blocks[pb.block_table[0, j]] = k0[:, None, :]
    got = run_attention(lib, pb, out_dtype="fp32", chunk_tokens=64)
    rows = np.concatenate([pb.as_float("v_blocks")[pb.block_table[0, j]] for j in range(8)], axis=1)
    assert np.abs(got[0] - rows.astype(np.float64).mean(axis=1)).max() <= 1e-5


def test_randomised_shapes_against_oracle(lib):
    """Seeded random sweep over batch size, lengths, head layout, head_dim,
    dtype, output dtype, chunking, poison and host-length use."""
    from paper_2605_23389_amd import binding as als
    rng = np.random.default_rng(2024)
    for trial in range(40):
        dtype = ["fp32", "bf16"][int(rng.integers(0, 2))]
        D = [64, 128][int(rng.integers(0, 2))]
        Hkv = int(rng.choice([1, 2, 3, 4, 8]))
        G = int(rng.choice([1, 1, 2, 3, 4, 5, 8, 16, 20, 32]))
        B = int(rng.integers(1, 24))
        hi = int(rng.choice([40, 300, 1500, 5000]))
        lens = rng.integers(1, hi + 1, B).astype(np.int32)
        pb = wl.make_paged_batch(lens, Hkv * G, Hkv, D, dtype=dtype, seed=1000 + trial,
                                 spare_blocks=int(rng.integers(0, 3)),
                                 poison=[None, "nan", "inf", "big"][int(rng.integers(0, 4))],
                                 extra_table_cols=int(rng.integers(0, 4)))
        chunk = int(rng.choice([0, 0, 16, 64, 208, 512, 4096]))
        flags = int(rng.choice([0, 0, als.ATTN_NO_MFMA]))
        out_dtype = "fp32" if dtype == "fp32" or rng.random() < 0.7 else "bf16"
        ref = oracle_out(pb)
        got = run_attention(lib, pb, out_dtype=out_dtype, chunk_tokens=chunk, flags=flags,
                            host_lens=bool(rng.integers(0, 2)))
        check_parity(got, ref, pb, out_dtype=out_dtype, flags=flags,
                     what=str((trial, dtype, D, Hkv, G, B, chunk, flags)))


@pytest.mark.parametrize("host_lens", [True, False])
def test_device_built_plan_with_thousands_of_items(lib, host_lens):
    """More items than the argument-borne plan holds (960): the plan kernel
    builds the item table on several workgroups, full chunks first and the
    requests' last chunks after them, and every partial lands in its request's
    slots.  Lengths include exact multiples of the chunk and one-token requests."""
    rng = np.random.default_rng(77)
    lens = rng.integers(1, 700, 300).astype(np.int32)
    lens[:6] = [64, 128, 1, 63, 65, 640]
    pb = wl.make_paged_batch(lens, 2, 1, 64, dtype="fp32", seed=77, poison="nan", spare_blocks=1)
    assert sum((int(l) + 63) // 64 for l in lens) > 960
    _check(lib, pb, chunk_tokens=64, host_lens=host_lens)
    pb16 = wl.make_paged_batch(lens, 8, 2, 128, dtype="bf16", seed=78, poison="nan")
    _check(lib, pb16, chunk_tokens=64, host_lens=host_lens, out_dtype="fp32")   # matrix-core kernel


def test_more_requests_than_the_inline_plan_holds_none_split(lib):
    """1500 short requests, one chunk each: no plan at all (item i is request
    i), a grid that is not a multiple of the XCD interleave, fp32 and bf16."""
    rng = np.random.default_rng(91)
    lens = rng.integers(1, 100, 1500).astype(np.int32)
    pb = wl.make_paged_batch(lens, 2, 2, 64, dtype="fp32", seed=91, poison="nan", spare_blocks=1)
    _check(lib, pb)
    pb = wl.make_paged_batch(lens[:1111], 3, 1, 128, dtype="bf16", seed=92, poison="big")
    _check(lib, pb, out_dtype="fp32")


def test_one_very_long_request(lib):
    """A single request far longer than the largest chunk (4096 tokens): 18
    chunks of 64 tiles per wave, merged by the combine kernel; ragged tail."""
    lens = np.array([70003], dtype=np.int32)
    pb = wl.make_paged_batch(lens, 2, 2, 128, dtype="bf16", seed=93, poison="nan", spare_blocks=1)
    _check(lib, pb, out_dtype="fp32")
    _check(lib, pb, out_dtype="fp32", chunk_tokens=4096)
    pb = wl.make_paged_batch(lens, 8, 1, 128, dtype="bf16", seed=94, poison="nan")     # matrix-core kernel
    _check(lib, pb, out_dtype="fp32")


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2)])
def test_device_plan_sized_by_a_block_bound(lib, Hq, Hkv):
    """Calls without host lengths may carry the caller's bound on the number of blocks the batch
    holds: the launch is sized for it instead of batch * row length.  Exact bound, generous bound,
    a wide block table (so that the worst case is far larger), split and unsplit requests."""
    import torch
    from paper_2605_23389_amd import binding as als
    rng = np.random.default_rng(314)
    lens = np.concatenate([rng.integers(1, 3000, 20), [1, 16, 17, 4096]]).astype(np.int32)
    pb = wl.make_paged_batch(lens, Hq, Hkv, 128, dtype="bf16", seed=314, poison="nan", spare_blocks=1,
                             extra_table_cols=300)
    ref = oracle_out(pb)
    d = to_device(pb)
    exact = int(((lens.astype(np.int64) + 15) // 16).sum())
    for bound in (exact, 3 * exact):
        for chunk in (0, 64):
            out = torch.full(d["q"].shape, float("nan"), dtype=torch.float32, device="cuda")
            params = als.attn_params(d["q"], d["k"], d["bt"], out, chunk_tokens=chunk, total_blocks_bound=bound)
            ws = torch.empty(lib.decode_attention_workspace(params, bound * 16), dtype=torch.uint8, device="cuda")
            assert ws.numel() < lib.decode_attention_workspace(params, -1)
            lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out, workspace=ws, params=params)
            torch.cuda.synchronize()
            check_parity(out.double().cpu().numpy(), ref, pb, out_dtype="fp32", what=f"bound {bound} chunk {chunk}")
    params = als.attn_params(d["q"], d["k"], d["bt"], out, total_blocks_bound=-1)
    with pytest.raises(als.AlignedServeError):
        lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out, params=params)


def test_device_length_beyond_the_table_row_is_cut_to_it(lib):
    """Without host lengths nothing is validated: a device length larger than the block-table
    row can hold is cut to the row (documented: a wrong answer for that request, never a read
    outside its row), and the other requests are unaffected."""
    import torch
    lens = np.array([48, 80, 33], dtype=np.int32)
    pb = wl.make_paged_batch(lens, 4, 2, 128, dtype="bf16", seed=55, spare_blocks=1)
    cap = pb.block_table.shape[1] * 16
    assert cap == 80
    d = to_device(pb)
    d["lens"][0] = cap + 1000                     # request 0 claims more than its row holds
    out = torch.full(d["q"].shape, float("nan"), dtype=torch.float32, device="cuda")
    lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out, chunk_tokens=32)
    torch.cuda.synchronize()
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all()
    ref = oracle_out(pb)
    assert np.abs(got[1:] - ref[1:]).max() <= 1e-5
    # request 0: attention over the whole row (its own 48 tokens, then the row's remaining entries)
    pb.kv_lens = np.array([cap, 80, 33], dtype=np.int32)
    ref_cut = oracle_out(pb)
    assert np.abs(got[0] - ref_cut[0]).max() <= 1e-5


@pytest.mark.parametrize("Hq,Hkv,dtype", [(4, 4, "fp32"), (4, 4, "bf16"), (8, 1, "bf16"), (32, 1, "bf16")])
def test_peaked_and_flat_softmax_at_length(lib, Hq, Hkv, dtype):
    """The two ends of the softmax: scale 1 (scores with a spread of about +-35, weights close to
    one-hot, outputs of order 1 -- the running maximum moves often and rescaling matters) and
    scale 1e-3 (weights almost uniform over thousands of tokens -- the sum l is large), through
    split and unsplit launches of both kernels."""
    lens = np.array([5000, 1, 777, 4096, 18], dtype=np.int32)
    pb = wl.make_paged_batch(lens, Hq, Hkv, 128, dtype=dtype, seed=808, poison="nan", spare_blocks=1)
    dev = to_device(pb)
    for scale in (1.0, 1e-3):
        ref = oracle_out(pb, scale=scale)
        for chunk in (0, 256):
            got = run_attention(lib, pb, out_dtype="fp32", chunk_tokens=chunk, scale=scale, dev=dev)
            check_parity(got, ref, pb, out_dtype="fp32", what=f"scale {scale} chunk {chunk}")
    peaked = oracle_out(pb, scale=1.0)
    assert np.abs(peaked[0]).max() > 0.5          # the peaked case really is near one-hot: outputs of order 1


@pytest.mark.parametrize("dtype,out_dtype", [("bf16", "fp16"), ("fp32", "bf16"), ("fp32", "fp16")])
def test_output_type_is_independent_of_the_input_type(lib, dtype, out_dtype):
    lens = np.array([1, 40, 300, 1025], dtype=np.int32)
    for Hq, Hkv in ((4, 4), (8, 1)):
        pb = wl.make_paged_batch(lens, Hq, Hkv, 128, dtype=dtype, seed=99, poison="nan", spare_blocks=1)
        ref = oracle_out(pb)
        for chunk in (0, 128):
            got = run_attention(lib, pb, out_dtype=out_dtype, chunk_tokens=chunk)
            check_parity(got, ref, pb, out_dtype=out_dtype, what=f"{dtype}->{out_dtype} {Hq}/{Hkv} chunk {chunk}")
