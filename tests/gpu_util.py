"""Helpers shared by the GPU parity tests: move a seeded PagedBatch to the
device, run the C-ABI attention on it, fetch the result as float64, and
compare it with the oracle under the bounds of tests/parity_bounds.py."""
import numpy as np

from tests import parity_bounds as pbnd


def to_device(pb):
    import torch
    dev = torch.device("cuda:0")

    def up(a):
        if pb.dtype in ("bf16", "fp16"):
            tdt = torch.bfloat16 if pb.dtype == "bf16" else torch.float16
            return torch.from_numpy(a.view(np.int16)).to(dev).view(tdt)
        return torch.from_numpy(a).to(dev)

    return dict(q=up(pb.q), k=up(pb.k_blocks), v=up(pb.v_blocks),
                bt=torch.from_numpy(pb.block_table).to(dev),
                lens=torch.from_numpy(pb.kv_lens).to(dev))


def run_attention(lib, pb, out_dtype=None, chunk_tokens=0, host_lens=True, scale=0.0, dev=None, flags=0):
    import torch
    d = dev or to_device(pb)
    odt = {"fp32": torch.float32, "bf16": torch.bfloat16, "fp16": torch.float16}[out_dtype or pb.dtype]
    out = torch.full(d["q"].shape, float("nan"), dtype=odt, device=d["q"].device)
    lib.decode_attention(d["q"], d["k"], d["v"], d["bt"], d["lens"], out,
                         kv_lens_host=pb.kv_lens if host_lens else None,
                         chunk_tokens=chunk_tokens, scale=scale, flags=flags)
    torch.cuda.synchronize()
    return out.to(torch.float64).cpu().numpy()


def oracle_out(pb, scale=None):
    from oracle import attention as oa
    return oa.decode_attention(pb.as_float("q"), pb.as_float("k_blocks"), pb.as_float("v_blocks"),
                               pb.block_table, pb.kv_lens, scale=scale)


def check_parity(got, ref, pb, out_dtype=None, flags=0, what=""):
    """Tight (kernel-arithmetic) bound and the contract, for a result of the
    library's own kernel choice on this batch's shape."""
    Hq, D = pb.q.shape[1], pb.q.shape[2]
    Hkv = pb.k_blocks.shape[1]
    mc = pbnd.uses_matrix_core(pb.dtype, D, Hq, Hkv, no_mfma=bool(flags & 2))
    return pbnd.assert_parity(got, ref, pb.dtype, out_dtype or pb.dtype, mc, what)
