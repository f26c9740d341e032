"""Helpers shared by the GPU parity tests: move a seeded PagedBatch to the
device, run the C-ABI attention on it, and fetch the result as float64."""
import numpy as np


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
