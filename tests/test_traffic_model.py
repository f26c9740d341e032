"""The byte model behind the roofline numbers, pinned to the paper's printed
arithmetic (Section 3.2: about 512 KB of KV per token for Llama2-7B in 16-bit;
Table 1: 2*s*h KV elements per generated token)."""
import json
import os

import numpy as np

from paper_2605_23389_amd import traffic

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_kv_bytes_per_token_matches_the_paper():
    g = json.load(open(os.path.join(GOLD, "kv_bytes_per_token.json")))
    per_tok = traffic.kv_bytes_per_token(g["num_kv_heads"], g["head_dim"], g["elem_bytes"], g["layers"])
    assert per_tok == g["bytes_per_token_all_layers"] == 512 * 1024
    assert traffic.kv_bytes_per_token(g["num_kv_heads"], g["head_dim"], g["elem_bytes"]) == g["bytes_per_token_per_layer"]
    assert round(2e12 / per_tok / 1e6) == g["tokens_in_2TB_approx_millions"]


def test_attention_bytes_is_2sh_plus_small_terms():
    lens = np.array([100, 1000, 17])
    h = 32 * 128
    b = traffic.attention_bytes(lens, 32, 32, 128, elem_bytes=2, out_bytes=2)
    kv = 2 * int(lens.sum()) * h * 2          # Table 1: 2*s*h elements, 2 bytes each
    assert b - kv == 3 * h * 4 + (7 + 63 + 2) * 4 + 3 * 4
    # GQA: KV counted once per KV head
    assert traffic.attention_bytes(lens, 64, 8, 128) - 3 * 64 * 128 * 4 - 75 * 4 == 2 * int(lens.sum()) * 8 * 128 * 2
    assert traffic.attention_flops(lens, 32, 128) == int(lens.sum()) * 32 * 4 * 128
