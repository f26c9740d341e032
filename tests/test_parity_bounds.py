"""Negative controls for the GPU parity bounds, on the CPU: mistakes are
planted in the *oracle's* result for long requests and the bound the GPU tests
assert (tests/parity_bounds.py) must reject them, while the contract's absolute
1.5e-2 alone accepts them -- which is why the tight bound exists."""
import math

import numpy as np
import pytest

from oracle import attention as oa
from paper_2605_23389_amd import workloads as wl
from tests import parity_bounds as pbnd


def _request(L, D=128, seed=0):
    rng = np.random.default_rng(seed)
    rb = lambda a: wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(a)).astype(np.float64)
    q = rb(rng.standard_normal(D, dtype=np.float32))
    K = rb(rng.standard_normal((L, D), dtype=np.float32))
    V = rb(rng.standard_normal((L, D), dtype=np.float32))
    return q, K, V


def _rejected(got, ref, matrix_core, out_dtype="fp32"):
    try:
        pbnd.assert_parity(got, ref, "bf16", out_dtype, matrix_core)
    except AssertionError:
        return True
    return False


def _check_planted(wrong, ref):
    assert np.abs(wrong - ref).max() <= pbnd.CONTRACT["bf16"], "the contract alone would have caught it"
    for matrix_core in (False, True):
        assert _rejected(wrong, ref, matrix_core)
        # also with bf16 output: the rounding allowance scales with |ref|
        assert _rejected(wrong, ref, matrix_core, out_dtype="bf16")


@pytest.mark.parametrize("L", [4096, 32768, 70003, 200000])
def test_planted_mistakes_pass_the_contract_alone_but_not_the_tight_bound(L):
    q, K, V = _request(L, seed=L)
    sc = 1.0 / math.sqrt(128)
    ref = oa.attention_single(q, K, V, sc)
    # (a) one 16-token tile dropped from the middle of the request
    keep = np.ones(L, dtype=bool)
    keep[L // 2 // 16 * 16: L // 2 // 16 * 16 + 16] = False
    _check_planted(oa.attention_single(q, K[keep], V[keep], sc), ref)
    # (b) the last 4096-token split-KV chunk dropped
    if L >= 32768:
        _check_planted(oa.attention_single(q, K[:L - 4096], V[:L - 4096], sc), ref)
    # (c) nothing computed at all: |out| ~ sqrt(e / L) sinks below the contract
    if L >= 200000:
        _check_planted(np.zeros_like(ref), ref)
    # and the bound is not so tight that a correct result fails it: fp32
    # rounding of the exact result, and its bf16 rounding for 16-bit output
    assert not _rejected(ref.astype(np.float32).astype(np.float64), ref, False)
    as_bf16 = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(ref.astype(np.float32))).astype(np.float64)
    assert not _rejected(as_bf16, ref, False, out_dtype="bf16")


def test_kernel_selection_rule_helper():
    assert not pbnd.uses_matrix_core("fp32", 128, 8, 1)
    assert not pbnd.uses_matrix_core("bf16", 64, 8, 1)
    assert not pbnd.uses_matrix_core("bf16", 128, 6, 2)
    assert pbnd.uses_matrix_core("bf16", 128, 8, 2)
    assert pbnd.uses_matrix_core("fp16", 128, 64, 8)
    assert pbnd.uses_matrix_core("bf16", 128, 24, 1)       # one workgroup of 24 heads
    assert pbnd.uses_matrix_core("bf16", 128, 20, 1)
    assert pbnd.uses_matrix_core("bf16", 128, 40, 1)       # cut into groups of 8
    assert not pbnd.uses_matrix_core("bf16", 128, 36, 1)   # neither <= 32 nor a multiple of 8
    assert not pbnd.uses_matrix_core("bf16", 128, 8, 1, no_mfma=True)
