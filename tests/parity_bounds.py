"""Bounds the GPU parity tests assert, and why there are two of them.

The contract (the build's stated tolerance) is a max-abs error of 1e-5 for
fp32 inputs and 1.5e-2 for bf16 inputs with fp32 accumulation.  For N(0,1)
inputs the Eq. 2 output of a request of L tokens has magnitude about
sqrt(e / L): 0.026 at 4096 tokens, 0.009 at 32768.  An absolute 1.5e-2 is then
as large as the signal -- an all-zero output, a dropped split-KV chunk or a
dropped 16-token tile would pass (tests/test_oracle_attention.py shows this on
the CPU).  The tests therefore also assert what the arithmetic of the kernels
gives, which can fail:

  fp32 output (isolates the kernel's own error; inputs are consumed exactly):
    vector-ALU kernel, any input type : fp32 products and sums     -> 1e-5
    matrix-core kernel, bf16 inputs   : weights as two bf16 terms  -> 1e-4
    matrix-core kernel, fp16 inputs   : weights as two fp16 terms  -> 2e-5
  16-bit output: the same, plus half an ulp of the output format per element
    (2^-9 relative for bf16, 2^-12 for fp16; bounded here by 2^-8 / 2^-11 of
    |ref| to leave room for a value that rounds across a binade).

No GPU is needed to import this module.
"""
import numpy as np

CONTRACT = {"fp32": 1e-5, "bf16": 1.5e-2}

OUT_ROUNDING = {"fp32": 0.0, "bf16": 2.0 ** -8, "fp16": 2.0 ** -11}


def uses_matrix_core(dtype: str, head_dim: int, num_q_heads: int, num_kv_heads: int,
                     no_mfma: bool = False) -> bool:
    """The documented kernel-selection rule of as_decode_attention: 16-bit
    inputs, head_dim 128, at least 4 query heads per KV head, and a group that
    is at most 32 or a multiple of 8."""
    g = num_q_heads // num_kv_heads
    if dtype == "fp32" or head_dim != 128 or g < 4 or no_mfma:
        return False
    return g <= 32 or g % 8 == 0


def kernel_bound(dtype: str, matrix_core: bool) -> float:
    if not matrix_core:
        return 1e-5
    return 1e-4 if dtype == "bf16" else 2e-5


def elementwise_bound(ref: np.ndarray, dtype: str, out_dtype: str, matrix_core: bool) -> np.ndarray:
    """Per-element error allowed for an output of type out_dtype."""
    kb = kernel_bound(dtype, matrix_core)
    return kb + OUT_ROUNDING[out_dtype] * (np.abs(ref) + kb)


def assert_parity(got: np.ndarray, ref: np.ndarray, dtype: str, out_dtype: str, matrix_core: bool,
                  what: str = "") -> float:
    """Asserts the tight bound (and the contract beside it); returns the
    max-abs error."""
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    worst = float(err.max()) if err.size else 0.0
    excess = err - elementwise_bound(ref, dtype, out_dtype, matrix_core)
    assert (excess <= 0).all(), (f"{what}: max-abs err {worst:.3e}, over the "
                                 f"{'matrix-core' if matrix_core else 'vector'} bound by {float(excess.max()):.3e}")
    # the contract for fp32 inputs (1e-5) is stated for fp32 results; a 16-bit result of fp32
    # inputs carries its output rounding, which the element-wise bound above already limits
    if dtype in CONTRACT and not (dtype == "fp32" and out_dtype != "fp32"):
        assert worst <= CONTRACT[dtype], f"{what}: max-abs err {worst:.3e} over the contract"
    return worst
