"""Shared helpers for the tests: torch <-> oracle value conversion and the parity metrics."""

import numpy as np
import torch

from oracle import numerics


def to_oracle(t: torch.Tensor) -> np.ndarray:
    """Exact values of a tensor as int64 / float64 (bfloat16 goes through its bit pattern)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).numpy().view(np.uint16)
        return numerics.bf16_bits_to_f64(bits)
    if t.dtype == torch.float8_e4m3fn:
        return numerics.e4m3_bits_to_f64(t.view(torch.uint8).numpy())
    if t.dtype in (torch.int8, torch.int32, torch.int64):
        return t.numpy().astype(np.int64)
    return t.numpy().astype(np.float64)


def expected_storage(ref: np.ndarray, dtype: torch.dtype) -> np.ndarray:
    """Round an oracle result (int64 / float64) to the storage type of the GPU output."""
    if dtype == torch.int32:
        return numerics.to_i32_checked(ref).astype(np.int64)
    if dtype == torch.int8:
        assert ref.min() >= -128 and ref.max() <= 127
        return ref.astype(np.int64)
    if dtype == torch.float32:
        return numerics.round_to_f32(ref).astype(np.float64)
    if dtype == torch.bfloat16:
        return numerics.round_to_bf16_value(ref)
    raise TypeError(dtype)


def rel_error(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |g_i - r_i| / max(|r_i|, 1e-3 * max|r|): relative error with a floor for outputs near zero."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    floor = 1e-3 * np.abs(ref).max()
    denom = np.maximum(np.abs(ref), max(floor, 1e-30))
    return float((np.abs(got - ref) / denom).max())


def fp8_slack(a0: np.ndarray, a1: np.ndarray) -> np.ndarray:
    """Absolute error allowance for contractions of 8-bit floats, per result element.

    The 32x32x64 MFMA adds the 64 products of a step after aligning them to the largest exponent
    among them with a limited number of bits: a small product next to large ones loses low bits
    (or vanishes), which fp32 accumulation of exact products would keep.  Measured on random
    operands the error stays below 3.1e-5 of sum_k |a_k b_k|; the tests allow 2^-13 (1.2e-4) of
    that sum on top of the relative tolerance.  a0 (I,K), a1 (J,K) as float64 -> (I,J)."""
    return 2.0 ** -13 * (np.abs(a0) @ np.abs(a1).T)


def assert_parity(got_t: torch.Tensor, ref: np.ndarray, float_tol: float = 1e-2, what: str = "", slack=None):
    """Bit-exact for integer outputs; max relative error <= float_tol for float outputs (after an
    optional per-element absolute allowance `slack`, see fp8_slack)."""
    got = to_oracle(got_t)
    want = expected_storage(np.asarray(ref), got_t.dtype).reshape(np.shape(ref))
    assert got.shape == want.shape, (what, got.shape, want.shape)
    got, want = np.atleast_1d(got), np.atleast_1d(want)           # results with no dimensions at all
    if got_t.dtype in (torch.int8, torch.int32):
        bad = np.nonzero(got != want)
        assert bad[0].size == 0, f"{what}: {bad[0].size} integer mismatches, first at {[b[0] for b in bad]}"
    else:
        assert np.isfinite(got).all() or not np.isfinite(want).all(), what + ": non-finite output"
        if slack is not None:
            excess = np.maximum(np.abs(got - want) - np.asarray(slack, dtype=np.float64).reshape(want.shape), 0.0)
            got = want + np.sign(got - want) * excess
        err = rel_error(got, want)
        assert err <= float_tol, f"{what}: max relative error {err:.3e} > {float_tol}"
