"""Helpers for the GPU parity tests: upload / download raw 16-bit tensors, error measure."""
import numpy as np

from workloads import bits_to_f64
from workloads.device import from_dev_bits, to_dev, to_dev_i32, torch_dtype, upload_csr  # noqa: F401


# Half the spacing of the output type's subnormal grid.  A result below the smallest normal number
# (2^-14 for fp16) cannot be stored with a relative error of 2^-11: the stored value is off by up to
# this absolute amount however it was computed, so the comparison grants it on top of the relative bound.
OUTPUT_GRID_FLOOR = {"f16": 2.0 ** -25, "bf16": 2.0 ** -134}


def scaled_error(gpu_bits: np.ndarray, ref: np.ndarray, S: np.ndarray, dtype: str) -> float:
    """max (|gpu - ref| - floor) / S with S = sum |a||b| from the oracle, floor = OUTPUT_GRID_FLOOR.

    Equals the plain relative error wherever nothing cancels and stays
    meaningful where the reference is tiny by cancellation.  Where S == 0 the
    exact result is 0 and the GPU value must be exactly zero.
    """
    got = bits_to_f64(gpu_bits, dtype).reshape(ref.shape)
    zero = S == 0
    assert (got[zero] == 0).all(), "non-zero output where the exact result is 0"
    if zero.all():
        return 0.0
    err = np.maximum(np.abs(got[~zero] - ref[~zero]) - OUTPUT_GRID_FLOOR[dtype], 0.0) / S[~zero]
    return float(err.max())


# The contract: max scaled error 1e-2.  The regression bars are twice the half-ulp of the output type --
# what one rounding of an fp32 sum of exact products can reach plus room for the fp32 summation itself --
# so that a dropped vector in a row of a few hundred entries no longer hides under the contract's bar.
CONTRACT = 1e-2
BAR = {"f16": 2.0 ** -10, "bf16": 2.0 ** -7}


def plain_relative_error(gpu_bits: np.ndarray, ref: np.ndarray, S: np.ndarray, dtype: str) -> float:
    """max |gpu - ref| / |ref| over the entries that did not cancel (|ref| >= 1e-3 * S, S > 0)."""
    got = bits_to_f64(gpu_bits, dtype).reshape(ref.shape)
    keep = (S > 0) & (np.abs(ref) >= 1e-3 * S) & (np.abs(ref) >= 2.0 ** (-14 if dtype == "f16" else -126))
    if not keep.any():
        return 0.0
    return float((np.abs(got[keep] - ref[keep]) / np.abs(ref[keep])).max())


def check_close(gpu_bits: np.ndarray, ref: np.ndarray, S: np.ndarray, dtype: str, what: str = "", stages: int = 1) -> float:
    """Asserts the regression bar (`stages` roundings to the output type on the way) and the contract;
    prints both error measures."""
    err = scaled_error(gpu_bits, ref, S, dtype)
    rel = plain_relative_error(gpu_bits, ref, S, dtype)
    print("\n%s [%s]: scaled error %.3e (bar %.3e, contract %.0e), plain relative error where |ref| >= 1e-3 S: %.3e" % (
        what, dtype, err, stages * BAR[dtype], CONTRACT, rel))
    assert err <= stages * BAR[dtype], (what, dtype, err)
    assert err <= CONTRACT, (what, dtype, err)
    return err
