"""Helpers for the GPU parity tests: upload / download raw 16-bit tensors, error measure."""
import numpy as np

from workloads import bits_to_f64


# Half the spacing of the output type's subnormal grid.  A result below the smallest normal number
# (2^-14 for fp16) cannot be stored with a relative error of 2^-11: the stored value is off by up to
# this absolute amount however it was computed, so the comparison grants it on top of the relative bound.
OUTPUT_GRID_FLOOR = {"f16": 2.0 ** -25, "bf16": 2.0 ** -134}


def torch_dtype(dtype: str):
    import torch
    return torch.float16 if dtype == "f16" else torch.bfloat16


def to_dev(bits: np.ndarray, dtype: str):
    """uint16 raw bits (any shape) -> device tensor of the matching 16-bit float type."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch_dtype(dtype))


def to_dev_i32(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def from_dev_bits(t) -> np.ndarray:
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def upload_csr(A):
    return to_dev_i32(A.rowptr), to_dev_i32(A.colidx), to_dev(A.vals, A.dtype)


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
