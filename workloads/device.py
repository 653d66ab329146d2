"""Moving the seeded inputs to and from the GPU as raw 16-bit tensors (torch is only memory here).

Input plumbing only, like the rest of this package: no arithmetic of the method.
"""
import numpy as np


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
