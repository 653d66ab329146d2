"""fs_spmm_static -- the entry point for callers that cannot allocate -- against fs_spmm, bit for bit.

Two calls in a row through the C ABI, the second on a smaller input, so that the second one runs over
whatever the first left in the library's fixed workspace.  Collected last on purpose.
"""
import ctypes

import numpy as np
import pytest

from gpu_util import from_dev_bits, to_dev, upload_csr
from workloads import dense, make_config, random_csr, stream

pytestmark = pytest.mark.gpu
STATIC_BYTES = 32 << 20


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2412_11007_amd as fs
    fs.load_library()
    return fs


def _case(fs, A, B, V, chunk):
    """Returns (result of fs_spmm with a caller's workspace, result of fs_spmm_static, workspace bytes)."""
    import torch
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, V=V, chunk=chunk)
    Bd = to_dev(B.bits, B.dtype)
    want = fs.fs_spmm(fmt, Bd)
    got = torch.full_like(want, 3.0)
    print("fs_spmm_static: M=%d nnz=%d N=%d V=%d split_items=%d" % (A.M, A.nnz, B.shape[1], V, fmt.n_split_items), flush=True)
    fs.fs_spmm_static(fmt, Bd, got)
    torch.cuda.synchronize()
    return from_dev_bits(want), from_dev_bits(got), fs.fs_spmm_workspace_bytes(fmt, B.shape[1])


def test_static_workspace_two_calls_second_smaller(fs):
    c = make_config("cfg2_rmat16", shrink=4)  # R-MAT scale 14: hub windows cut into many parts
    A, B = c["A"], c["spmm"][0]
    want, got, need = _case(fs, A, B, 8, 64)
    assert 0 < need <= STATIC_BYTES
    assert np.array_equal(got, want)
    # a smaller problem right after it: fewer and smaller partial tiles over the first call's leftovers
    A2 = random_csr(203, 150, 0.3, "bf16", seed=5, empty_rows=0.2)
    B2 = dense(150, 72, "n01", "bf16", stream(11, 96, 0))
    want2, got2, need2 = _case(fs, A2, B2, 4, 32)
    assert 0 < need2 < need
    assert np.array_equal(got2, want2)
    # and a matrix without cut windows: no workspace at all
    A3 = random_csr(64, 90, 0.05, "f16", seed=6)
    B3 = dense(90, 16, "n01", "f16", stream(11, 96, 1))
    want3, got3, need3 = _case(fs, A3, B3, 8, 0)
    assert need3 == 0 and np.array_equal(got3, want3)


def test_static_workspace_limit_is_an_error(fs):
    """A workspace need above the fixed size is refused before anything is queued."""
    import torch
    c = make_config("cfg2_rmat16", shrink=4)
    A = c["A"]
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, V=16, chunk=32)
    N = 8
    while fs.fs_spmm_workspace_bytes(fmt, N) <= STATIC_BYTES:
        N *= 2
    Bd = torch.zeros((A.K, N), dtype=torch.float16, device="cuda")
    out = torch.full((A.M, N), 3.0, dtype=torch.float16, device="cuda")
    with pytest.raises(fs.FsError) as e:
        fs.fs_spmm_static(fmt, Bd, out)
    assert e.value.code == 5
    torch.cuda.synchronize()
    assert (out == 3.0).all()
    del Bd, out
    torch.cuda.empty_cache()
