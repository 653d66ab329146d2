"""GPU parity of the CSR transposition (through the C ABI) against the CPU oracle -- index work, so
bit for bit -- and of the two gradients of C = A * B computed with it: A^T * dC through a second
converted format, and the sampled dC * B^T through fs_sddmm (bar: 1e-2 relative to sum |a||b|)."""
import ctypes

import numpy as np
import pytest

import oracle
from gpu_util import check_close, from_dev_bits, to_dev, to_dev_i32, upload_csr
from workloads import Csr, csr_from_coo, dense, make_config, random_csr, stream

pytestmark = pytest.mark.gpu
TOL = 1e-2


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2412_11007_amd as fs
    fs.load_library()  # raises if the HIP library is missing: there is no fallback
    return fs


def check_transpose(fs, A):
    rp, ci = to_dev_i32(A.rowptr), to_dev_i32(A.colidx)
    rt, ct, perm = fs.fs_csr_transpose(rp, ci, A.M, A.K)
    ref_rt, ref_ct, ref_perm = oracle.csr_transpose(A.M, A.K, A.rowptr, A.colidx)
    assert np.array_equal(rt.cpu().numpy(), ref_rt)
    assert np.array_equal(ct.cpu().numpy(), ref_ct)
    assert np.array_equal(perm.cpu().numpy(), ref_perm)
    return rt, ct, perm


@pytest.mark.parametrize("M,K,density,seed", [
    (1, 1, 1.0, 0), (1, 700, 0.5, 1), (700, 1, 0.5, 2),   # single row / single column
    (203, 150, 0.15, 3),                                      # one digit pass
    (150, 300, 0.1, 4), (97, 65536, 0.002, 5),                # two passes, K a power of 256
    (400, 70001, 0.001, 6),                                   # three passes
    (3000, 5000, 0.012, 7),                                   # many tiles and a ragged tail
    (64, 64, 0.0, 8),                                         # no stored entries
])
def test_transpose_small(fs, M, K, density, seed):
    A = random_csr(M, K, density, "f16", seed=seed, empty_rows=0.1 if M > 1 else 0.0)
    check_transpose(fs, A)


def test_transpose_hub_columns(fs):
    """A few columns referenced by most rows: equal keys span many tiles, where stability matters."""
    rng = np.random.default_rng(21)
    M, K = 20000, 900
    rows, cols = [], []
    for c in (0, 255, 256, 899):
        r = np.nonzero(rng.random(M) < 0.8)[0]
        rows.append(r); cols.append(np.full(r.shape[0], c))
    r = rng.integers(0, M, 30000); c = rng.integers(0, K, 30000)
    rows.append(r); cols.append(c)
    key = np.unique(np.concatenate(rows).astype(np.int64) * K + np.concatenate(cols))
    A = csr_from_coo(M, K, key // K, key % K, "u01", "f16", rng)
    rt, ct, perm = check_transpose(fs, A)
    again = fs.fs_csr_transpose(to_dev_i32(A.rowptr), to_dev_i32(A.colidx), A.M, A.K)
    assert all(np.array_equal(a.cpu().numpy(), b.cpu().numpy()) for a, b in zip((rt, ct, perm), again))


def test_transpose_mostly_empty_rows(fs):
    """256 consecutive stored entries span thousands of rows: the row of an entry is searched in place."""
    rng = np.random.default_rng(5)
    M, K = 20000, 300
    r = np.sort(rng.choice(M, 900, replace=False)); c = rng.integers(0, K, 900)
    dense_r = np.repeat(np.arange(100, 140), 50); dense_c = np.tile(np.arange(0, 250, 5), 40)
    key = np.unique(np.concatenate([r, dense_r]).astype(np.int64) * K + np.concatenate([c, dense_c]))
    check_transpose(fs, csr_from_coo(M, K, key // K, key % K, "u01", "f16", rng))


@pytest.mark.parametrize("name", ["cfg2_rmat16", "cfg3_stencil", "cfg4_rmat20"])
def test_transpose_full_size(fs, name):
    check_transpose(fs, make_config(name)["A"])


@pytest.mark.parametrize("dtype,V", [("f16", 8), ("bf16", 4), ("f16", 16)])
def test_gradients_of_spmm(fs, dtype, V):
    """C = A * B.  dB = A^T * dC on the converted transpose; dA = (dC * B^T) at A's pattern."""
    M, K, N = 517, 390, 64
    A = random_csr(M, K, 0.05, dtype, seed=31 + V, dist="n01", empty_rows=0.1)
    B = dense(K, N, "n01", dtype, stream(5, 9, V))
    dC = dense(M, N, "n01", dtype, stream(5, 9, V + 100))
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, M, K, torch_dtype=va.dtype, V=V)
    rt, ct, perm = fs.fs_csr_transpose(rp, ci, M, K)
    vt = fs.fs_gather16(va, perm)
    fmt_t = fs.fs_convert(rt, ct, vt, K, M, torch_dtype=va.dtype, V=V)
    dB = fs.fs_spmm(fmt_t, to_dev(dC.bits, dtype))
    # the oracle's own transpose and its own product
    ort, oct_, operm = oracle.csr_transpose(M, K, A.rowptr, A.colidx)
    ref, S = oracle.spmm(K, M, ort, oct_, A.vals[operm], dC.bits, dtype)
    check_close(from_dev_bits(dB), ref, S, dtype, "dB = A^T dC")
    dA = fs.fs_blk_to_csr(fmt, fs.fs_sddmm(fmt, to_dev(dC.bits, dtype), to_dev(B.bits, dtype)))
    ref, S = oracle.sddmm(M, K, A.rowptr, A.colidx, dC.bits, B.bits, dtype)
    check_close(from_dev_bits(dA), ref, S, dtype, "dA = sddmm(dC, B)")


def test_gradient_wrt_dense_operand_full_size(fs):
    """cfg 2 at full size: A^T * dC on sampled rows."""
    cfg = make_config("cfg2_rmat16")
    A = cfg["A"]
    dC = dense(A.M, 128, "n01", "f16", stream(0, 2, 77))
    rp, ci, va = upload_csr(A)
    rt, ct, perm = fs.fs_csr_transpose(rp, ci, A.M, A.K)
    fmt_t = fs.fs_convert(rt, ct, fs.fs_gather16(va, perm), A.K, A.M, torch_dtype=va.dtype)
    dB = from_dev_bits(fs.fs_spmm(fmt_t, to_dev(dC.bits, "f16")))
    ort, oct_, operm = oracle.csr_transpose(A.M, A.K, A.rowptr, A.colidx)
    deg_t = np.diff(ort)
    rows = np.unique(np.concatenate([np.argsort(deg_t)[-8:], np.random.default_rng(3).integers(0, A.K, 600)]))
    ref, S = oracle.spmm(A.K, A.M, ort, oct_, A.vals[operm], dC.bits, "f16", rows=rows)
    check_close(dB[rows], ref, S, "f16", "dB full size, sampled rows")


def test_transpose_argument_errors(fs):
    import torch
    lib = fs.load_library()
    A = random_csr(50, 60, 0.2, "f16", seed=1)
    rp, ci = to_dev_i32(A.rowptr), to_dev_i32(A.colidx)
    need = ctypes.c_size_t(0)
    assert lib.fs_csr_transpose_bytes(A.M, A.K, A.nnz, ctypes.byref(need)) == 0
    assert lib.fs_csr_transpose_bytes(-1, A.K, A.nnz, ctypes.byref(need)) == 1
    assert lib.fs_csr_transpose_bytes(A.M, A.K, 2 ** 31, ctypes.byref(need)) == 5
    rt = torch.empty(A.K + 1, dtype=torch.int32, device="cuda")
    ct = torch.empty(A.nnz, dtype=torch.int32, device="cuda")
    pm = torch.empty(A.nnz, dtype=torch.int32, device="cuda")
    sc = torch.empty(need.value + 256, dtype=torch.uint8, device="cuda")
    call = lambda scratch, nbytes, perm: lib.fs_csr_transpose(
        A.M, A.K, A.nnz, rp.data_ptr(), ci.data_ptr(), rt.data_ptr(), ct.data_ptr(), perm, scratch, nbytes, None)
    assert call(sc.data_ptr(), 1024, pm.data_ptr()) == 4          # scratch too small
    assert call(sc.data_ptr() + 64, need.value, pm.data_ptr()) == 1   # scratch not 256-byte aligned
    assert call(sc.data_ptr(), need.value, None) == 1               # no output for the permutation
    assert call(sc.data_ptr(), need.value, pm.data_ptr()) == 0
    torch.cuda.synchronize()
    assert np.array_equal(pm.cpu().numpy(), oracle.csr_transpose(A.M, A.K, A.rowptr, A.colidx)[2])
