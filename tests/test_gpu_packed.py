"""GPU parity of the bitmap-packed value path (through the C ABI): the packed array and its per-block
offsets bit for bit against the reference converter's, and fs_spmm_packed bit for bit against fs_spmm
(the two feed identical operands to the matrix cores) as well as against the oracle."""
import ctypes
import os

import numpy as np
import pytest

import oracle
from gpu_util import check_close, from_dev_bits, to_dev, upload_csr
from workloads import csr_from_coo, dense, make_config, random_csr, stream

pytestmark = pytest.mark.gpu
TOL = 1e-2


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2412_11007_amd as fs
    fs.load_library()  # raises if the HIP library is missing: there is no fallback
    return fs


def unpack_buffer(fs, fmt, buf):
    """(blk_ofs, packed values) out of the library's buffer; its layout: offsets first, values in the last
    256-byte-aligned region (nnz elements and 16 spare bytes)."""
    raw = buf.cpu().numpy()
    n_blocks = fmt.c.n_blocks
    ofs = raw[: 4 * (n_blocks + 1)].view(np.int32)
    vals_region = ((fmt.c.nnz * 2 + 16 + 255) // 256) * 256
    vals = raw[raw.shape[0] - vals_region:][: 2 * fmt.c.nnz].view(np.uint16)
    return ofs, vals


def check(fs, A, V, chunk, N, seed):
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, torch_dtype=va.dtype, V=V, chunk=chunk)
    buf = fs.fs_pack_values(fmt)
    ref_fmt = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, fmt.V, 32)
    ref_ofs, ref_packed = oracle.pack_ref(ref_fmt, A.vals)
    ofs, packed = unpack_buffer(fs, fmt, buf)
    assert np.array_equal(ofs, ref_ofs)
    assert np.array_equal(packed, ref_packed)
    B = dense(A.K, N, "n01", A.dtype, stream(seed, 70, N))
    Bd = to_dev(B.bits, A.dtype)
    C_packed = from_dev_bits(fs.fs_spmm_packed(fmt, buf, Bd))
    C_plain = from_dev_bits(fs.fs_spmm(fmt, Bd))
    assert np.array_equal(C_packed, C_plain)
    return fmt, C_packed, B


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("N,chunk", [(8, 0), (64, 32), (72, 0), (128, 64), (136, 0), (256, 32)])
def test_packed_small(fs, V, dtype, N, chunk):
    A = random_csr(203, 150, 0.15, dtype, seed=V + N, empty_rows=0.2)
    fmt, C, B = check(fs, A, V, chunk, N, seed=V + N)
    ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, dtype)
    check_close(C, ref, S, dtype, "packed spmm V=%d N=%d" % (V, N))


@pytest.mark.parametrize("seed", range(int(os.environ.get("FS_SWEEP_CASES", "10"))))
def test_packed_random(fs, seed):
    rng = np.random.default_rng(300 + seed)
    M = int(rng.choice([1, 7, 9, 64, 257, 600])); K = int(rng.choice([1, 33, 200, 4000]))
    dens = float(rng.choice([0.002, 0.05, 0.4, 0.95]))
    A = random_csr(M, K, dens, "f16" if seed % 2 else "bf16", seed=900 + seed, empty_rows=float(rng.choice([0.0, 0.5])))
    check(fs, A, (4, 8, 16)[seed % 3], int(rng.choice([0, 32, 160])), int(rng.choice([16, 64, 128, 200])), seed)


def test_packed_hub_rows(fs):
    rng = np.random.default_rng(5)
    M, K = 70, 6000
    rows, cols = [], []
    for i in range(M):
        deg = 3000 if i in (3, 41) else (900 if i == 20 else int(rng.integers(0, 12)))
        rows.append(np.full(deg, i)); cols.append(rng.choice(K, size=deg, replace=False))
    A = csr_from_coo(M, K, np.concatenate(rows), np.concatenate(cols), "n01", "f16", rng)
    fmt, _, _ = check(fs, A, 8, 64, 128, seed=1)
    assert fmt.n_split_windows > 0


@pytest.mark.parametrize("name", ["cfg2_rmat16", "cfg4_rmat20"])
def test_packed_full_size(fs, name):
    cfg = make_config(name)
    A = cfg["A"]
    B = cfg["spmm"][0]
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, torch_dtype=va.dtype)
    buf = fs.fs_pack_values(fmt)
    ref_fmt = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, fmt.V, 32)
    ref_ofs, ref_packed = oracle.pack_ref(ref_fmt, A.vals)
    ofs, packed = unpack_buffer(fs, fmt, buf)
    assert np.array_equal(ofs, ref_ofs) and np.array_equal(packed, ref_packed)
    Bd = to_dev(B.bits, A.dtype)
    C = from_dev_bits(fs.fs_spmm_packed(fmt, buf, Bd))
    assert np.array_equal(C, from_dev_bits(fs.fs_spmm(fmt, Bd)))
    rows = np.unique(np.concatenate([np.argsort(np.diff(A.rowptr))[-4:], np.random.default_rng(2).integers(0, A.M, 300)]))
    ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, A.dtype, rows=rows)
    check_close(C[rows], ref, S, A.dtype, "packed spmm, full size, sampled rows")


def test_packed_new_values_and_errors(fs):
    import torch
    A = random_csr(120, 90, 0.2, "f16", seed=8)
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, torch_dtype=va.dtype, V=8)
    # pack another value array of the same pattern (here: SDDMM scores)
    X = to_dev(dense(A.M, 16, "n01", "f16", stream(2, 71, 0)).bits, "f16")
    Y = to_dev(dense(A.K, 16, "n01", "f16", stream(2, 71, 1)).bits, "f16")
    scores = fs.fs_sddmm(fmt, X, Y)
    buf = fs.fs_pack_values(fmt, vals=scores)
    H = to_dev(dense(A.K, 64, "n01", "f16", stream(2, 71, 2)).bits, "f16")
    assert np.array_equal(from_dev_bits(fs.fs_spmm_packed(fmt, buf, H)), from_dev_bits(fs.fs_spmm(fmt, H, vals=scores)))
    lib = fs.load_library()
    need = ctypes.c_size_t(0)
    assert lib.fs_pack_bytes(ctypes.byref(fmt.c), ctypes.byref(need)) == 0
    small = torch.empty(need.value - 256, dtype=torch.uint8, device="cuda")
    assert lib.fs_pack_values(ctypes.byref(fmt.c), None, small.data_ptr(), small.numel(), None) == 4
    assert lib.fs_pack_values(ctypes.byref(fmt.c), None, buf.data_ptr() + 16, buf.numel(), None) == 1
    assert lib.fs_spmm_packed(ctypes.byref(fmt.c), buf.data_ptr() + 16, H.data_ptr(), 64, 64, H.data_ptr(), 64, None, 0, None) == 1


def test_packed_strided_operands(fs):
    import torch
    A = random_csr(150, 120, 0.2, "f16", seed=61, empty_rows=0.1)
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, torch_dtype=va.dtype, V=8, chunk=32)
    N = 72
    B = to_dev(dense(A.K, N, "n01", "f16", stream(4, 72, 0)).bits, "f16")
    Bbig = torch.full((A.K, N + 24), 3.0, dtype=B.dtype, device="cuda"); Bbig[:, :N] = B
    Cbig = torch.full((A.M, N + 8), 7.0, dtype=B.dtype, device="cuda")
    fs.fs_spmm_packed(fmt, fs.fs_pack_values(fmt), Bbig[:, :N], out=Cbig[:, :N])
    assert (Cbig[:, N:] == 7.0).all(), "wrote outside the M x N region"
    assert np.array_equal(from_dev_bits(Cbig[:, :N]), from_dev_bits(fs.fs_spmm(fmt, B)))
