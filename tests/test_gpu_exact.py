"""Exact-arithmetic parity: GPU == oracle BIT FOR BIT.

All stored values and dense entries are small multiples of 1/2, so every product and every partial sum
is exactly representable in fp32 whatever the summation order; the only rounding on either side is the
single one to the 16-bit output type (nearest even).  The oracle's fp64 result, rounded once the same
way, must therefore equal the GPU's bits exactly -- a dropped, doubled or misplaced vector anywhere
(hub windows cut into many parts, the merge of their partial tiles, narrow last blocks, the packed path,
the fused path) changes a sum by at least 1/4 and fails, however long the row is.
"""
import numpy as np
import pytest

import oracle
from gpu_util import from_dev_bits, to_dev, upload_csr
from workloads import Csr, Dense, csr_from_coo, make_config, round_to_bits, stream

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2412_11007_amd as fs
    fs.load_library()
    return fs


def halves(rng, shape, lo, hi, dtype) -> np.ndarray:
    """Raw bits of uniformly drawn multiples of 1/2 in [lo/2, hi/2] (exact in fp16 and bf16)."""
    return round_to_bits((rng.integers(lo, hi + 1, size=shape).astype(np.float32) * np.float32(0.5)), dtype)


def with_exact_values(A: Csr, dtype: str, seed: int) -> Csr:
    """The same pattern with values that are multiples of 1/2 in [-2, 2], explicit zeros included."""
    return Csr(A.M, A.K, A.rowptr, A.colidx, halves(stream(seed, 98, 0), A.nnz, -4, 4, dtype), dtype)


def int_dense(rows, cols, dtype, seed, tid, lim=3) -> Dense:
    """Integer-valued dense operand in [-lim, lim]."""
    return Dense(round_to_bits(stream(seed, 98, tid).integers(-lim, lim + 1, size=(rows, cols)).astype(np.float32), dtype), dtype)


def hub_matrix(M: int, K: int, dtype: str, seed: int) -> Csr:
    """A few rows with thousands of entries (windows cut into dozens of parts), the rest sparse or empty;
    M is not a multiple of any window height."""
    rng = stream(seed, 98, 9)
    rows, cols = [], []
    for r, n in ((1, 6000), (2, 3500), (M - 2, 2100), (M // 2, 900)):
        c = rng.choice(K, size=n, replace=False)
        rows.append(np.full(n, r))
        cols.append(c)
    sparse_rows = rng.integers(0, M, size=4 * M)
    rows.append(sparse_rows)
    cols.append(rng.integers(0, K, size=sparse_rows.shape[0]))
    A = csr_from_coo(M, K, np.concatenate(rows), np.concatenate(cols), "u11", dtype, stream(seed, 98, 8))
    return with_exact_values(A, dtype, seed)


def expect_spmm(A: Csr, B: Dense) -> np.ndarray:
    ref, _ = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, A.dtype, want_scale=False)
    assert np.abs(ref).max() < 60000  # no overflow of the 16-bit output on either side
    assert np.array_equal(ref * 4, np.rint(ref * 4))  # the exact results are multiples of 1/4: nothing was rounded in fp64
    return oracle.round_f64_to_bits(ref, A.dtype).reshape(ref.shape)


def same_bits(got: np.ndarray, want: np.ndarray, what: str):
    """Equal bit patterns (a zero result is +0 on both sides: x + (-x) is +0 under round-to-nearest)."""
    bad = np.nonzero(got.reshape(-1) != want.reshape(-1))[0]
    assert bad.size == 0, "%s: %d of %d outputs differ, first at flat index %d: gpu 0x%04x, expected 0x%04x" % (
        what, bad.size, got.size, bad[0], got.reshape(-1)[bad[0]], want.reshape(-1)[bad[0]])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("N", [128, 256])
def test_hub_matrix_cut_windows_bit_exact(fs, N, V, dtype):
    A = hub_matrix(77, 20000, dtype, seed=V + N)
    B = int_dense(A.K, N, dtype, seed=V + N, tid=1)
    want = expect_spmm(A, B)
    rp, ci, va = upload_csr(A)
    Bd = to_dev(B.bits, dtype)
    for chunk in (64, 0):  # 64: every hub window in dozens of parts (the 32-, 16-, 8- and tail loops of the merge)
        fmt = fs.fs_convert(rp, ci, va, A.M, A.K, V=V, chunk=chunk)
        if chunk:
            assert fmt.n_split_windows >= 3 and fmt.n_split_items >= 100
        same_bits(from_dev_bits(fs.fs_spmm(fmt, Bd)), want, "fs_spmm V=%d N=%d chunk=%d" % (V, N, chunk))
        same_bits(from_dev_bits(fs.fs_spmm_packed(fmt, fs.fs_pack_values(fmt), Bd)), want,
                  "fs_spmm_packed V=%d N=%d chunk=%d" % (V, N, chunk))


@pytest.mark.parametrize("V", [0, 4, 16])
def test_rmat16_full_size_bit_exact(fs, V):
    """The full cfg 2 pattern (hub windows of ten thousand vectors, 378 cut windows at the default
    settings) with exact values: all 65 536 x 128 outputs, plain and packed."""
    c = make_config("cfg2_rmat16")
    A = with_exact_values(c["A"], "f16", seed=21)
    B = int_dense(A.K, 128, "f16", seed=21, tid=1)
    want = expect_spmm(A, B)
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, V=V)
    assert fmt.n_split_windows > 0
    Bd = to_dev(B.bits, "f16")
    same_bits(from_dev_bits(fs.fs_spmm(fmt, Bd)), want, "fs_spmm cfg2 V=%d" % fmt.V)
    same_bits(from_dev_bits(fs.fs_spmm_packed(fmt, fs.fs_pack_values(fmt), Bd)), want, "fs_spmm_packed cfg2 V=%d" % fmt.V)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("d", [32, 64, 128, 160])
def test_sddmm_bit_exact(fs, d, V, dtype):
    A = hub_matrix(77, 20000, dtype, seed=V + d)
    X = Dense(halves(stream(V + d, 98, 2), (A.M, d), -2, 2, dtype), dtype)  # multiples of 1/2 in [-1, 1]
    Y = int_dense(A.K, d, dtype, seed=V + d, tid=3, lim=2)
    ref, _ = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, dtype, want_scale=False)
    want = oracle.round_f64_to_bits(ref, dtype)
    rp, ci, _ = upload_csr(A)
    import torch
    fmt = fs.fs_convert(rp, ci, None, A.M, A.K, torch_dtype=torch.float16 if dtype == "f16" else torch.bfloat16, V=V, chunk=64)
    out = fs.fs_sddmm(fmt, to_dev(X.bits, dtype), to_dev(Y.bits, dtype))
    same_bits(from_dev_bits(fs.fs_blk_to_csr(fmt, out)), want, "fs_sddmm V=%d d=%d" % (V, d))
    direct = fs.fs_sddmm(fmt, to_dev(X.bits, dtype), to_dev(Y.bits, dtype), blocked=False)
    same_bits(from_dev_bits(direct), want, "fs_sddmm, CSR-order output, V=%d d=%d" % (V, d))


def test_sddmm_rmat16_full_size_bit_exact(fs):
    c = make_config("cfg2_rmat16")
    A = c["A"]
    d = 32
    X = Dense(halves(stream(5, 98, 2), (A.M, d), -2, 2, "f16"), "f16")
    Y = int_dense(A.K, d, "f16", seed=5, tid=3, lim=2)
    ref, _ = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, "f16", want_scale=False)
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K)
    out = fs.fs_sddmm(fmt, to_dev(X.bits, "f16"), to_dev(Y.bits, "f16"))
    same_bits(from_dev_bits(fs.fs_blk_to_csr(fmt, out)), oracle.round_f64_to_bits(ref, "f16"), "fs_sddmm cfg2")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8])
@pytest.mark.parametrize("d,N", [(32, 128), (64, 256)])
def test_sddmm_spmm_fused_bit_exact(fs, d, N, V, dtype):
    """fs_sddmm_spmm: the scores are multiples of 1/2 of magnitude at most 2 d (d for bf16) -- exact in the
    16-bit type -- and their products with an integer H sum exactly in fp32 as well."""
    A = hub_matrix(77, 20000, dtype, seed=V + d + 1)
    lim = 1 if dtype == "bf16" else 2  # bf16 keeps 8 bits: scores stay multiples of 1/2 below 64
    X = Dense(halves(stream(V + d, 98, 4), (A.M, d), -2, 2, dtype), dtype)
    Y = int_dense(A.K, d, dtype, seed=V + d, tid=5, lim=lim)
    H = int_dense(A.K, N, dtype, seed=V + d, tid=6, lim=2)
    sref, _ = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, dtype, want_scale=False)
    scores = oracle.round_f64_to_bits(sref, dtype)
    from workloads import bits_to_f64
    assert np.array_equal(bits_to_f64(scores, dtype), sref), "the scores must be exact in the 16-bit type"
    ref, _ = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, scores, H.bits, dtype, want_scale=False)
    assert np.abs(ref).max() < 60000
    want = oracle.round_f64_to_bits(ref, dtype).reshape(ref.shape)
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, V=V, chunk=64)
    got = fs.fs_sddmm_spmm(fmt, to_dev(X.bits, dtype), to_dev(Y.bits, dtype), to_dev(H.bits, dtype))
    same_bits(from_dev_bits(got), want, "fs_sddmm_spmm V=%d d=%d N=%d" % (V, d, N))
