"""A seeded sweep over small random problems: shapes, densities, window heights, item sizes, widths and
both element types, every operator against the oracle.  Catches what the hand-picked cases miss (odd tails,
empty windows in odd places, single-row matrices, cut windows of every length)."""
import os

import numpy as np
import pytest

import oracle
from gpu_util import check_close, from_dev_bits, to_dev, upload_csr
from workloads import Csr, bits_to_f64, dense, random_csr, stream

pytestmark = pytest.mark.gpu
TOL = 1e-2


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2412_11007_amd as fs
    fs.load_library()
    return fs


N_CASES = int(os.environ.get("FS_SWEEP_CASES", "48"))  # a longer sweep for occasional soak runs


@pytest.mark.parametrize("seed", list(range(N_CASES)))
def test_random_case(fs, seed):
    rng = np.random.default_rng(1000 + seed)
    M = int(rng.choice([1, 2, 7, 8, 9, 31, 64, 100, 257, 600]))
    K = int(rng.choice([1, 5, 32, 33, 200, 1000, 4000]))
    dens = float(rng.choice([0.002, 0.02, 0.1, 0.4, 0.9]))
    dtype = "f16" if seed % 2 == 0 else "bf16"
    V = (8, 16, 4)[seed % 3]
    chunk = int(rng.choice([0, 32, 64, 160, 1024]))
    N = int(rng.choice([8, 16, 24, 64, 72, 128, 136, 256, 320]))
    d = int(rng.choice([8, 16, 32, 48, 64, 128, 136]))
    A = random_csr(M, K, dens, dtype, seed=5000 + seed, empty_rows=float(rng.choice([0.0, 0.3, 0.8])))
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, torch_dtype=va.dtype, V=V, chunk=chunk)
    ref_fmt = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, V, 32)
    assert np.array_equal(fmt.win_ptr_t().cpu().numpy(), ref_fmt.win_ptr)
    assert np.array_equal(fmt.vec_col_t().cpu().numpy(), ref_fmt.vec_col)
    assert np.array_equal(fmt.csr_to_slot_t().cpu().numpy(), ref_fmt.csr_to_slot)
    assert np.array_equal(from_dev_bits(fmt.vals_blk_t()), ref_fmt.vals_blk)
    # SpMM
    B = dense(K, N, "n01", dtype, stream(seed, 99, 0))
    C = from_dev_bits(fs.fs_spmm(fmt, to_dev(B.bits, dtype)))
    ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, dtype)
    check_close(C, ref, S, dtype, "spmm %r" % ((M, K, dens, V, chunk, N),))
    # SDDMM (+ positions outside the pattern are zero)
    X = dense(M, d, "n01", dtype, stream(seed, 99, 1))
    Y = dense(K, d, "n01", dtype, stream(seed, 99, 2))
    scores = fs.fs_sddmm(fmt, to_dev(X.bits, dtype), to_dev(Y.bits, dtype))
    sref, sS = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, dtype)
    blk = from_dev_bits(scores)
    check_close(blk[ref_fmt.csr_to_slot], sref, sS, dtype, "sddmm %r" % ((M, K, dens, V, chunk, d),))
    other = np.ones(blk.shape[0], dtype=bool)
    other[ref_fmt.csr_to_slot] = False
    assert not blk[other].any()
    # edge softmax of the GPU's own scores, in place
    scale = float(rng.choice([1.0, 0.125, -0.5]))
    gpu_scores = blk[ref_fmt.csr_to_slot].copy()
    att = from_dev_bits(fs.fs_edge_softmax(fmt, scores, out=scores, scale=scale))
    aref = oracle.edge_softmax(A.M, A.rowptr, gpu_scores, dtype, scale=scale)
    if A.nnz:
        check_close(att[ref_fmt.csr_to_slot], aref, aref, dtype, "softmax %r" % ((M, K, dens, V, chunk),))
    assert not att[other].any()
    # gradient of that softmax for a random incoming gradient (in the SDDMM output layout)
    if A.nnz:
        g_csr = dense(1, A.nnz, "n01", dtype, stream(seed, 99, 3)).bits.reshape(-1)
        g_blk = fs.fs_csr_to_blk(fmt, to_dev(g_csr, dtype))
        ds = from_dev_bits(fs.fs_edge_softmax_backward(fmt, scores, g_blk, scale=scale))
        dref, dS = oracle.edge_softmax_backward(A.M, A.rowptr, att[ref_fmt.csr_to_slot], g_csr, dtype, scale=scale)
        check_close(ds[ref_fmt.csr_to_slot], dref, dS, dtype, "softmax gradient %r" % ((M, K, dens, V, chunk),))
        assert not ds[other].any()
    # the same chain as one kernel, against its fp64 definition (B serves as H)
    if d <= 128:
        fused = from_dev_bits(fs.fs_attention(fmt, to_dev(X.bits, dtype), to_dev(Y.bits, dtype), to_dev(B.bits, dtype), scale=scale))
        fref, fS = oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, B.bits, dtype, scale)
        check_close(fused, fref, fS, dtype, "attention %r" % ((M, K, dens, V, chunk, d, N, scale),), stages=2)
    # CSR of the transposed matrix, bit for bit
    got_t = fs.fs_csr_transpose(rp, ci, A.M, A.K)
    for g_arr, r_arr in zip(got_t, oracle.csr_transpose(A.M, A.K, A.rowptr, A.colidx)):
        assert np.array_equal(g_arr.cpu().numpy(), r_arr)


@pytest.mark.parametrize("seed", list(range(max(12, N_CASES // 4))))
def test_random_case_with_hub_rows(fs, seed):
    """Heavy-tailed row lengths: a few rows with thousands of entries among short ones, so that windows are
    cut into many parts (partial tiles, merged softmax statistics) next to runs of tiny windows."""
    from workloads import csr_from_coo
    rng = np.random.default_rng(7000 + seed)
    M = int(rng.choice([300, 1500, 6000]))
    K = int(rng.choice([3000, 20000]))
    deg = np.minimum(np.round(np.exp(rng.normal(1.0, 1.8, size=M))).astype(np.int64), K)
    deg[rng.integers(0, M, size=3)] = min(K, int(rng.choice([900, 2500])))
    deg[rng.random(M) < 0.3] = 0
    rows = np.repeat(np.arange(M), deg)
    cols = np.concatenate([rng.choice(K, size=int(n), replace=False) for n in deg if n > 0]) if rows.size else np.zeros(0, dtype=np.int64)
    dtype = "f16" if seed % 2 == 0 else "bf16"
    A = csr_from_coo(M, K, rows, cols, "n01", dtype, rng)
    V = (8, 16, 4)[seed % 3]
    chunk = int(rng.choice([0, 64, 256]))
    N = int(rng.choice([32, 128, 200]))
    d = int(rng.choice([32, 64]))
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K, torch_dtype=va.dtype, V=V, chunk=chunk)
    if seed < 12:  # the standing cases all have cut windows (a longer sweep may draw a matrix whose hubs were emptied)
        assert fmt.n_split_windows > 0
    ref_fmt = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, V, 32)
    assert np.array_equal(fmt.vec_col_t().cpu().numpy(), ref_fmt.vec_col)
    assert np.array_equal(fmt.csr_to_slot_t().cpu().numpy(), ref_fmt.csr_to_slot)
    B = dense(K, N, "n01", dtype, stream(seed, 100, 0))
    C = from_dev_bits(fs.fs_spmm(fmt, to_dev(B.bits, dtype)))
    ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, dtype)
    check_close(C, ref, S, dtype, "spmm, hub rows")
    X = dense(M, d, "n0_8th", dtype, stream(seed, 100, 1))
    Y = dense(K, d, "n0_8th", dtype, stream(seed, 100, 2))
    scores = fs.fs_sddmm(fmt, to_dev(X.bits, dtype), to_dev(Y.bits, dtype))
    sref, sS = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, dtype)
    gpu_scores = from_dev_bits(scores)[ref_fmt.csr_to_slot].copy()
    check_close(gpu_scores, sref, sS, dtype, "sddmm, hub rows")
    att = from_dev_bits(fs.fs_edge_softmax(fmt, scores, scale=2.0))
    aref = oracle.edge_softmax(A.M, A.rowptr, gpu_scores, dtype, scale=2.0)
    check_close(att[ref_fmt.csr_to_slot], aref, aref, dtype, "softmax, hub rows")
    g_csr = dense(1, A.nnz, "n01", dtype, stream(seed, 100, 3)).bits.reshape(-1)
    ds = from_dev_bits(fs.fs_edge_softmax_backward(fmt, to_dev(att, dtype), fs.fs_csr_to_blk(fmt, to_dev(g_csr, dtype)), scale=2.0))
    dref, dS = oracle.edge_softmax_backward(A.M, A.rowptr, att[ref_fmt.csr_to_slot], g_csr, dtype, scale=2.0)
    check_close(ds[ref_fmt.csr_to_slot], dref, dS, dtype, "softmax gradient, hub rows")
    fused = from_dev_bits(fs.fs_attention(fmt, to_dev(X.bits, dtype), to_dev(Y.bits, dtype), to_dev(B.bits, dtype), scale=2.0))
    fref, fS = oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, B.bits, dtype, 2.0)
    check_close(fused, fref, fS, dtype, "attention, hub rows", stages=2)
    got_t = fs.fs_csr_transpose(rp, ci, A.M, A.K)
    for g_arr, r_arr in zip(got_t, oracle.csr_transpose(A.M, A.K, A.rowptr, A.colidx)):
        assert np.array_equal(g_arr.cpu().numpy(), r_arr)
