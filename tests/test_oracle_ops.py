"""Pins for the SpMM / SDDMM oracle (CPU only).

Each test ties ``oracle.spmm`` / ``oracle.sddmm`` to something that is not the
oracle itself: hand-computed numbers, numpy's dense matmul on a densified A,
scipy's CSR product, special cases with a known answer, algebraic invariants.
"""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from workloads import Csr, bits_to_f64, dense, random_csr, round_to_bits, stream


def _densify(A: Csr) -> np.ndarray:
    D = np.zeros((A.M, A.K))
    rows = np.repeat(np.arange(A.M), np.diff(A.rowptr))
    D[rows, A.colidx] = bits_to_f64(A.vals, A.dtype)
    return D


def _f16(x):
    return round_to_bits(np.asarray(x, dtype=np.float32), "f16")


def test_widening_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    want16 = bits.view(np.float16).astype(np.float64)
    with np.errstate(invalid="ignore"):
        wantbf = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    for b in range(0, 65536, 7):  # stride keeps it fast; 0, subnormals, inf, nan all hit below too
        for dt, want in (("f16", want16), ("bf16", wantbf)):
            got = oracle.widen(b, dt)
            assert (np.isnan(got) and np.isnan(want[b])) or got == want[b]
    for b in (0x0000, 0x8000, 0x0001, 0x03FF, 0x0400, 0x7BFF, 0x7C00, 0xFC00, 0x7E00, 0x3C00):
        got = oracle.widen(b, "f16")
        assert (np.isnan(got) and np.isnan(want16[b])) or got == want16[b]


def test_golden_small_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "spmm_sddmm_small_example.json")))
    rp = np.array(g["rowptr"], dtype=np.int32)
    ci = np.array(g["colidx"], dtype=np.int32)
    C, S = oracle.spmm(g["M"], g["K"], rp, ci, _f16(g["vals"]), _f16(g["B"]), "f16")
    assert np.array_equal(C, np.array(g["C"]))
    assert np.array_equal(S, np.array(g["S"]))
    out, _ = oracle.sddmm(g["M"], g["K"], rp, ci, _f16(g["X"]), _f16(g["Y"]), "f16")
    assert np.array_equal(out, np.array(g["sddmm_out"]))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("M,K,N,dens", [(5, 9, 3, 0.4), (33, 17, 8, 0.2), (64, 64, 32, 0.1), (40, 64, 1, 0.5)])
def test_spmm_against_dense_brute_force(M, K, N, dens, dtype):
    A = random_csr(M, K, dens, dtype, seed=M + K, empty_rows=0.2)
    B = dense(K, N, "n01", dtype, stream(1, 98, N))
    C, S = oracle.spmm(M, K, A.rowptr, A.colidx, A.vals, B.bits, dtype)
    D = _densify(A)
    Bf = bits_to_f64(B.bits, dtype)
    assert np.allclose(C, D @ Bf, rtol=1e-13, atol=1e-13)
    assert np.allclose(S, np.abs(D) @ np.abs(Bf), rtol=1e-13, atol=1e-13)
    assert (S >= np.abs(C) - 1e-12).all()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("M,K,d,dens", [(7, 11, 5, 0.3), (32, 48, 32, 0.15), (20, 9, 64, 0.5)])
def test_sddmm_against_dense_brute_force(M, K, d, dens, dtype):
    A = random_csr(M, K, dens, dtype, seed=M * K, empty_rows=0.1)
    X = dense(M, d, "n01", dtype, stream(2, 98, 0))
    Y = dense(K, d, "n01", dtype, stream(2, 98, 1))
    out, S = oracle.sddmm(M, K, A.rowptr, A.colidx, X.bits, Y.bits, dtype)
    P = bits_to_f64(X.bits, dtype) @ bits_to_f64(Y.bits, dtype).T  # M x K
    rows = np.repeat(np.arange(M), np.diff(A.rowptr))
    assert np.allclose(out, P[rows, A.colidx], rtol=1e-13, atol=1e-13)
    Pa = np.abs(bits_to_f64(X.bits, dtype)) @ np.abs(bits_to_f64(Y.bits, dtype)).T
    assert np.allclose(S, Pa[rows, A.colidx], rtol=1e-13, atol=1e-13)


def test_sddmm_ignores_the_stored_values_of_A():
    A = random_csr(30, 30, 0.2, "f16", seed=3)
    X = dense(30, 16, "n01", "f16", stream(3, 98, 0))
    Y = dense(30, 16, "n01", "f16", stream(3, 98, 1))
    o1, _ = oracle.sddmm(30, 30, A.rowptr, A.colidx, X.bits, Y.bits, "f16")
    assert o1.shape == (A.nnz,)  # one output per stored entry; the API takes no values at all


def test_spmm_against_scipy_midsize():
    A = random_csr(700, 900, 0.02, "f16", seed=11)
    B = dense(900, 48, "n01", "f16", stream(4, 98, 0))
    C, _ = oracle.spmm(700, 900, A.rowptr, A.colidx, A.vals, B.bits, "f16")
    As = sp.csr_matrix((bits_to_f64(A.vals, "f16"), A.colidx, A.rowptr), shape=(700, 900))
    assert np.allclose(C, As @ bits_to_f64(B.bits, "f16"), rtol=1e-12, atol=1e-12)


def test_identity_A_returns_B_exactly():
    K, N = 50, 24
    rp = np.arange(K + 1, dtype=np.int32)
    ci = np.arange(K, dtype=np.int32)
    one = _f16(np.ones(K))
    B = dense(K, N, "n01", "f16", stream(5, 98, 0))
    C, S = oracle.spmm(K, K, rp, ci, one, B.bits, "f16")
    assert np.array_equal(C, bits_to_f64(B.bits, "f16"))
    assert np.array_equal(S, np.abs(C))


def test_all_ones_pattern_sddmm_is_dense_product():
    M, K, d = 12, 9, 32
    rp = (np.arange(M + 1) * K).astype(np.int32)
    ci = np.tile(np.arange(K), M).astype(np.int32)
    X = dense(M, d, "u11", "f16", stream(6, 98, 0))
    Y = dense(K, d, "u11", "f16", stream(6, 98, 1))
    out, _ = oracle.sddmm(M, K, rp, ci, X.bits, Y.bits, "f16")
    want = bits_to_f64(X.bits, "f16") @ bits_to_f64(Y.bits, "f16").T
    assert np.allclose(out.reshape(M, K), want, rtol=1e-14, atol=1e-14)


def test_invariants_of_spmm():
    M, K, N = 40, 37, 16
    A = random_csr(M, K, 0.15, "f16", seed=21)
    B = dense(K, N, "n01", "f16", stream(7, 98, 0))
    C, _ = oracle.spmm(M, K, A.rowptr, A.colidx, A.vals, B.bits, "f16")
    # a column slice of B gives the same slice of C
    Cs, _ = oracle.spmm(M, K, A.rowptr, A.colidx, A.vals, np.ascontiguousarray(B.bits[:, 3:11]), "f16")
    assert np.array_equal(Cs, C[:, 3:11])
    # a strided view (leading dimension > N) gives the same result
    Cv, _ = oracle.spmm(M, K, A.rowptr, A.colidx, A.vals, B.bits[:, 3:11], "f16")
    assert np.array_equal(Cv, C[:, 3:11])
    # scaling the values by 4 (exact in fp16) scales C exactly
    v4 = _f16(bits_to_f64(A.vals, "f16") * 4.0)
    C4, _ = oracle.spmm(M, K, A.rowptr, A.colidx, v4, B.bits, "f16")
    assert np.array_equal(C4, 4.0 * C)
    # row subset equals the rows of the full result
    rows = np.array([5, 0, 39, 17, 17], dtype=np.int64)
    Cr, _ = oracle.spmm(M, K, A.rowptr, A.colidx, A.vals, B.bits, "f16", rows=rows)
    assert np.array_equal(Cr, C[rows])
    # permuting A's columns together with B's rows leaves C unchanged (up to summation order)
    perm = stream(8, 98, 0).permutation(K)
    inv = np.argsort(perm)
    D = _densify(A)[:, perm]
    Ap = sp.csr_matrix(D)
    Ap.sort_indices()
    rowsA = np.repeat(np.arange(M), np.diff(A.rowptr))
    # rebuild value bits for the permuted matrix from the original bits
    bitsD = np.zeros((M, K), dtype=np.uint16)
    bitsD[rowsA, A.colidx] = A.vals
    bitsP = bitsD[:, perm]
    occ = np.zeros((M, K), dtype=bool)
    occ[rowsA, A.colidx] = True
    occP = occ[:, perm]
    rp = np.zeros(M + 1, dtype=np.int32)
    rp[1:] = np.cumsum(occP.sum(1))
    rr, cc = np.nonzero(occP)
    Cp, _ = oracle.spmm(M, K, rp, cc.astype(np.int32), bitsP[rr, cc], np.ascontiguousarray(B.bits[perm]), "f16")
    assert np.allclose(Cp, C, rtol=1e-13, atol=1e-13)
    assert inv.shape == perm.shape


def test_sddmm_transpose_symmetry():
    M, K, d = 14, 23, 8
    A = random_csr(M, K, 0.3, "f16", seed=31)
    X = dense(M, d, "n01", "f16", stream(9, 98, 0))
    Y = dense(K, d, "n01", "f16", stream(9, 98, 1))
    out, _ = oracle.sddmm(M, K, A.rowptr, A.colidx, X.bits, Y.bits, "f16")
    rows = np.repeat(np.arange(M), np.diff(A.rowptr))
    T = sp.csr_matrix((np.arange(1, A.nnz + 1), (A.colidx, rows)), shape=(K, M))  # pattern of A^T, payload = p+1
    T.sort_indices()
    outT, _ = oracle.sddmm(K, M, T.indptr.astype(np.int32), T.indices.astype(np.int32), Y.bits, X.bits, "f16")
    assert np.allclose(outT, out[T.data - 1], rtol=1e-14, atol=1e-14)


def test_out_of_range_index_is_reported():
    rp = np.array([0, 1], dtype=np.int32)
    ci = np.array([7], dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.spmm(1, 4, rp, ci, _f16([1.0]), _f16(np.ones((4, 2))), "f16")


def test_round_f64_to_bits_is_single_rounding():
    x = np.array([1.0 + 2.0 ** -8 + 2.0 ** -30, 1.0 + 2.0 ** -8, 3.0, -0.1, 65504.0 / 3])
    got = oracle.round_f64_to_bits(x, "bf16")
    # bf16 keeps 8 significant bits: 1 + 2^-8 is a tie (to even -> 1.0), a hair above goes up
    assert got[0] == 0x3F81 and got[1] == 0x3F80 and got[2] == 0x4040
    f = oracle.round_f64_to_bits(x, "f16")
    assert np.array_equal(f, x.astype(np.float16).view(np.uint16))
