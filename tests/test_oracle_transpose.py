"""Pins of the oracle's CSR transposition (the index structure behind A^T * dC, the backward pass of
C = A * B in the paper's Section 4.4 training workloads) against things that are not the oracle:
a dense transposition, scipy's conversion, the involution property, a brute-force enumeration."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle


def _random_csr(rng, M, K, density):
    mask = rng.random((M, K)) < density
    rowptr = np.zeros(M + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(mask.sum(axis=1))
    colidx = np.nonzero(mask)[1].astype(np.int32)
    return mask, rowptr, colidx


@pytest.mark.parametrize("M,K,density", [(1, 1, 1.0), (7, 5, 0.4), (5, 300, 0.05), (300, 5, 0.3), (64, 64, 0.0), (40, 70, 1.0)])
def test_dense_transposition(M, K, density):
    rng = np.random.default_rng([7, M, K])
    mask, rowptr, colidx = _random_csr(rng, M, K, density)
    vals = rng.standard_normal(colidx.shape[0])
    rt, ct, perm = oracle.csr_transpose(M, K, rowptr, colidx)
    # rebuild A^T densely from the result and compare with the dense transposition of A
    A = np.zeros((M, K)); A[mask] = vals  # boolean assignment runs in row-major = CSR order
    At = np.zeros((K, M))
    for k in range(K):
        cols = ct[rt[k]:rt[k + 1]]
        assert np.all(np.diff(cols) > 0), "rows of A^T must have strictly ascending columns"
        At[k, cols] = vals[perm[rt[k]:rt[k + 1]]]
    assert rt[0] == 0 and rt[K] == colidx.shape[0]
    assert np.array_equal(At, A.T)
    assert np.array_equal(np.sort(perm), np.arange(colidx.shape[0]))


def test_against_scipy():
    rng = np.random.default_rng(11)
    M, K = 500, 321
    _, rowptr, colidx = _random_csr(rng, M, K, 0.03)
    tags = np.arange(1, colidx.shape[0] + 1, dtype=np.float64)  # a distinct value per entry exposes the permutation
    T = sp.csr_matrix((tags, colidx, rowptr), shape=(M, K)).T.tocsr()
    T.sort_indices()
    rt, ct, perm = oracle.csr_transpose(M, K, rowptr, colidx)
    assert np.array_equal(rt, T.indptr) and np.array_equal(ct, T.indices)
    assert np.array_equal(tags[perm], T.data)


def test_transposing_twice_is_the_identity():
    rng = np.random.default_rng(12)
    M, K = 90, 130
    _, rowptr, colidx = _random_csr(rng, M, K, 0.1)
    rt, ct, perm = oracle.csr_transpose(M, K, rowptr, colidx)
    rtt, ctt, perm2 = oracle.csr_transpose(K, M, rt, ct)
    assert np.array_equal(rtt, rowptr) and np.array_equal(ctt, colidx)
    assert np.array_equal(perm[perm2], np.arange(colidx.shape[0]))


def test_brute_force_enumeration():
    # every pattern of a 3 x 3 matrix: sort the coordinate list by (column, row) and compare
    for code in range(512):
        coords = [(i, k) for i in range(3) for k in range(3) if code >> (3 * i + k) & 1]
        rowptr = np.zeros(4, dtype=np.int32)
        for i, _ in coords:
            rowptr[i + 1] += 1
        rowptr = np.cumsum(rowptr).astype(np.int32)
        colidx = np.array([k for _, k in coords], dtype=np.int32)
        rt, ct, perm = oracle.csr_transpose(3, 3, rowptr, colidx)
        order = sorted(range(len(coords)), key=lambda p: (coords[p][1], coords[p][0]))
        assert list(perm) == order
        assert list(ct) == [coords[p][0] for p in order]
        assert [int(rt[k + 1] - rt[k]) for k in range(3)] == [sum(1 for _, k2 in coords if k2 == k) for k in range(3)]


def test_rejects_a_column_out_of_range():
    rowptr = np.array([0, 1], dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.csr_transpose(1, 3, rowptr, np.array([3], dtype=np.int32))
