"""Pins for the edge-softmax oracle (CPU only): closed forms, a library routine on densified rows,
invariants, and a hand-worked example."""
import numpy as np
import pytest
import scipy.special

import oracle
from workloads import bits_to_f64, random_csr, round_to_bits


def _f16(x):
    return round_to_bits(np.asarray(x, dtype=np.float32), "f16")


def _row_of(A):
    return np.repeat(np.arange(A.M), np.diff(A.rowptr))


def test_hand_worked_rows():
    # row 0: scores (0, ln 3) -> exp = (1, 3) -> (0.25, 0.75); row 1: empty; row 2: single entry -> 1;
    # row 3: (1, 1, 1, 1) -> 0.25 each
    rowptr = np.array([0, 2, 2, 3, 7], dtype=np.int32)
    ln3 = float(np.float16(np.log(3.0)))  # the stored (rounded) score
    vals = _f16([0.0, ln3, -5.0, 1.0, 1.0, 1.0, 1.0])
    out = oracle.edge_softmax(4, rowptr, vals, "f16")
    e = np.exp(ln3)
    np.testing.assert_allclose(out, [1 / (1 + e), e / (1 + e), 1.0, 0.25, 0.25, 0.25, 0.25], rtol=1e-15)


def test_two_entry_rows_are_the_logistic_function():
    rng = np.random.default_rng(1)
    a = rng.normal(size=50).astype(np.float16)
    b = rng.normal(size=50).astype(np.float16)
    rowptr = np.arange(0, 101, 2, dtype=np.int32)
    vals = np.stack([a, b], axis=1).reshape(-1).view(np.uint16)
    for scale in (1.0, 0.125, -2.0):
        out = oracle.edge_softmax(50, rowptr, vals, "f16", scale=scale).reshape(50, 2)
        diff = scale * (a.astype(np.float64) - b.astype(np.float64))
        np.testing.assert_allclose(out[:, 0], 1.0 / (1.0 + np.exp(-diff)), rtol=1e-13)
        np.testing.assert_allclose(out[:, 1], 1.0 / (1.0 + np.exp(diff)), rtol=1e-13)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_matches_scipy_softmax_on_densified_rows(dtype):
    A = random_csr(60, 45, 0.3, dtype, seed=5, empty_rows=0.2)
    out = oracle.edge_softmax(A.M, A.rowptr, A.vals, dtype, scale=1.7)
    D = np.full((A.M, A.K), -np.inf)
    D[_row_of(A), A.colidx] = 1.7 * bits_to_f64(A.vals, dtype)
    with np.errstate(invalid="ignore"):
        want = scipy.special.softmax(D, axis=1)
    np.testing.assert_allclose(out, want[_row_of(A), A.colidx], rtol=1e-12)
    assert not np.isnan(out).any()  # every stored position was written


def test_rows_sum_to_one_and_uniform_scores_give_reciprocal_degree():
    A = random_csr(200, 300, 0.1, "f16", seed=9, empty_rows=0.1)
    out = oracle.edge_softmax(A.M, A.rowptr, A.vals, "f16")
    sums = np.bincount(_row_of(A), weights=out, minlength=A.M)
    deg = np.diff(A.rowptr)
    np.testing.assert_allclose(sums[deg > 0], 1.0, rtol=1e-13)
    assert (sums[deg == 0] == 0).all()
    flat = oracle.edge_softmax(A.M, A.rowptr, _f16(np.full(A.nnz, 0.375)), "f16", scale=3.0)
    np.testing.assert_allclose(flat, 1.0 / deg[_row_of(A)], rtol=1e-14)
    zero = oracle.edge_softmax(A.M, A.rowptr, A.vals, "f16", scale=0.0)
    np.testing.assert_allclose(zero, 1.0 / deg[_row_of(A)], rtol=1e-14)


def test_shift_invariance_and_monotonicity():
    # adding a per-row constant (exactly representable) leaves the result unchanged; a larger score gets a
    # larger weight inside a row
    A = random_csr(80, 64, 0.25, "f16", seed=3)
    v = np.round(bits_to_f64(A.vals, "f16") * 64) / 64  # multiples of 1/64 in (-1, 1): sums below stay exact
    shift = (np.arange(A.M) % 7 - 3).astype(np.float64)[_row_of(A)]
    a = oracle.edge_softmax(A.M, A.rowptr, _f16(v), "f16")
    b = oracle.edge_softmax(A.M, A.rowptr, _f16(v + shift), "f16")
    np.testing.assert_allclose(a, b, rtol=1e-12)
    for i in range(A.M):
        p0, p1 = A.rowptr[i], A.rowptr[i + 1]
        order = np.argsort(v[p0:p1], kind="stable")
        assert (np.diff(a[p0:p1][order]) >= 0).all()


def test_large_scores_do_not_overflow_and_row_subset():
    rowptr = np.array([0, 3, 5], dtype=np.int32)
    vals = _f16([60000.0, 59999.0 + 1, -60000.0, 3.0, 1.0])  # f16 max is 65504; 60000 rounds to 60000
    out = oracle.edge_softmax(2, rowptr, vals, "f16", scale=10.0)
    assert np.isfinite(out).all() and abs(out[:3].sum() - 1) < 1e-15 and out[2] == 0.0
    only1 = oracle.edge_softmax(2, rowptr, vals, "f16", rows=np.array([1]))
    assert np.isnan(only1[:3]).all()
    e = np.exp(2.0)
    np.testing.assert_allclose(only1[3:], [e / (1 + e), 1 / (1 + e)], rtol=1e-14)
