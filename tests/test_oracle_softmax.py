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


# ---------------------------------------------------------------- gradient of the row softmax
def _bits(x, dtype="f16"):
    return round_to_bits(np.asarray(x, dtype=np.float32), dtype)


def test_backward_hand_worked_rows():
    """tests/golden/edge_softmax_backward_example.json: p = (1/2, 1/4, 1/4), g = (1, 2, 4): the row's
    p.g = 2, so ds = scale * (1/2 (1 - 2), 1/4 (2 - 2), 1/4 (4 - 2)); an empty row; a single entry (p = 1)
    has no freedom: 0."""
    import json, os
    ex = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "edge_softmax_backward_example.json")))
    rowptr = np.array(ex["rowptr"], dtype=np.int32)
    ds, S = oracle.edge_softmax_backward(len(rowptr) - 1, rowptr, _bits(ex["p"]), _bits(ex["g"]), "f16", scale=ex["scale"])
    np.testing.assert_array_equal(ds, ex["ds"])
    np.testing.assert_array_equal(S, ex["S"])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_backward_matches_plain_loops(dtype):
    """The vectorised sums against the definition written as loops over rows and entries."""
    A = random_csr(70, 50, 0.25, dtype, seed=11, empty_rows=0.2)
    rng = np.random.default_rng(3)
    p_bits = _bits(rng.uniform(0, 1, size=A.nnz), dtype)
    g_bits = _bits(rng.normal(size=A.nnz), dtype)
    ds, S = oracle.edge_softmax_backward(A.M, A.rowptr, p_bits, g_bits, dtype, scale=-0.7)
    p, g = bits_to_f64(p_bits, dtype), bits_to_f64(g_bits, dtype)
    for i in range(A.M):
        lo, hi = A.rowptr[i], A.rowptr[i + 1]
        dot = sum(p[r] * g[r] for r in range(lo, hi))
        mag = sum(abs(p[r] * g[r]) for r in range(lo, hi))
        for q in range(lo, hi):
            assert ds[q] == pytest.approx(-0.7 * p[q] * (g[q] - dot), rel=1e-13, abs=1e-300)
            assert S[q] == pytest.approx(0.7 * abs(p[q]) * (abs(g[q]) + mag), rel=1e-13)


def test_backward_is_the_derivative_of_the_forward_oracle():
    """Central differences of L(s) = sum_q g[q] * softmax(scale * s)[q] (scipy's softmax on each row, fp64)
    against the formula fed with probabilities that are exact in fp16: rows whose scores are multiples of
    ln 2 apart give dyadic probabilities."""
    scale = 0.5
    # scores s with scale * s in {0, ln 2, 2 ln 2}: exp = 1, 2, 4
    rows = [np.array([0.0, 1.0, 2.0, 0.0]), np.array([1.0, 1.0]), np.array([2.0, 0.0, 0.0, 1.0, 1.0, 2.0, 0.0, 0.0])]
    g_rows = [np.array([1.0, -2.0, 0.5, 3.0]), np.array([4.0, -1.0]), np.array([1, 2, 3, 4, -4, -3, -2, -1.0])]
    rowptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    s = np.concatenate(rows) * np.log(2.0) / scale
    g = np.concatenate(g_rows)
    p = np.concatenate([scipy.special.softmax(np.log(2.0) * r) for r in rows])
    p_bits = _bits(p)
    np.testing.assert_array_equal(bits_to_f64(p_bits, "f16"), p)  # (1,2,4,1)/8, (1,1)/2, (4,1,1,2,2,4,1,1)/16: exact

    def loss(sv):
        return sum(float(np.dot(g[rowptr[i]:rowptr[i + 1]], scipy.special.softmax(scale * sv[rowptr[i]:rowptr[i + 1]])))
                   for i in range(len(rows)))

    ds, _ = oracle.edge_softmax_backward(len(rows), rowptr, p_bits, _bits(g), "f16", scale=scale)
    h = 1e-6
    for q in range(len(s)):
        e = np.zeros_like(s)
        e[q] = h
        fd = (loss(s + e) - loss(s - e)) / (2 * h)
        assert ds[q] == pytest.approx(fd, rel=1e-7, abs=1e-9)


def test_backward_two_entry_rows_closed_form():
    """p = (t, 1 - t): ds = scale * t (1 - t) * (g0 - g1) * (+1, -1)."""
    t = np.array([0.5, 0.25, 0.125, 0.75])
    g0 = np.array([1.0, -3.0, 2.0, 0.5])
    g1 = np.array([2.0, 5.0, 2.0, -0.5])
    rowptr = np.arange(0, 9, 2, dtype=np.int32)
    p = np.stack([t, 1 - t], axis=1).reshape(-1)
    g = np.stack([g0, g1], axis=1).reshape(-1)
    ds, _ = oracle.edge_softmax_backward(4, rowptr, _bits(p), _bits(g), "f16", scale=3.0)
    want = 3.0 * t * (1 - t) * (g0 - g1)
    np.testing.assert_allclose(ds.reshape(4, 2), np.stack([want, -want], axis=1), rtol=1e-15)


def test_backward_invariants():
    """With probabilities that sum to one per row: the gradients of a row sum to zero, a gradient that is
    constant over a row gives zero, and adding a constant to g changes nothing.  (Probabilities k/64 are
    exact in both 16-bit types.)"""
    rng = np.random.default_rng(8)
    deg = rng.integers(0, 9, size=80)
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    p = []
    for n in deg:
        if n == 0:
            continue
        cuts = np.sort(rng.choice(np.arange(1, 64), size=n - 1, replace=False)) if n > 1 else np.array([], dtype=int)
        p.append(np.diff(np.concatenate([[0], cuts, [64]])) / 64.0)
    p = np.concatenate(p)
    row = np.repeat(np.arange(80), deg)
    for dtype in ("f16", "bf16"):
        p_bits = _bits(p, dtype)
        np.testing.assert_array_equal(bits_to_f64(p_bits, dtype), p)
        g = np.round(rng.normal(size=p.shape[0]) * 4) / 4
        ds, _ = oracle.edge_softmax_backward(80, rowptr, p_bits, _bits(g, dtype), dtype, scale=1.25)
        np.testing.assert_allclose(np.bincount(row, weights=ds, minlength=80), 0.0, atol=1e-13)
        ds_c, _ = oracle.edge_softmax_backward(80, rowptr, p_bits, _bits(np.full_like(g, 2.5), dtype), dtype, scale=1.25)
        np.testing.assert_allclose(ds_c, 0.0, atol=1e-15)
        ds_s, _ = oracle.edge_softmax_backward(80, rowptr, p_bits, _bits(g + 8.0, dtype), dtype, scale=1.25)
        np.testing.assert_allclose(ds_s, ds, atol=1e-13)


def test_widening_of_whole_arrays_is_the_c_oracle_s():
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    for dtype in ("f16", "bf16"):
        a = oracle._widen_all(bits, dtype)
        b = np.array([oracle.widen(int(x), dtype) for x in bits])
        assert np.array_equal(a, b, equal_nan=True)
