"""Pins of the oracle's sparse attention (softmax over each row's stored entries of scale * X Y^T, times H:
the SDDMM -> softmax -> SpMM chain of the paper's Section 4.4 attention GNN) against things that are not
the oracle: a dense masked-softmax formula, closed forms, and the separately pinned operators."""
import numpy as np
import pytest

import oracle
from workloads import bits_to_f64, dense, random_csr, round_to_bits, stream


def _case(M, K, d, N, density, dtype, seed, empty_rows=0.15):
    A = random_csr(M, K, density, dtype, seed=seed, empty_rows=empty_rows)
    X = dense(M, d, "n01", dtype, stream(seed, 50, 1))
    Y = dense(K, d, "n01", dtype, stream(seed, 50, 2))
    H = dense(K, N, "n01", dtype, stream(seed, 50, 3))
    return A, X, Y, H


def _dense_mask(A):
    mask = np.zeros((A.M, A.K), dtype=bool)
    mask[np.repeat(np.arange(A.M), np.diff(A.rowptr)), A.colidx] = True
    return mask


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("scale", [1.0, 0.125, -0.7])
def test_dense_masked_softmax_formula(dtype, scale):
    A, X, Y, H = _case(37, 53, 16, 24, 0.2, dtype, seed=3)
    Xf, Yf, Hf = (bits_to_f64(t.bits, dtype) for t in (X, Y, H))
    mask = _dense_mask(A)
    T = np.where(mask, scale * (Xf @ Yf.T), -np.inf)
    with np.errstate(invalid="ignore"):
        P = np.exp(T - np.where(mask.any(1), T.max(1), 0.0)[:, None])
    P = np.where(mask, P, 0.0)
    den = P.sum(1, keepdims=True)
    W = np.divide(P, den, out=np.zeros_like(P), where=den > 0)
    out, S = oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, H.bits, dtype, scale)
    assert np.allclose(out, W @ Hf, rtol=1e-12, atol=1e-13)
    assert np.allclose(S, W @ np.abs(Hf), rtol=1e-12, atol=1e-13)
    assert not out[~mask.any(1)].any()  # rows without stored entries


def test_zero_queries_average_the_neighbours():
    A, X, Y, H = _case(40, 30, 8, 16, 0.3, "f16", seed=5)
    X.bits[:] = 0
    out, _ = oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, H.bits, "f16", 3.0)
    Hf = bits_to_f64(H.bits, "f16")
    for i in range(A.M):
        cols = A.colidx[A.rowptr[i]:A.rowptr[i + 1]]
        want = Hf[cols].mean(0) if cols.size else np.zeros(16)
        assert np.allclose(out[i], want, rtol=1e-13, atol=1e-15)


def test_single_entry_rows_copy_one_row_of_h():
    rng = np.random.default_rng(8)
    M, K = 25, 40
    rowptr = np.arange(M + 1, dtype=np.int32)
    colidx = rng.integers(0, K, M).astype(np.int32)
    X = dense(M, 8, "n01", "bf16", stream(1, 51, 1)); Y = dense(K, 8, "n01", "bf16", stream(1, 51, 2))
    H = dense(K, 8, "n01", "bf16", stream(1, 51, 3))
    out, S = oracle.attention(M, K, rowptr, colidx, X.bits, Y.bits, H.bits, "bf16", 2.0)
    assert np.array_equal(out, bits_to_f64(H.bits, "bf16")[colidx])
    assert np.array_equal(S, np.abs(out))


def test_a_large_scale_selects_the_best_match():
    A, X, Y, H = _case(30, 45, 16, 8, 0.25, "f16", seed=9, empty_rows=0.0)
    T, _ = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, "f16")  # the separately pinned scores
    out, _ = oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, H.bits, "f16", 1e4)
    Hf = bits_to_f64(H.bits, "f16")
    for i in range(A.M):
        p0, p1 = A.rowptr[i], A.rowptr[i + 1]
        if p1 > p0:
            best = A.colidx[p0 + int(np.argmax(T[p0:p1]))]
            assert np.allclose(out[i], Hf[best], rtol=1e-9, atol=1e-12)


def test_equals_the_three_pinned_operators_when_nothing_rounds():
    """Scores that are exactly representable in fp16 (small integers) and a softmax whose values are exact
    powers of two let the chain of the three separately pinned functions reproduce the definition."""
    rng = np.random.default_rng(13)
    M, K, d, N = 20, 28, 4, 8
    A = random_csr(M, K, 0.3, "f16", seed=13)
    X = round_to_bits(rng.integers(-2, 3, (M, d)).astype(np.float32), "f16")
    Y = round_to_bits(rng.integers(-2, 3, (K, d)).astype(np.float32), "f16")
    H = dense(K, N, "n01", "f16", stream(13, 52, 3))
    T, _ = oracle.sddmm(M, K, A.rowptr, A.colidx, X, Y, "f16")
    tb = oracle.round_f64_to_bits(T, "f16")
    assert np.array_equal(bits_to_f64(tb, "f16"), T)  # integers: nothing lost
    W = oracle.edge_softmax(M, A.rowptr, tb, "f16", scale=np.log(2.0))  # 2^t / sum 2^t
    out, _ = oracle.attention(M, K, A.rowptr, A.colidx, X, Y, H.bits, "f16", np.log(2.0))
    Hf = bits_to_f64(H.bits, "f16")
    for i in range(M):
        p0, p1 = A.rowptr[i], A.rowptr[i + 1]
        want = (W[p0:p1, None] * Hf[A.colidx[p0:p1]]).sum(0) if p1 > p0 else np.zeros(N)
        assert np.allclose(out[i], want, rtol=1e-12, atol=1e-14)


def test_row_subset_and_bad_index():
    A, X, Y, H = _case(33, 21, 8, 8, 0.3, "f16", seed=17)
    full, _ = oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, H.bits, "f16", 0.5)
    rows = np.array([32, 0, 7, 7])
    sub, _ = oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, H.bits, "f16", 0.5, rows=rows)
    assert np.array_equal(sub, full[rows])
    with pytest.raises(ValueError):
        oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, H.bits, "f16", 0.5, rows=np.array([33]))
