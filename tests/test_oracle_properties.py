"""Property tests (hypothesis) of the CPU oracle on tiny generated matrices: any shape, empty rows and
windows, M not a multiple of V, vector counts not a multiple of KB, explicit zeros, a hub row."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from fmt_decode import decode_to_dense
from workloads import Csr, bits_to_f64, round_to_bits


@st.composite
def tiny_csr(draw):
    M = draw(st.integers(1, 24))
    K = draw(st.integers(1, 40))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    rng = np.random.default_rng(seed)
    dens = draw(st.sampled_from([0.0, 0.05, 0.3, 0.8, 1.0]))
    mask = rng.random((M, K)) < dens
    if draw(st.booleans()):
        mask[draw(st.integers(0, M - 1)), :] = True  # a hub row
    if draw(st.booleans()):
        mask[draw(st.integers(0, M - 1)), :] = False  # an empty row
    vals = rng.integers(-6, 7, size=(M, K)).astype(np.float32) / 2  # small multiples of 1/2, zeros included
    rowptr = np.concatenate([[0], np.cumsum(mask.sum(1))]).astype(np.int32)
    colidx = np.nonzero(mask)[1].astype(np.int32)
    dtype = draw(st.sampled_from(["f16", "bf16"]))
    return Csr(M, K, rowptr, colidx, round_to_bits(vals[mask], dtype), dtype), mask, vals


@settings(max_examples=80, deadline=None)
@given(tiny_csr(), st.sampled_from([1, 2, 4, 8, 16]), st.sampled_from([1, 3, 4, 32]))
def test_converter_round_trip_and_structure(case, V, KB):
    A, mask, vals = case
    f = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, V, KB)
    dense, occ = decode_to_dense(A.M, A.K, V, KB, f.win_ptr, f.vec_col, f.vals_blk, f.vec_mask)
    assert np.array_equal(occ, mask)  # stored positions, explicit zeros included
    assert np.array_equal(bits_to_f64(dense, A.dtype)[mask], vals[mask].astype(np.float64))
    assert f.vals_blk.shape[0] == V * f.nvec and f.win_ptr[-1] == f.nvec
    for w in range(f.W):
        seg = f.vec_col[f.win_ptr[w]:f.win_ptr[w + 1]]
        assert (np.diff(seg) > 0).all()
        rows = mask[w * V:(w + 1) * V]
        assert seg.tolist() == np.nonzero(rows.any(0))[0].tolist()  # exactly the columns the window stores
    assert sorted(set(f.csr_to_slot.tolist())) == sorted(f.csr_to_slot.tolist())
    assert np.array_equal(f.vals_blk[f.csr_to_slot], A.vals)


@settings(max_examples=60, deadline=None)
@given(tiny_csr(), st.integers(1, 9), st.integers(1, 9))
def test_operators_equal_dense_products_exactly(case, N, d):
    # small multiples of 1/2: every product and sum below is exact in double, so equality is exact
    A, mask, vals = case
    rng = np.random.default_rng(A.M * 131 + A.K)
    Bv = rng.integers(-4, 5, size=(A.K, N)).astype(np.float32)
    Xv = rng.integers(-3, 4, size=(A.M, d)).astype(np.float32) / 2
    Yv = rng.integers(-3, 4, size=(A.K, d)).astype(np.float32)
    Ad = np.where(mask, vals, 0).astype(np.float64)
    C, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, round_to_bits(Bv, A.dtype), A.dtype)
    assert np.array_equal(C, Ad @ Bv.astype(np.float64))
    assert np.array_equal(S, np.abs(Ad) @ np.abs(Bv).astype(np.float64))
    out, _ = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, round_to_bits(Xv, A.dtype), round_to_bits(Yv, A.dtype), A.dtype)
    full = Xv.astype(np.float64) @ Yv.astype(np.float64).T
    assert np.array_equal(out, full[mask])


@settings(max_examples=60, deadline=None)
@given(tiny_csr(), st.sampled_from([1.0, 0.25, -1.5]))
def test_edge_softmax_rows_are_probability_vectors(case, scale):
    A, mask, vals = case
    out = oracle.edge_softmax(A.M, A.rowptr, A.vals, A.dtype, scale=scale)
    assert out.shape[0] == A.nnz and not np.isnan(out).any()
    for i in range(A.M):
        p0, p1 = A.rowptr[i], A.rowptr[i + 1]
        if p1 > p0:
            seg = out[p0:p1]
            assert (seg > 0).all() and abs(seg.sum() - 1) < 1e-12
            z = scale * vals[i][mask[i]].astype(np.float64)
            e = np.exp(z - z.max())
            np.testing.assert_allclose(seg, e / e.sum(), rtol=1e-12)
