"""Pins for the reference converter (CPU only): a hand-worked example, a
per-element brute force over a dense occupancy mask, round trip through an
independent decoder, closed-form counts and structural invariants."""
import json
import os

import numpy as np
import pytest

import oracle
from fmt_decode import decode_to_dense
from workloads import make_config, random_csr, stencil5, csr_from_coo, stream


def test_golden_2x4_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "mebcrs_2x4_example.json")))
    # the fixture's CSR is consistent with its own dense picture
    D = np.array(g["dense_rows"])
    rr, cc = np.nonzero(D)
    assert list(cc) == g["colidx"] and list(D[rr, cc]) == g["vals"]
    f = oracle.convert_ref(g["M"], g["K"], np.array(g["rowptr"]), np.array(g["colidx"]),
                           np.array(g["vals"], dtype=np.uint16), g["V"], g["KB"])
    assert f.W == 2 and f.nvec == 9
    assert f.win_ptr.tolist() == g["win_ptr"]
    assert f.vec_col.tolist() == g["vec_col"]
    assert f.vec_mask.tolist() == g["vec_mask"]
    assert f.vals_blk.tolist() == g["vals_blk"]
    assert f.csr_to_slot.tolist() == g["csr_to_slot"]
    R = oracle.issued_mac_ratio(f.win_ptr, g["V"], g["KB"], len(g["vals"]))
    assert R == g["mac_slots_issued"] / len(g["vals"])


def _brute(M, K, rowptr, colidx, vals, V, KB):
    """Element-by-element construction from a dense occupancy mask (tiny inputs only)."""
    occ = np.zeros((M, K), dtype=bool)
    val = np.zeros((M, K), dtype=np.uint16)
    pos = -np.ones((M, K), dtype=np.int64)
    for i in range(M):
        for p in range(rowptr[i], rowptr[i + 1]):
            occ[i, colidx[p]] = True
            val[i, colidx[p]] = vals[p]
            pos[i, colidx[p]] = p
    W = -(-M // V)
    win_ptr, vec_col, vec_mask = [0], [], []
    vals_blk, slot_of = [], {}
    for w in range(W):
        rows = range(w * V, min(M, w * V + V))
        cols = [k for k in range(K) if any(occ[i, k] for i in rows)]
        for k in cols:
            vec_col.append(k)
            vec_mask.append(sum(1 << (i - w * V) for i in rows if occ[i, k]))
        for b0 in range(0, len(cols), KB):
            blk = cols[b0:b0 + KB]
            for r in range(V):
                i = w * V + r
                for k in blk:
                    if i < M and occ[i, k]:
                        slot_of[pos[i, k]] = len(vals_blk)
                        vals_blk.append(val[i, k])
                    else:
                        vals_blk.append(0)
        win_ptr.append(len(vec_col))
    return win_ptr, vec_col, vec_mask, vals_blk, [slot_of[p] for p in range(len(colidx))]


@pytest.mark.parametrize("V,KB", [(8, 32), (16, 32), (8, 8), (4, 4), (2, 4), (1, 3), (8, 5)])
@pytest.mark.parametrize("M,K,dens,seed", [(37, 50, 0.2, 0), (64, 40, 0.6, 1), (9, 300, 0.5, 2), (20, 20, 0.02, 3)])
def test_against_brute_force(M, K, dens, seed, V, KB):
    A = random_csr(M, K, dens, "f16", seed, empty_rows=0.3)
    f = oracle.convert_ref(M, K, A.rowptr, A.colidx, A.vals, V, KB)
    wp, vc, vm, vb, sl = _brute(M, K, A.rowptr, A.colidx, A.vals, V, KB)
    assert f.win_ptr.tolist() == wp
    assert f.vec_col.tolist() == vc
    assert f.vec_mask.tolist() == vm
    assert f.vals_blk.tolist() == [int(x) for x in vb]
    assert f.csr_to_slot.tolist() == sl


@pytest.mark.parametrize("V,KB", [(8, 32), (16, 32), (4, 4)])
def test_round_trip_and_invariants(V, KB):
    A = random_csr(203, 180, 0.08, "bf16", seed=5, empty_rows=0.2)
    f = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, V, KB)
    dense, occ = decode_to_dense(A.M, A.K, V, KB, f.win_ptr, f.vec_col, f.vals_blk, f.vec_mask)
    rows = np.repeat(np.arange(A.M), np.diff(A.rowptr))
    want = np.zeros((A.M, A.K), dtype=np.uint16)
    want[rows, A.colidx] = A.vals
    wocc = np.zeros((A.M, A.K), dtype=bool)
    wocc[rows, A.colidx] = True
    assert np.array_equal(occ, wocc) and np.array_equal(dense, want)
    # structure
    assert f.win_ptr[0] == 0 and f.win_ptr[-1] == f.nvec and (np.diff(f.win_ptr) >= 0).all()
    for w in range(f.W):
        seg = f.vec_col[f.win_ptr[w]:f.win_ptr[w + 1]]
        assert (np.diff(seg) > 0).all()
    assert (f.vec_mask != 0).all() and (f.vec_mask < (1 << V)).all()
    assert sum(bin(int(m)).count("1") for m in f.vec_mask) == A.nnz
    assert len(set(f.csr_to_slot.tolist())) == A.nnz
    assert np.array_equal(f.vals_blk[f.csr_to_slot], A.vals)
    other = np.ones(V * f.nvec, dtype=bool)
    other[f.csr_to_slot] = False
    assert (f.vals_blk[other] == 0).all()
    assert f.vals_blk.shape[0] == V * f.nvec


def test_V1_is_csr_and_vector_counts_nest():
    A = random_csr(96, 120, 0.1, "f16", seed=6)
    f1 = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, 1, 8)
    assert f1.nvec == A.nnz and np.array_equal(f1.vec_col, A.colidx)
    assert np.array_equal(f1.win_ptr, A.rowptr)
    n = {V: oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, V, 8).nvec for V in (2, 4, 8, 16)}
    for V in (2, 4, 8):
        assert n[2 * V] <= n[V] <= 2 * n[2 * V]


def test_explicit_zero_still_marks_a_vector():
    rp = np.array([0, 1, 2], dtype=np.int32)
    ci = np.array([3, 5], dtype=np.int32)
    vals = np.array([0, 0x3C00], dtype=np.uint16)  # first stored value is an explicit +0.0
    f = oracle.convert_ref(2, 8, rp, ci, vals, 2, 4)
    assert f.nvec == 2 and f.vec_col.tolist() == [3, 5] and f.vec_mask.tolist() == [1, 2]


def test_pattern_only_conversion():
    A = random_csr(30, 30, 0.2, "f16", seed=7)
    f = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, None, 8, 32)
    g = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, 8, 32)
    assert (f.vals_blk == 0).all() and np.array_equal(f.csr_to_slot, g.csr_to_slot)


def test_stencil_closed_forms():
    g = 64
    r, c = stencil5(g)
    A = csr_from_coo(g * g, g * g, r, c, "n01", "f16", stream(0, 3, 1))
    assert A.nnz == 5 * g * g - 4 * g
    V = 8  # V divides g: a window is 8 consecutive cells of one grid row
    f = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals, V, 32)
    n = np.diff(f.win_ptr).reshape(g, g // V)  # [grid row][window in row]
    # interior window: its 8 cells, one neighbour left and right, 8 above, 8 below = 3V + 2
    assert (n[1:-1, 1:-1] == 3 * V + 2).all()
    # closed form for the total: per grid row, (g + 2*(g/V) - 2) in-row vectors ... summed with the
    # vertical neighbours (one row of V per window above and below, absent at the top/bottom edge)
    per_row_inrow = g + 2 * (g // V) - 2
    total = g * per_row_inrow + 2 * (g - 1) * g
    assert f.nvec == total


def test_config1_counts():
    c = make_config("cfg1_uniform")
    A = c["A"]
    assert A.nnz == 65536 and (np.diff(A.rowptr) == 16).all()
    for i in (0, 100, 4095):
        seg = A.colidx[A.rowptr[i]:A.rowptr[i + 1]]
        assert (np.diff(seg) > 0).all()


def test_padded_footprint_formula():
    # 3 windows with 5, 0 and 8 vectors, V=2, KB=4: padded counts are 8, 0, 8
    wp = np.array([0, 5, 5, 13])
    d = oracle.padded_format_bytes(wp, 2, 4)
    assert d["me_bcrs"] == 4 * 4 + 4 * 13 + 2 * 2 * 13
    assert d["padded"] == 4 * 6 + 4 * 16 + 2 * 2 * 16


@pytest.mark.parametrize("M,K,dens,seed,V,KB", [(19, 23, 0.3, 1, 8, 4), (40, 70, 0.5, 2, 4, 32), (33, 90, 0.08, 3, 8, 32),
                                                 (9, 200, 0.6, 4, 16, 32), (64, 64, 0.0, 5, 8, 32)])
def test_packed_values_against_brute_force(M, K, dens, seed, V, KB):
    """pack_ref against loops over windows, blocks, rows and vectors of a dense occupancy mask, and the
    golden example's value array with its zeros struck out by hand."""
    A = random_csr(M, K, dens, "f16", seed=seed, empty_rows=0.2)
    vals = (np.arange(A.nnz) + 1).astype(np.uint16)  # distinct, non-zero: a misplaced value shows
    f = oracle.convert_ref(M, K, A.rowptr, A.colidx, vals, V, KB)
    blk_ofs, packed = oracle.pack_ref(f, vals)
    D = np.zeros((M, K), dtype=np.uint16)
    D[np.repeat(np.arange(M), np.diff(A.rowptr)), A.colidx] = vals
    want, want_ofs = [], []
    for w in range((M + V - 1) // V):
        rows = range(w * V, min(M, w * V + V))
        cols = [c for c in range(K) if any(D[i, c] for i in rows)]  # the window's vectors, ascending
        for b0 in range(0, max(len(cols), 1), KB):
            want_ofs.append(len(want))
            for i in rows:
                want += [D[i, c] for c in cols[b0:b0 + KB] if D[i, c]]
    want_ofs.append(len(want))
    assert packed.tolist() == want and blk_ofs.tolist() == want_ofs
    # the padded array with the never-stored positions removed, in order
    keep = np.zeros(f.vals_blk.shape[0], dtype=bool)
    keep[f.csr_to_slot] = True
    assert np.array_equal(packed, f.vals_blk[keep])


def test_packed_values_of_the_golden_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "mebcrs_2x4_example.json")))
    vals = np.array(g["vals"], dtype=np.uint16)
    f = oracle.convert_ref(g["M"], g["K"], np.array(g["rowptr"]), np.array(g["colidx"]), vals, g["V"], g["KB"])
    blk_ofs, packed = oracle.pack_ref(f, vals)
    assert packed.tolist() == [v for v in g["vals_blk"] if v != 0]  # the example stores no explicit zero
    assert blk_ofs[0] == 0 and blk_ofs[-1] == len(g["vals"]) and np.all(np.diff(blk_ofs) >= 0)
