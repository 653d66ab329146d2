"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Bars: converted indices, masks, slots and value bits are compared bit for bit;
floating results must satisfy  max |gpu - ref| / S <= 1e-2  with S = sum |a||b|
from the oracle (fp16 / bf16 inputs, fp32 accumulation, one rounding on store) -- the contract --
and, as the regression bar, 2^-10 (fp16) or 2^-7 (bf16) of S: twice the half-ulp of the one output rounding
(gpu_util.check_close asserts both and prints the plain relative error where nothing cancels).
"""
import numpy as np
import pytest

import oracle
from gpu_util import check_close, from_dev_bits, scaled_error, to_dev, to_dev_i32, upload_csr
from workloads import (Csr, bits_to_f64, csr_from_coo, dense, make_config, random_csr, round_to_bits, stream)

pytestmark = pytest.mark.gpu
TOL = 1e-2


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2412_11007_amd as fs
    fs.load_library()  # raises if the HIP library is missing: there is no fallback
    return fs


_cfg_cache = {}


def cfg(name, shrink=None):
    key = (name, shrink)
    if key not in _cfg_cache:
        if len(_cfg_cache) > 3:
            _cfg_cache.clear()
        _cfg_cache[key] = make_config(name, shrink=shrink)
    return _cfg_cache[key]


def convert(fs, A: Csr, V=8, KB=32, chunk=0, with_vals=True):
    rp, ci, va = upload_csr(A)
    return fs.fs_convert(rp, ci, va if with_vals else None, A.M, A.K, torch_dtype=va.dtype, V=V, KB=KB, chunk=chunk)


def assert_format_equal(fmt, A: Csr, V, KB, with_vals=True):
    ref = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, A.vals if with_vals else None, V, KB)
    assert (fmt.M, fmt.K, fmt.nnz, fmt.W, fmt.V, fmt.KB) == (A.M, A.K, A.nnz, ref.W, V, KB)
    assert fmt.nvec == ref.nvec
    assert np.array_equal(fmt.win_ptr_t().cpu().numpy(), ref.win_ptr)
    assert np.array_equal(fmt.vec_col_t().cpu().numpy(), ref.vec_col)
    assert np.array_equal(fmt.vec_mask_t().cpu().numpy().view(np.uint32), ref.vec_mask)
    assert np.array_equal(fmt.csr_to_slot_t().cpu().numpy(), ref.csr_to_slot)
    assert np.array_equal(from_dev_bits(fmt.vals_blk_t()), ref.vals_blk)
    return ref


def assert_row_base_valid(fmt, A: Csr):
    """blk_row_base against a search in the CSR arrays (vectorised over all (block, row) pairs)."""
    rb = fmt.blk_row_base_t().cpu().numpy().astype(np.int64)
    desc = fmt.blk_desc_t().cpu().numpy().astype(np.int64)
    vc = fmt.vec_col_t().cpu().numpy().astype(np.int64)
    V = fmt.V
    rows = desc[:, 2][:, None] * V + np.arange(V)[None, :]
    live = rows < A.M
    rr = np.minimum(rows, A.M - 1)
    lo, hi = A.rowptr[rr].astype(np.int64), A.rowptr[rr + 1].astype(np.int64)
    width = desc[:, 1] & 255
    first_col = np.where(width > 0, vc[np.minimum(desc[:, 0], max(fmt.nvec - 1, 0))] if fmt.nvec else 0, 0)
    # entries of a row are ascending in column: key = row * K + column is ascending over the whole CSR order
    key = np.repeat(np.arange(A.M, dtype=np.int64), np.diff(A.rowptr)) * A.K + A.colidx.astype(np.int64)
    want = np.searchsorted(key, rr * A.K + first_col[:, None])
    want = np.where(width[:, None] > 0, want, lo)
    want = np.where(live, want, 0)
    assert np.array_equal(rb, want)
    assert (want >= np.where(live, lo, 0)).all() and (want <= np.where(live, hi, 0)).all()


def assert_items_valid(fmt):
    """The block table describes every block of every window; the work list walks its slots exactly
    once, in order; the partial-tile slots this implies are the ones the split-window table names."""
    items = fmt.items_t().cpu().numpy()
    desc = fmt.blk_desc_t().cpu().numpy()
    wp = fmt.win_ptr_t().cpu().numpy().astype(np.int64)
    KB, T = fmt.KB, fmt.chunk // fmt.KB
    assert items.shape[0] == fmt.n_items
    # block table against the window pointers
    n_w = np.diff(wp)
    nblk_w = np.maximum(1, -(-n_w // KB))
    blk_ptr = np.concatenate([[0], np.cumsum(nblk_w)])
    assert desc.shape[0] == fmt.n_blocks == blk_ptr[-1]
    w_of = np.repeat(np.arange(fmt.W), nblk_w)
    b_of = np.arange(desc.shape[0]) - blk_ptr[w_of]
    assert np.array_equal(desc[:, 2], w_of)
    assert np.array_equal(desc[:, 0], wp[w_of] + b_of * KB)
    assert np.array_equal(desc[:, 1] & 255, np.clip(n_w[w_of] - b_of * KB, 0, KB))
    assert np.array_equal((desc[:, 1] & 256) != 0, b_of == nblk_w[w_of] - 1)
    assert np.array_equal((desc[:, 1] & 512) != 0, b_of == 0)
    # CSR position of each window row's first entry at or after the block's first column
    assert tuple(fmt.blk_row_base_t().shape) == (fmt.n_blocks, fmt.V)
    # work list
    expect = 0  # next block slot the walk must produce
    next_slot = 0
    tiles = {}  # window -> list of partial slots
    for g0, nb, slot0, s_first in items:
        if nb == 0:
            continue
        assert g0 == expect and nb <= 2 * T + 4 and nb <= 64 and s_first == desc[g0, 0]
        slot = int(slot0)
        assert slot == next_slot
        from_first = bool(desc[g0, 1] & 512)
        for x in range(g0, g0 + nb):
            last_blk = bool(desc[x, 1] & 256)
            if last_blk or x == g0 + nb - 1:
                if not (from_first and last_blk):
                    tiles.setdefault(int(desc[x, 2]), []).append(slot)
                    slot += 1
            if last_blk:
                from_first = True
        expect = g0 + nb
        next_slot = slot
    assert expect == fmt.n_blocks
    assert next_slot == fmt.n_split_items
    sw = fmt.split_windows_t().cpu().numpy()
    assert sw.shape[0] == fmt.n_split_windows == len(tiles)
    for (w, first, cnt, _), (tw, tl) in zip(sw, sorted(tiles.items())):
        assert w == tw and tl == list(range(first, first + cnt)) and cnt >= 2
    assert set(np.nonzero(nblk_w > T)[0]) >= set(tiles.keys())  # only windows longer than an item are cut
    # every partial-tile slot knows its window's slot range
    sr = fmt.slot_range_t().cpu().numpy()
    assert sr.shape == (fmt.n_split_items, 2)
    for (w, first, cnt, _) in sw:
        assert (sr[first:first + cnt, 0] == first).all() and (sr[first:first + cnt, 1] == cnt).all()
    assert int(sw[:, 2].sum()) == fmt.n_split_items if len(sw) else fmt.n_split_items == 0
    # launch order: a permutation; parts of cut windows first, by the column of their first vector (16 bits),
    # then whole windows, costliest first (blocks + window-ending blocks); ties in work-list order
    order = fmt.item_order_t().cpu().numpy().astype(np.int64)
    assert np.array_equal(np.sort(order), np.arange(fmt.n_items))
    ends = np.concatenate([[0], np.cumsum((desc[:, 1] & 256) != 0)])
    g0, nb = items[:, 0].astype(np.int64), items[:, 1].astype(np.int64)
    live = nb > 0
    cost = np.minimum(nb + ends[g0 + nb] - ends[g0], 128)
    last = np.where(live, g0 + nb - 1, 0)
    cut = live & (((desc[np.where(live, g0, 0), 1] & 512) == 0) | ((desc[last, 1] & 256) == 0))
    vc = fmt.vec_col_t().cpu().numpy().astype(np.int64)
    first_col = vc[np.minimum(items[:, 3], max(fmt.nvec - 1, 0))] if fmt.nvec else np.zeros(len(items), dtype=np.int64)
    key = np.where(cut, (first_col << 16) // max(fmt.K, 1), (1 + 128 - cost) << 16)
    key = np.where(live, key, 0x00FFFFFF)
    assert np.array_equal(order, np.argsort(key, kind="stable"))
    assert fmt.n_cut_items == int(cut.sum())
    assert np.array_equal(fmt.items_by_cost_t().cpu().numpy(), items[order])


# ------------------------------------------------------------------ conversion
@pytest.mark.parametrize("V,KB", [(8, 32), (16, 32), (8, 8), (4, 4), (2, 4), (1, 3), (32, 64), (8, 5)])
@pytest.mark.parametrize("M,K,dens,seed", [(37, 50, 0.2, 0), (64, 40, 0.6, 1), (9, 300, 0.5, 2), (203, 180, 0.05, 3)])
def test_convert_small_bit_exact(fs, M, K, dens, seed, V, KB):
    A = random_csr(M, K, dens, "f16", seed, empty_rows=0.3)
    fmt = convert(fs, A, V, KB)
    assert_format_equal(fmt, A, V, KB)
    assert_items_valid(fmt)
    assert_row_base_valid(fmt, A)


def test_convert_edge_cases(fs):
    # no stored entries at all
    A = Csr(10, 7, np.zeros(11, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16), "f16")
    fmt = convert(fs, A)
    assert fmt.nvec == 0 and fmt.n_split_items == 0
    assert_items_valid(fmt)
    assert_format_equal(fmt, A, 8, 32)
    # one hub row among empty ones, M not a multiple of V, long enough to be cut into items
    K = 5000
    cols = np.arange(0, K, 2)
    rows = np.full(cols.shape, 11)
    A = csr_from_coo(13, K, rows, cols, "u11", "bf16", stream(0, 97, 0))
    fmt = convert(fs, A, 8, 32, chunk=64)
    assert_format_equal(fmt, A, 8, 32)
    assert_items_valid(fmt)
    # 79 blocks in parts of two from the window's start; the odd last block joins the part before it
    assert fmt.n_split_windows == 1 and fmt.n_split_items == 39
    # pattern-only conversion
    A = random_csr(50, 60, 0.2, "f16", 5)
    fmt = convert(fs, A, with_vals=False)
    assert_format_equal(fmt, A, 8, 32, with_vals=False)
    # a matrix without rows: nothing to convert, nothing to launch
    import torch
    Z = Csr(0, 9, np.zeros(1, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16), "f16")
    fz = convert(fs, Z)
    assert fz.W == 0 and fz.nvec == 0 and fz.n_items == 0 and fz.n_blocks == 0
    fs.fs_spmm(fz, torch.zeros((9, 16), dtype=torch.float16, device="cuda"))
    fs.fs_sddmm(fz, torch.zeros((0, 8), dtype=torch.float16, device="cuda"), torch.zeros((9, 8), dtype=torch.float16, device="cuda"))
    fs.fs_edge_softmax(fz, torch.zeros(0, dtype=torch.float16, device="cuda"))


def _mostly_empty_rows(seed):
    """Stored entries so thin that 256 consecutive ones span far more than 256 rows (the per-entry kernels
    then search the row pointers in place, not in LDS), next to a dense stretch where they span a few."""
    rng = np.random.default_rng(seed)
    M, K = 9000, 700
    rows, cols = [], []
    for r in range(0, 6000, 7):  # every seventh row, one to three entries
        k = int(rng.integers(1, 4))
        rows.append(np.full(k, r)); cols.append(rng.choice(K, k, replace=False))
    for r in range(6000, 6200):  # a dense stretch
        k = int(rng.integers(20, 60))
        rows.append(np.full(k, r)); cols.append(rng.choice(K, k, replace=False))
    rows.append(np.array([8999])); cols.append(np.array([3]))  # and the last row after 2800 empty ones
    key = np.unique(np.concatenate(rows).astype(np.int64) * K + np.concatenate(cols))
    return csr_from_coo(M, K, key // K, key % K, "u11", "f16", rng)


@pytest.mark.parametrize("V", [4, 8, 16])
def test_convert_mostly_empty_rows(fs, V):
    A = _mostly_empty_rows(V)
    fmt = convert(fs, A, V, 32)
    assert_format_equal(fmt, A, V, 32)
    assert_items_valid(fmt)
    assert_row_base_valid(fmt, A)


def test_convert_rejects_bad_csr_and_bad_args(fs):
    import torch
    A = random_csr(40, 40, 0.2, "f16", 9)
    rp, ci, va = upload_csr(A)
    bad = ci.clone()
    bad[3] = 40  # out of range
    with pytest.raises(fs.FsError) as e:
        fs.fs_convert(rp, bad, va, 40, 40)
    assert e.value.code == 2
    bad = ci.clone()
    lo = int(A.rowptr[np.argmax(np.diff(A.rowptr) >= 2)])
    bad[lo + 1] = bad[lo]  # duplicate column inside a row
    with pytest.raises(fs.FsError) as e:
        fs.fs_convert(rp, bad, va, 40, 40)
    assert e.value.code == 2
    badrp = rp.clone()
    badrp[5] = 10 ** 6
    with pytest.raises(fs.FsError) as e:
        fs.fs_convert(badrp, ci, va, 40, 40)
    assert e.value.code == 2
    with pytest.raises(fs.FsError) as e:
        fs.fs_convert(rp, ci, va, 40, 40, V=40)
    assert e.value.code == 1
    with pytest.raises(fs.FsError) as e:
        fs.fs_convert(rp, ci, va, 40, 40, chunk=48)  # not a multiple of KB
    assert e.value.code == 1
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(fs.FsError) as e:
        fs.fs_convert(rp, ci, va, 40, 40, arena=small)
    assert e.value.code == 4
    # formats the compute kernels do not implement are refused, not mis-computed
    fmt = fs.fs_convert(rp, ci, va, 40, 40, V=4, KB=4)
    B = to_dev(dense(40, 32, "n01", "f16", stream(0, 97, 1)).bits, "f16")
    with pytest.raises(fs.FsError) as e:
        fs.fs_spmm(fmt, B)
    assert e.value.code == 3


@pytest.mark.parametrize("name,V", [("cfg1_uniform", 8), ("cfg1_uniform", 16), ("cfg2_rmat16", 8), ("cfg2_rmat16", 16),
                                    ("cfg3_stencil", 8), ("cfg5_lognormal", 8), ("cfg4_rmat20", 8), ("cfg4_rmat20", 0)])
def test_convert_full_configs_bit_exact(fs, name, V):
    A = cfg(name)["A"]
    fmt = convert(fs, A, V, 32)
    V = fmt.V  # V = 0 leaves the height to the library
    ref = assert_format_equal(fmt, A, V, 32)
    assert_items_valid(fmt)
    assert_row_base_valid(fmt, A)
    print("\n%s V=%d: nnz=%d nvec=%d items=%d split=%d chunk=%d R(VxKB)=%.3f" % (
        name, V, A.nnz, fmt.nvec, fmt.n_items, fmt.n_split_items, fmt.chunk,
        oracle.issued_mac_ratio(ref.win_ptr, V, 32, A.nnz)))


# ------------------------------------------------------------------------ SpMM
def run_spmm(fs, A, B, V=8, chunk=0, strided=False):
    import torch
    fmt = convert(fs, A, V, 32, chunk)
    Bd = to_dev(B.bits, B.dtype)
    N = B.shape[1]
    if strided:  # leading dimensions larger than N
        Bbig = torch.zeros((B.shape[0], N + 8), dtype=Bd.dtype, device="cuda")
        Bbig[:, :N] = Bd
        Cbig = torch.full((A.M, N + 8), 7.0, dtype=Bd.dtype, device="cuda")
        fs.fs_spmm(fmt, Bbig[:, :N], out=Cbig[:, :N])
        assert (Cbig[:, N:] == 7.0).all(), "wrote outside the M x N region"
        return fmt, from_dev_bits(Cbig[:, :N])
    C = fs.fs_spmm(fmt, Bd)
    return fmt, from_dev_bits(C)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("N", [8, 32, 48, 64, 128, 200, 256])
def test_spmm_small(fs, N, V, dtype):
    A = random_csr(203, 150, 0.15, dtype, seed=N + V, empty_rows=0.2)  # 203 = ragged last window; >32 vectors per window
    B = dense(150, N, "n01", dtype, stream(1, 96, N))
    ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, dtype)
    for chunk, strided in ((0, False), (32, True)):  # chunk=32 cuts almost every window: partial-tile path
        fmt, C = run_spmm(fs, A, B, V, chunk, strided)
        check_close(C, ref, S, dtype, "spmm N=%d V=%d chunk=%d" % (N, V, chunk))
        if chunk:
            assert fmt.n_split_windows > 0


def test_spmm_identity_returns_B_bit_for_bit(fs):
    K, N = 1000, 128
    A = Csr(K, K, np.arange(K + 1, dtype=np.int32), np.arange(K, dtype=np.int32),
            round_to_bits(np.ones(K, dtype=np.float32), "f16"), "f16")
    B = dense(K, N, "n01", "f16", stream(2, 96, 0))
    _, C = run_spmm(fs, A, B)
    assert np.array_equal(C, B.bits)


def test_spmm_empty_matrix_writes_zeros(fs):
    import torch
    A = Csr(20, 16, np.zeros(21, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16), "f16")
    fmt = convert(fs, A)
    B = to_dev(dense(16, 32, "n01", "f16", stream(3, 96, 0)).bits, "f16")
    C = torch.full((20, 32), 5.0, dtype=torch.float16, device="cuda")
    fs.fs_spmm(fmt, B, out=C)
    assert (C == 0).all()


def test_spmm_is_deterministic_and_checks_arguments(fs):
    import torch
    c = cfg("cfg2_rmat16", 16)
    A, B = c["A"], c["spmm"][0]
    fmt = convert(fs, A, 8, 32, chunk=64)
    Bd = to_dev(B.bits, "f16")
    C1 = from_dev_bits(fs.fs_spmm(fmt, Bd))
    C2 = from_dev_bits(fs.fs_spmm(fmt, Bd))
    assert np.array_equal(C1, C2)
    with pytest.raises(fs.FsError) as e:  # N not a multiple of 8
        fs.fs_spmm(fmt, Bd[:, :12].contiguous())
    assert e.value.code == 1
    with pytest.raises(fs.FsError) as e:  # workspace too small
        fs.fs_spmm(fmt, Bd, work=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 4
    with pytest.raises(fs.FsError) as e:  # misaligned B
        fs.fs_spmm(fmt, Bd[:, 4:36])
    assert e.value.code == 1


@pytest.mark.parametrize("name,V", [("cfg1_uniform", 8), ("cfg1_uniform", 16), ("cfg2_rmat16", 8), ("cfg2_rmat16", 16),
                                    ("cfg3_stencil", 8), ("cfg4_rmat20", 8),
                                    # V = 0: the library's defaults (cfg 4 and cfg 5 then read bitmap-packed values)
                                    ("cfg2_rmat16", 0), ("cfg4_rmat20", 0), ("cfg5_lognormal", 0)])
def test_spmm_full_configs(fs, name, V):
    c = cfg(name)
    A = c["A"]
    for B in (c["spmm"] if "spmm" in c else [c["chain"]]):  # cfg 5: its stored values times H
        fmt, C = run_spmm(fs, A, B, V)
        if V == 0:  # cfg 5's rows share no columns: four rows; cfg 4's do: eight; both large: packed values
            assert fmt.V == (4 if name == "cfg5_lognormal" else 8)
            assert bool(fmt.packed) == (name in ("cfg4_rmat20", "cfg5_lognormal"))
        ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, A.dtype)
        check_close(C, ref, S, A.dtype, "%s spmm V=%d N=%d" % (name, fmt.V, B.shape[1]))
        del ref, S, C, fmt


# ----------------------------------------------------------------------- SDDMM
def run_sddmm(fs, A, X, Y, V=8, chunk=0):
    fmt = convert(fs, A, V, 32, chunk, with_vals=False)
    out = fs.fs_sddmm(fmt, to_dev(X.bits, X.dtype), to_dev(Y.bits, Y.dtype))
    return fmt, out


def check_sddmm(fs, A, X, Y, V, fmt, out_blk):
    ref, S = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, X.dtype)
    fr = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, None, V, 32)
    blk = from_dev_bits(out_blk)
    other = np.ones(blk.shape[0], dtype=bool)
    other[fr.csr_to_slot] = False
    assert (blk[other] == 0).all(), "positions outside the pattern must be +0.0"
    err = check_close(blk[fr.csr_to_slot], ref, S, X.dtype, "sddmm V=%d d=%d" % (V, X.shape[1]))
    csr_order = from_dev_bits(fs.fs_blk_to_csr(fmt, out_blk))
    assert np.array_equal(csr_order, blk[fr.csr_to_slot])
    # the same scores in CSR order straight from the kernel, with and without the blocked output beside them
    import torch
    Xd, Yd = to_dev(X.bits, X.dtype), to_dev(Y.bits, Y.dtype)
    both_csr = torch.full((A.nnz,), 7.0, dtype=Xd.dtype, device="cuda")
    both_blk = fs.fs_sddmm(fmt, Xd, Yd, out_csr=both_csr)
    assert np.array_equal(from_dev_bits(both_blk), blk) and np.array_equal(from_dev_bits(both_csr), csr_order)
    only_csr = fs.fs_sddmm(fmt, Xd, Yd, blocked=False)
    assert np.array_equal(from_dev_bits(only_csr), csr_order)
    return err


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("d", [8, 32, 40, 64, 128, 160])
def test_sddmm_small(fs, d, V, dtype):
    A = random_csr(203, 150, 0.15, dtype, seed=d + V, empty_rows=0.2)
    X = dense(203, d, "n01", dtype, stream(4, 96, d))
    Y = dense(150, d, "n01", dtype, stream(5, 96, d))
    fmt, out = run_sddmm(fs, A, X, Y, V, chunk=32 if d == 40 else 0)
    err = check_sddmm(fs, A, X, Y, V, fmt, out)
    assert err <= TOL, (d, V, dtype, err)


def test_sddmm_all_ones_pattern_is_dense_product(fs):
    M, K, d = 40, 70, 32
    rp = (np.arange(M + 1) * K).astype(np.int32)
    ci = np.tile(np.arange(K), M).astype(np.int32)
    A = Csr(M, K, rp, ci, np.zeros(M * K, dtype=np.uint16), "f16")
    X = dense(M, d, "u11", "f16", stream(6, 96, 0))
    Y = dense(K, d, "u11", "f16", stream(6, 96, 1))
    fmt, out = run_sddmm(fs, A, X, Y)
    got = bits_to_f64(from_dev_bits(fs.fs_blk_to_csr(fmt, out)), "f16").reshape(M, K)
    want = bits_to_f64(X.bits, "f16") @ bits_to_f64(Y.bits, "f16").T
    assert np.abs(got - want).max() <= 1e-2 * (np.abs(bits_to_f64(X.bits, "f16")) @ np.abs(bits_to_f64(Y.bits, "f16")).T).max()


@pytest.mark.parametrize("name,V", [("cfg1_uniform", 8), ("cfg1_uniform", 16), ("cfg2_rmat16", 8), ("cfg2_rmat16", 16)])
def test_sddmm_full_configs(fs, name, V):
    c = cfg(name)
    A = c["A"]
    X, Y = c["sddmm"]
    fmt, out = run_sddmm(fs, A, X, Y, V)
    err = check_sddmm(fs, A, X, Y, V, fmt, out)
    print("\n%s V=%d d=%d: scaled error %.3e" % (name, V, X.shape[1], err))
    assert err <= TOL


def test_chain_sddmm_then_spmm_config5(fs):
    """Scores from SDDMM (fp16) feed SpMM as A's values, both on the GPU; checked stage by stage."""
    c = cfg("cfg5_lognormal")
    A = c["A"]
    X, Y = c["sddmm"]
    H = c["chain"]
    fmt, scores_blk = run_sddmm(fs, A, X, Y, 8)
    err1 = check_sddmm(fs, A, X, Y, 8, fmt, scores_blk)
    assert err1 <= TOL
    C = from_dev_bits(fs.fs_spmm(fmt, to_dev(H.bits, "f16"), vals=scores_blk))
    # (a) SpMM alone: oracle fed the GPU's own fp16 scores
    gpu_scores = from_dev_bits(fs.fs_blk_to_csr(fmt, scores_blk))
    ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, gpu_scores, H.bits, "f16")
    err2 = check_close(C, ref, S, "f16", "cfg5 spmm on the GPU's own scores")
    # (b) the whole chain against an independent oracle chain (oracle scores rounded once to fp16)
    sref, _ = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, "f16")
    ref2, S2 = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, oracle.round_f64_to_bits(sref, "f16"), H.bits, "f16")
    err3 = check_close(C, ref2, S2, "f16", "cfg5 chain sddmm -> spmm", stages=2)
    print("\ncfg5 chain: sddmm %.3e, spmm-only %.3e, whole chain %.3e" % (err1, err2, err3))


def test_operands_beyond_4_gib_take_the_64_bit_address_path(fs):
    """B (SpMM) and Y (SDDMM) with a leading dimension that makes them span more than 4 GiB: the
    kernels switch from 32-bit offsets off a scalar base to 64-bit addresses."""
    import torch
    K, ld = 70000, 32768  # 70000 rows of 64 KiB: 4.6 GB
    A = random_csr(300, K, 0.002, "f16", seed=77, empty_rows=0.1)
    assert A.colidx.max() > 69000  # rows near the far end are read
    B = dense(K, 64, "n01", "f16", stream(8, 96, 0))
    X = dense(300, 32, "n01", "f16", stream(8, 96, 1))
    Y = dense(K, 32, "n01", "f16", stream(8, 96, 2))
    big = torch.zeros((K, ld), dtype=torch.float16, device="cuda")
    assert big.numel() * 2 > 1 << 32
    fmt = convert(fs, A)
    big[:, :64] = to_dev(B.bits, "f16")
    C = from_dev_bits(fs.fs_spmm(fmt, big[:, :64]))
    ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, "f16")
    check_close(C, ref, S, "f16", "spmm, B beyond 4 GiB")
    big[:, :32] = to_dev(Y.bits, "f16")
    out = fs.fs_sddmm(fmt, to_dev(X.bits, "f16"), big[:, :32])
    assert check_sddmm(fs, A, X, Y, 8, fmt, out) <= TOL
    del big
    torch.cuda.empty_cache()


def test_library_defaults(fs):
    """V = 0 means eight-row windows -- except for a large long-row matrix whose rows share no columns, which
    gets four.  A matrix with at least 4 Mi stored entries and at least twelve per row also gets its values
    bitmap-packed by the conversion, and fs_spmm on the format's own values reads those: bit for bit the result
    of the unpacked array."""
    import torch
    small = random_csr(500, 400, 0.05, "f16", seed=3)
    rp, ci, va = upload_csr(small)
    f0 = fs.fs_convert(rp, ci, va, small.M, small.K)
    assert f0.V == 8 and not f0.packed
    M, K, deg = 300000, 1 << 20, 14  # 4.2 M entries, 14 per row
    for shared, want_v in ((False, 4), (True, 8)):
        # shared: both rows of a pair store the same columns, so an eight-row window holds four distinct sets
        base = np.arange(M, dtype=np.int64) // 2 if shared else np.arange(M, dtype=np.int64)
        cols = (np.arange(deg, dtype=np.int64)[None, :] * 5003 + base[:, None] * 17) % K
        cols.sort(axis=1)
        assert (np.diff(cols, axis=1) > 0).all()
        A = Csr(M, K, (np.arange(M + 1, dtype=np.int64) * deg).astype(np.int32), cols.reshape(-1).astype(np.int32),
                round_to_bits(stream(0, 97, 5).standard_normal(M * deg, dtype=np.float32), "f16"), "f16")
        rp, ci, va = upload_csr(A)
        fmt = fs.fs_convert(rp, ci, va, A.M, A.K)
        assert fmt.V == want_v and fmt.packed
        assert_format_equal(fmt, A, want_v, 32)
        assert not fs.fs_convert(rp, ci, None, A.M, A.K, torch_dtype=torch.float16).packed  # pattern only: nothing to pack
        B = to_dev(dense(K, 64, "n01", "f16", stream(0, 97, 6)).bits, "f16")
        C_packed = fs.fs_spmm(fmt, B)
        C_plain = fs.fs_spmm(fmt, B, vals=fmt.vals_blk_t())
        assert torch.equal(C_packed, C_plain)
        rows = np.arange(0, M, 1171, dtype=np.int64)
        ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, from_dev_bits(B), "f16", rows=rows)
        check_close(from_dev_bits(C_packed[torch.from_numpy(rows).cuda()]), ref, S, "f16", "spmm on values packed by the conversion")
        del fmt, C_packed, C_plain, B
        torch.cuda.empty_cache()


@pytest.mark.parametrize("V", [4, 8, 16])
def test_new_values_for_the_same_pattern(fs, V):
    """fs_csr_to_blk re-lays CSR-order values into the blocked layout: bit for bit what a fresh conversion
    with those values produces, and fs_spmm accepts it as the value array."""
    A = random_csr(173, 211, 0.12, "bf16", seed=31 + V, empty_rows=0.2)
    fmt = convert(fs, A, V, 32)
    new_vals = round_to_bits(stream(9, 97, V).standard_normal(A.nnz, dtype=np.float32), "bf16")
    blk = fs.fs_csr_to_blk(fmt, to_dev(new_vals, "bf16"))
    ref = oracle.convert_ref(A.M, A.K, A.rowptr, A.colidx, new_vals, V, 32)
    assert np.array_equal(from_dev_bits(blk), ref.vals_blk)
    assert np.array_equal(from_dev_bits(fs.fs_blk_to_csr(fmt, blk)), new_vals)  # and back
    B = dense(A.K, 40, "n01", "bf16", stream(9, 98, V))
    C = from_dev_bits(fs.fs_spmm(fmt, to_dev(B.bits, "bf16"), vals=blk))
    want, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, new_vals, B.bits, "bf16")
    check_close(C, want, S, "bf16", "spmm on re-laid values")


def test_gather_probe_runs_and_checks_arguments(fs):
    """The measurement aid reads what fs_spmm reads: it must accept the same operands, write its sink and
    refuse a sink that is too small."""
    import torch
    A = random_csr(300, 200, 0.1, "f16", seed=3, empty_rows=0.2)
    fmt = convert(fs, A)
    B = to_dev(dense(A.K, 72, "n01", "f16", stream(3, 95, 0)).bits, "f16")
    sink = torch.full((1024 * 256,), -1, dtype=torch.int32, device="cuda")
    fs.fs_gather_probe(fmt, B, sink=sink)
    torch.cuda.synchronize()
    assert (sink[256 * 1024 - 256:] != -1).any() or (sink != -1).any()
    with pytest.raises(fs.FsError) as e:
        fs.fs_gather_probe(fmt, B, sink=torch.empty(1000, dtype=torch.int32, device="cuda"))
    assert e.value.code == 4
