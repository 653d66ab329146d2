"""GPU parity of the one-kernel sparse attention (through the C ABI) against the CPU oracle's fp64
definition.  Bar: |gpu - ref| <= 1e-2 * S with S = sum_p a_p |h_p| (+ the output type's subnormal floor);
rows of A without stored entries must be exactly zero."""
import ctypes

import numpy as np
import pytest

import oracle
from gpu_util import BAR, from_dev_bits, scaled_error, to_dev, upload_csr
from workloads import csr_from_coo, dense, make_config, random_csr, stream

pytestmark = pytest.mark.gpu
TOL = 1e-2  # the contract


def bar(dtype):
    """Regression bar of the fused chain: the probabilities and the output are each rounded once."""
    return min(TOL, 2 * BAR[dtype])


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2412_11007_amd as fs
    fs.load_library()  # raises if the HIP library is missing: there is no fallback
    return fs


def convert(fs, A, V=8, chunk=0):
    rp, ci, va = upload_csr(A)
    return fs.fs_convert(rp, ci, va, A.M, A.K, torch_dtype=va.dtype, V=V, chunk=chunk)


def run_and_check(fs, A, fmt, X, Y, H, scale, rows=None):
    out = fs.fs_attention(fmt, to_dev(X.bits, A.dtype), to_dev(Y.bits, A.dtype), to_dev(H.bits, A.dtype), scale=scale)
    got = from_dev_bits(out)
    ref, S = oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, H.bits, A.dtype, scale, rows=rows)
    if rows is not None:
        got = got[rows]
    return scaled_error(got, ref, S, A.dtype), got


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("d,N,scale,chunk", [
    (8, 8, 1.0, 0), (32, 64, 0.25, 0), (64, 128, 0.125, 32), (40, 136, -0.5, 64),
    (64, 256, 0.125, 0), (128, 264, 0.09, 32), (16, 520, 2.0, 0),
])
def test_attention_small(fs, V, dtype, d, N, scale, chunk):
    A = random_csr(203, 150, 0.15, dtype, seed=V + d + N, empty_rows=0.2)  # ragged last window, > 32 vectors per window
    X = dense(A.M, d, "n01", dtype, stream(7, 60, d))
    Y = dense(A.K, d, "n01", dtype, stream(7, 61, d))
    H = dense(A.K, N, "n01", dtype, stream(7, 62, N))
    fmt = convert(fs, A, V, chunk)
    err, got = run_and_check(fs, A, fmt, X, Y, H, scale)
    assert err <= bar(dtype)
    assert not got[np.diff(A.rowptr) == 0].any()


@pytest.mark.parametrize("V,chunk,N", [(8, 0, 128), (8, 32, 256), (4, 64, 64), (4, 96, 264), (16, 64, 136)])
def test_attention_windows_cut_across_items(fs, V, chunk, N):
    """A few very long rows: their windows span many work items, so the parts are merged by the second kernel."""
    rng = np.random.default_rng(V + chunk)
    M, K, d = 70, 6000, 32
    rows, cols = [], []
    for i in range(M):
        deg = 3000 if i in (3, 41) else (900 if i == 20 else int(rng.integers(0, 12)))
        rows.append(np.full(deg, i)); cols.append(rng.choice(K, size=deg, replace=False))
    A = csr_from_coo(M, K, np.concatenate(rows), np.concatenate(cols), "n01", "f16", rng)
    X = dense(M, d, "n01", "f16", stream(8, 60, 0))
    Y = dense(K, d, "n01", "f16", stream(8, 61, 0))
    H = dense(K, N, "n01", "f16", stream(8, 62, N))
    fmt = convert(fs, A, V, chunk)
    assert fmt.n_split_windows > 0
    err, got = run_and_check(fs, A, fmt, X, Y, H, 0.3)
    assert err <= bar("f16")
    err2, again = run_and_check(fs, A, fmt, X, Y, H, 0.3)
    assert np.array_equal(got, again)  # deterministic
    # peaked rows: with a large scale one entry takes nearly all the weight, so the running maximum moves a lot
    err, _ = run_and_check(fs, A, fmt, X, Y, H, 4.0)
    assert err <= bar("f16")


def test_attention_closed_forms(fs):
    """Zero queries average the neighbours; a single neighbour is copied exactly."""
    import torch
    A = random_csr(120, 90, 0.1, "f16", seed=5, empty_rows=0.1)
    X = dense(A.M, 16, "n01", "f16", stream(9, 60, 0)); X.bits[:] = 0
    Y = dense(A.K, 16, "n01", "f16", stream(9, 61, 0))
    H = dense(A.K, 64, "n01", "f16", stream(9, 62, 0))
    fmt = convert(fs, A, 8)
    err, _ = run_and_check(fs, A, fmt, X, Y, H, 3.0)
    assert err <= 2e-3  # equal weights 1/deg: only the fp32 sum and the final rounding remain
    rng = np.random.default_rng(4)
    M, K = 77, 50
    A1 = csr_from_coo(M, K, np.arange(M), rng.integers(0, K, M), "u01", "f16", rng)
    X = dense(M, 16, "n01", "f16", stream(9, 63, 0)); Y = dense(K, 16, "n01", "f16", stream(9, 64, 0))
    H = dense(K, 32, "n01", "f16", stream(9, 65, 0))
    out = fs.fs_attention(convert(fs, A1, 4), to_dev(X.bits, "f16"), to_dev(Y.bits, "f16"), to_dev(H.bits, "f16"), scale=0.7)
    assert np.array_equal(from_dev_bits(out), H.bits[A1.colidx])


@pytest.mark.parametrize("name,rows_n", [("cfg2_rmat16", 400), ("cfg5_lognormal", 300)])
def test_attention_full_size(fs, name, rows_n):
    cfg = make_config(name)
    A = cfg["A"]
    X, Y = cfg["sddmm"]
    H = cfg["chain"] if "chain" in cfg else cfg["spmm"][0]
    d = X.shape[1]
    fmt = convert(fs, A, V=0)
    deg = np.diff(A.rowptr)
    rows = np.unique(np.concatenate([np.argsort(deg)[-6:], np.nonzero(deg == 0)[0][:4],
                                     np.random.default_rng(2).integers(0, A.M, rows_n), [0, A.M - 1]]))
    err, _ = run_and_check(fs, A, fmt, X, Y, H, float(d) ** -0.5, rows=rows)
    assert err <= bar(A.dtype)


def test_attention_argument_errors(fs):
    import torch
    A = random_csr(64, 48, 0.2, "f16", seed=2)
    fmt = convert(fs, A, 8, chunk=32)
    X = to_dev(dense(64, 16, "n01", "f16", stream(1, 1, 1)).bits, "f16")
    Y = to_dev(dense(48, 16, "n01", "f16", stream(1, 1, 2)).bits, "f16")
    H = to_dev(dense(48, 32, "n01", "f16", stream(1, 1, 3)).bits, "f16")
    with pytest.raises(fs.FsError) as e:
        fs.fs_attention(fmt, X, Y, H, scale=float("inf"))
    assert e.value.code == 1
    with pytest.raises(fs.FsError) as e:  # N not a multiple of 8
        fs.fs_attention(fmt, X, Y, H[:, :12].contiguous())
    assert e.value.code == 1
    Xw = to_dev(dense(64, 136, "n01", "f16", stream(1, 1, 4)).bits, "f16")
    Yw = to_dev(dense(48, 136, "n01", "f16", stream(1, 1, 5)).bits, "f16")
    with pytest.raises(fs.FsError) as e:  # d > 128
        fs.fs_attention(fmt, Xw, Yw, H)
    assert e.value.code == 3
    hub = csr_from_coo(8, 4000, np.zeros(3000, dtype=np.int64), np.arange(3000), "u01", "f16", np.random.default_rng(0))
    fmt_h = convert(fs, hub, 8, chunk=32)
    need = fs.fs_attention_workspace_bytes(fmt_h, 32)
    assert need == fmt_h.n_split_items * 8 * (32 + 2) * 4 and need > 0
    Xh = to_dev(dense(8, 16, "n01", "f16", stream(1, 1, 6)).bits, "f16")
    Yh = to_dev(dense(4000, 16, "n01", "f16", stream(1, 1, 7)).bits, "f16")
    Hh = to_dev(dense(4000, 32, "n01", "f16", stream(1, 1, 8)).bits, "f16")
    with pytest.raises(fs.FsError) as e:
        fs.fs_attention(fmt_h, Xh, Yh, Hh, work=torch.empty(need - 16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 4


@pytest.mark.parametrize("V,N", [(8, 72), (4, 264)])
def test_attention_strided_operands(fs, V, N):
    """Leading dimensions larger than the widths: the operands are column slices of wider tensors, and
    nothing outside the M x N region of the output is written."""
    import torch
    dtype, d = "f16", 40
    A = random_csr(150, 120, 0.2, dtype, seed=50 + V, empty_rows=0.1)
    X = dense(A.M, d, "n01", dtype, stream(3, 80, 0)); Y = dense(A.K, d, "n01", dtype, stream(3, 80, 1))
    H = dense(A.K, N, "n01", dtype, stream(3, 80, 2))
    fmt = convert(fs, A, V, chunk=32)
    def widen(t, extra):
        big = torch.full((t.shape[0], t.shape[1] + extra), 3.0, dtype=t.dtype, device="cuda")
        big[:, :t.shape[1]] = t
        return big[:, :t.shape[1]]
    Xv, Yv, Hv = widen(to_dev(X.bits, dtype), 8), widen(to_dev(Y.bits, dtype), 24), widen(to_dev(H.bits, dtype), 16)
    out_big = torch.full((A.M, N + 8), 7.0, dtype=Hv.dtype, device="cuda")
    fs.fs_attention(fmt, Xv, Yv, Hv, scale=0.3, out=out_big[:, :N])
    assert (out_big[:, N:] == 7.0).all(), "wrote outside the M x N region"
    ref, S = oracle.attention(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, H.bits, dtype, 0.3)
    assert scaled_error(from_dev_bits(out_big[:, :N]), ref, S, dtype) <= TOL


# ------------------------------------------------------------------ the same kernel without the softmax
def chain_two_calls(fs, fmt, Xd, Yd, Hd):
    return from_dev_bits(fs.fs_spmm(fmt, Hd, vals=fs.fs_sddmm(fmt, Xd, Yd)))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("d,N,chunk", [(8, 8, 0), (32, 64, 32), (64, 128, 0), (40, 136, 64), (64, 256, 32), (128, 264, 0), (16, 520, 32)])
def test_sddmm_spmm_is_the_two_calls_bit_for_bit(fs, V, dtype, d, N, chunk):
    A = random_csr(203, 150, 0.15, dtype, seed=V + d + N + 1, empty_rows=0.2)
    X = dense(A.M, d, "n01", dtype, stream(11, 60, d)); Y = dense(A.K, d, "n01", dtype, stream(11, 61, d))
    H = dense(A.K, N, "n01", dtype, stream(11, 62, N))
    fmt = convert(fs, A, V, chunk)
    Xd, Yd, Hd = to_dev(X.bits, dtype), to_dev(Y.bits, dtype), to_dev(H.bits, dtype)
    fused = from_dev_bits(fs.fs_sddmm_spmm(fmt, Xd, Yd, Hd))
    assert np.array_equal(fused, chain_two_calls(fs, fmt, Xd, Yd, Hd))
    # and against the oracle's chain: scores by definition, rounded once to the element type, then the product
    sref, _ = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, dtype)
    ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, oracle.round_f64_to_bits(sref, dtype), H.bits, dtype)
    assert scaled_error(fused, ref, S, dtype) <= 2 * TOL  # two rounded stages: scores, then the output
    # a scale other than one multiplies the scores before they are rounded
    half = from_dev_bits(fs.fs_sddmm_spmm(fmt, Xd, Yd, Hd, scale=0.5))
    ref2, S2 = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, oracle.round_f64_to_bits(0.5 * sref, dtype), H.bits, dtype)
    assert scaled_error(half, ref2, S2, dtype) <= 2 * TOL


def test_sddmm_spmm_cut_windows_and_full_size(fs):
    rng = np.random.default_rng(17)
    M, K, d, N = 70, 6000, 32, 256
    rows, cols = [], []
    for i in range(M):
        deg = 3000 if i in (3, 41) else (900 if i == 20 else int(rng.integers(0, 12)))
        rows.append(np.full(deg, i)); cols.append(rng.choice(K, size=deg, replace=False))
    A = csr_from_coo(M, K, np.concatenate(rows), np.concatenate(cols), "n01", "f16", rng)
    fmt = convert(fs, A, 8, 64)
    assert fmt.n_split_windows > 0
    Xd = to_dev(dense(M, d, "n0_8th", "f16", stream(12, 60, 0)).bits, "f16")
    Yd = to_dev(dense(K, d, "n0_8th", "f16", stream(12, 61, 0)).bits, "f16")
    Hd = to_dev(dense(K, N, "n01", "f16", stream(12, 62, 0)).bits, "f16")
    assert np.array_equal(from_dev_bits(fs.fs_sddmm_spmm(fmt, Xd, Yd, Hd)), chain_two_calls(fs, fmt, Xd, Yd, Hd))
    cfg = make_config("cfg5_lognormal")
    A = cfg["A"]
    X, Y = cfg["sddmm"]
    fmt = convert(fs, A, V=0)
    Xd, Yd, Hd = to_dev(X.bits, "f16"), to_dev(Y.bits, "f16"), to_dev(cfg["chain"].bits, "f16")
    assert np.array_equal(from_dev_bits(fs.fs_sddmm_spmm(fmt, Xd, Yd, Hd)), chain_two_calls(fs, fmt, Xd, Yd, Hd))


def test_attention_on_a_matrix_without_entries(fs):
    """No stored entries at all: every output row is zero for both fused calls, and packing yields an empty array."""
    import torch
    from workloads import Csr
    A = Csr(20, 16, np.zeros(21, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16), "f16")
    fmt = convert(fs, A, 8)
    X = to_dev(dense(20, 16, "n01", "f16", stream(1, 90, 0)).bits, "f16")
    Y = to_dev(dense(16, 16, "n01", "f16", stream(1, 90, 1)).bits, "f16")
    H = to_dev(dense(16, 40, "n01", "f16", stream(1, 90, 2)).bits, "f16")
    for call in (fs.fs_attention, fs.fs_sddmm_spmm):
        out = torch.full((20, 40), 5.0, dtype=torch.float16, device="cuda")
        call(fmt, X, Y, H, out=out)
        assert (out == 0).all()
    C = torch.full((20, 40), 5.0, dtype=torch.float16, device="cuda")
    fs.fs_spmm_packed(fmt, fs.fs_pack_values(fmt), H, out=C)
    assert (C == 0).all()
