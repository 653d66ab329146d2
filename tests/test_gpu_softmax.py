"""GPU parity of the edge softmax (through the C ABI) against the CPU oracle, and the attention chain
SDDMM -> softmax -> SpMM.  Bar: |gpu - ref| <= 1e-2 * ref (+ the output type's subnormal floor); positions
outside the pattern are +0.0 bit for bit."""
import numpy as np
import pytest

import oracle
from gpu_util import BAR, from_dev_bits, scaled_error, to_dev, upload_csr
from workloads import Csr, bits_to_f64, csr_from_coo, dense, make_config, random_csr, round_to_bits, stream

pytestmark = pytest.mark.gpu
TOL = 1e-2


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


def check(fs, A, fmt, out_blk, scale):
    """Relative error of the stored positions against the oracle; everything else must be +0.0."""
    ref = oracle.edge_softmax(A.M, A.rowptr, A.vals, A.dtype, scale=scale)
    got_csr = from_dev_bits(fs.fs_blk_to_csr(fmt, out_blk))
    err = scaled_error(got_csr, ref, ref, A.dtype)  # S = ref: plain relative error
    blk = from_dev_bits(out_blk).copy()
    blk[fmt.csr_to_slot_t().cpu().numpy()] = 0
    assert not blk.any(), "non-zero bits outside the pattern"
    # rows sum to one (within the rounding of deg terms)
    sums = np.bincount(np.repeat(np.arange(A.M), np.diff(A.rowptr)), weights=bits_to_f64(got_csr, A.dtype), minlength=A.M)
    deg = np.diff(A.rowptr)
    assert np.abs(sums[deg > 0] - 1).max() <= (2.0 ** -8 if A.dtype == "bf16" else 2.0 ** -10)
    return err


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("scale,chunk,inplace", [(1.0, 0, False), (0.25, 32, True), (-3.0, 64, False)])
def test_softmax_small(fs, V, dtype, scale, chunk, inplace):
    A = random_csr(203, 150, 0.15, dtype, seed=V + int(scale * 8) + 40, empty_rows=0.2)
    fmt = convert(fs, A, V, chunk)
    vals = fmt.vals_blk_t().clone()
    out = fs.fs_edge_softmax(fmt, vals, out=vals if inplace else None, scale=scale)
    assert check(fs, A, fmt, out, scale) <= BAR[A.dtype]


@pytest.mark.parametrize("V,chunk", [(8, 0), (8, 32), (16, 96), (4, 64)])
def test_softmax_windows_cut_across_items(fs, V, chunk):
    """A few very long rows: their windows span many work items, so the statistics are merged from parts."""
    rng = np.random.default_rng(V + chunk)
    M, K = 70, 6000
    rows, cols = [], []
    for i in range(M):
        deg = 3000 if i in (3, 41) else (900 if i == 20 else int(rng.integers(0, 12)))
        cs = rng.choice(K, size=deg, replace=False)
        rows.append(np.full(deg, i)); cols.append(cs)
    rows, cols = np.concatenate(rows), np.concatenate(cols)
    A = csr_from_coo(M, K, rows, cols, "n01", "f16", rng)
    fmt = convert(fs, A, V, chunk)
    assert fmt.n_split_windows > 0
    out = fs.fs_edge_softmax(fmt, fmt.vals_blk_t(), scale=1.5)
    assert check(fs, A, fmt, out, 1.5) <= BAR[A.dtype]
    again = fs.fs_edge_softmax(fmt, fmt.vals_blk_t(), scale=1.5)
    assert np.array_equal(from_dev_bits(out), from_dev_bits(again))  # deterministic
    # a workspace smaller than the parts need is refused before anything is launched
    import torch
    need = fs.fs_edge_softmax_workspace_bytes(fmt)
    assert need == fmt.n_split_items * 2 * V * 4
    with pytest.raises(fs.FsError) as e:
        fs.fs_edge_softmax(fmt, fmt.vals_blk_t(), work=torch.empty(need - 4, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 4


def test_softmax_special_rows_and_arguments(fs):
    import torch
    # uniform scores -> 1/deg exactly where 1/deg is representable; a single entry -> 1; an empty matrix
    rowptr = np.array([0, 4, 4, 5, 13], dtype=np.int32)
    colidx = np.array([0, 5, 9, 30, 2, 1, 2, 3, 4, 5, 6, 7, 8], dtype=np.int32)
    A = Csr(4, 40, rowptr, colidx, round_to_bits(np.full(13, 0.75, dtype=np.float32), "f16"), "f16")
    fmt = convert(fs, A)
    got = bits_to_f64(from_dev_bits(fs.fs_blk_to_csr(fmt, fs.fs_edge_softmax(fmt, fmt.vals_blk_t(), scale=2.0))), "f16")
    assert np.array_equal(got, np.array([0.25] * 4 + [1.0] + [0.125] * 8))
    E = Csr(16, 16, np.zeros(17, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16), "f16")
    fe = convert(fs, E)
    fs.fs_edge_softmax(fe, torch.empty(0, dtype=torch.float16, device="cuda"))
    # argument checks
    with pytest.raises(fs.FsError) as e:
        fs.fs_edge_softmax(fmt, fmt.vals_blk_t(), scale=float("nan"))
    assert e.value.code == 1
    with pytest.raises(fs.FsError) as e:
        fs.fs_edge_softmax(fmt, fmt.vals_blk_t(), scale=float("inf"))
    assert e.value.code == 1


@pytest.mark.parametrize("V", [4, 8])
def test_softmax_keeps_bf16_subnormal_probabilities(fs, V):
    """A peaked bf16 row: probabilities between 2^-133 and 2^-126 are subnormal in bf16 AND in fp32, the
    range where a fast fp32 exponential returns zero.  The kernel must still deliver them."""
    M, K = 9, 70
    rows = np.repeat(np.arange(M), 40)
    cols = np.tile(np.arange(40), M)
    A = csr_from_coo(M, K, rows, cols, "u01", "bf16", np.random.default_rng(0))
    # scores 0, -86, -86.5, ... -92: exp(-88) = 6e-39 and exp(-91.5) = 2e-40 are both bf16 subnormals
    row_scores = np.concatenate([[0.0], -86.0 - 0.5 * np.arange(13), -20.0 - np.arange(26)]).astype(np.float32)
    A.vals = np.tile(round_to_bits(row_scores, "bf16"), M)
    fmt = convert(fs, A, V)
    out = fs.fs_edge_softmax(fmt, fmt.vals_blk_t(), scale=1.0)
    got = bits_to_f64(from_dev_bits(fs.fs_blk_to_csr(fmt, out)), "bf16")
    ref = oracle.edge_softmax(A.M, A.rowptr, A.vals, "bf16", scale=1.0)
    tiny = (ref > 0) & (ref < 2.0 ** -126)
    assert tiny.sum() >= 5 * M and (got[tiny] > 0).all()
    assert check(fs, A, fmt, out, 1.0) <= BAR[A.dtype]


@pytest.mark.parametrize("name", ["cfg2_rmat16", "cfg5_lognormal"])
def test_attention_chain_full_configs(fs, name):
    """SDDMM scores -> edge softmax -> SpMM on the GPU, each stage against the oracle fed the GPU's own
    16-bit input of that stage, and the whole chain against an independent oracle chain."""
    c = make_config(name)
    A = c["A"]
    X, Y = c["sddmm"]
    H = c["chain"] if "chain" in c else c["spmm"][0]
    d = X.shape[1]
    scale = 1.0 / np.sqrt(d)
    fmt = convert(fs, A)
    scores = fs.fs_sddmm(fmt, to_dev(X.bits, "f16"), to_dev(Y.bits, "f16"))
    att = fs.fs_edge_softmax(fmt, scores, scale=scale)
    C = from_dev_bits(fs.fs_spmm(fmt, to_dev(H.bits, "f16"), vals=att))
    # stage 2 alone
    gpu_scores = from_dev_bits(fs.fs_blk_to_csr(fmt, scores))
    As = Csr(A.M, A.K, A.rowptr, A.colidx, gpu_scores, "f16")
    err_sm = check(fs, As, fmt, att, scale)
    # stage 3 alone
    gpu_att = from_dev_bits(fs.fs_blk_to_csr(fmt, att))
    ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, gpu_att, H.bits, "f16")
    err_spmm = scaled_error(C, ref, S, "f16")
    # whole chain, oracle only
    sref, _ = oracle.sddmm(A.M, A.K, A.rowptr, A.colidx, X.bits, Y.bits, "f16")
    aref = oracle.edge_softmax(A.M, A.rowptr, oracle.round_f64_to_bits(sref, "f16"), "f16", scale=scale)
    ref2, S2 = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, oracle.round_f64_to_bits(aref, "f16"), H.bits, "f16")
    err_chain = scaled_error(C, ref2, S2, "f16")
    print("\n%s attention chain: softmax %.3e, spmm %.3e, whole chain %.3e" % (name, err_sm, err_spmm, err_chain))
    assert err_sm <= TOL and err_spmm <= TOL and err_chain <= TOL


# ---------------------------------------------------------------- gradient of the edge softmax
def hub_csr(M, K, dtype, seed):
    """A few rows with thousands of entries (windows cut into many parts) among short and empty ones."""
    rng = np.random.default_rng(seed)
    rows, cols = [], []
    for i in range(M):
        deg = 3000 if i in (3, M - 2) else (900 if i == M // 2 else int(rng.integers(0, 12)))
        rows.append(np.full(deg, i)); cols.append(rng.choice(K, size=deg, replace=False))
    return csr_from_coo(M, K, np.concatenate(rows), np.concatenate(cols), "n01", dtype, rng)


def run_backward(fs, A, fmt, p_bits, g_bits, scale, inplace=False):
    """GPU gradient for probabilities / incoming gradients given in CSR order; returns (CSR-order bits, blocked bits)."""
    p_blk = fs.fs_csr_to_blk(fmt, to_dev(p_bits, A.dtype))
    g_blk = fs.fs_csr_to_blk(fmt, to_dev(g_bits, A.dtype))
    out = fs.fs_edge_softmax_backward(fmt, p_blk, g_blk, out=p_blk if inplace else None, scale=scale)
    got_csr = from_dev_bits(fs.fs_blk_to_csr(fmt, out))
    blk = from_dev_bits(out).copy()
    blk[fmt.csr_to_slot_t().cpu().numpy()] = 0
    assert not blk.any(), "non-zero bits outside the pattern"
    return got_csr


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("scale,chunk,inplace", [(1.0, 0, False), (0.25, 32, True), (-3.0, 64, False)])
def test_softmax_backward_small(fs, V, dtype, scale, chunk, inplace):
    """Probabilities from the GPU's own forward call (so they are what a training step would hold),
    a random incoming gradient; against the oracle on the same 16-bit inputs."""
    A = random_csr(203, 150, 0.15, dtype, seed=V + int(scale * 8) + 70, empty_rows=0.2)
    fmt = convert(fs, A, V, chunk)
    p_bits = from_dev_bits(fs.fs_blk_to_csr(fmt, fs.fs_edge_softmax(fmt, fmt.vals_blk_t(), scale=scale)))
    g_bits = round_to_bits(stream(V, 96, 1).normal(size=A.nnz).astype(np.float32), dtype)
    got = run_backward(fs, A, fmt, p_bits, g_bits, scale, inplace)
    ref, S = oracle.edge_softmax_backward(A.M, A.rowptr, p_bits, g_bits, dtype, scale=scale)
    assert scaled_error(got, ref, S, dtype) <= BAR[dtype]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V,chunk", [(8, 0), (8, 32), (16, 96), (4, 64)])
def test_softmax_backward_windows_cut_across_items(fs, V, chunk, dtype):
    """Rows of thousands of entries: the row sums of p * g are merged from the parts' partial sums."""
    A = hub_csr(70, 6000, dtype, seed=V + chunk)
    fmt = convert(fs, A, V, chunk)
    assert fmt.n_split_windows > 0
    p_bits = from_dev_bits(fs.fs_blk_to_csr(fmt, fs.fs_edge_softmax(fmt, fmt.vals_blk_t(), scale=1.5)))
    g_bits = round_to_bits(stream(V, 96, 2).normal(size=A.nnz).astype(np.float32), dtype)
    got = run_backward(fs, A, fmt, p_bits, g_bits, 1.5)
    ref, S = oracle.edge_softmax_backward(A.M, A.rowptr, p_bits, g_bits, dtype, scale=1.5)
    assert scaled_error(got, ref, S, dtype) <= BAR[dtype]
    assert np.array_equal(got, run_backward(fs, A, fmt, p_bits, g_bits, 1.5))  # deterministic
    import torch
    need = fs.fs_edge_softmax_workspace_bytes(fmt)
    blk = fs.fs_csr_to_blk(fmt, to_dev(p_bits, dtype))
    with pytest.raises(fs.FsError) as e:
        fs.fs_edge_softmax_backward(fmt, blk, blk, work=torch.empty(need - 4, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 4


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V", [4, 8, 16])
def test_softmax_backward_bit_exact(fs, V, dtype):
    """Probabilities k/64 and gradients that are multiples of 1/4: every product and every partial sum is
    exact in fp32 whatever the order, so the only rounding on either side is the one to the 16-bit type --
    GPU bits == oracle bits, hub rows cut into dozens of parts included."""
    A = hub_csr(70, 6000, dtype, seed=V + 5)
    rng = stream(V, 96, 3)
    deg = np.diff(A.rowptr)
    # p = k/64 with small k (the values need not sum to one: the kernel computes the formula on what it is given)
    p = rng.integers(0, 5, size=A.nnz).astype(np.float32) / 64.0
    g = rng.integers(-8, 9, size=A.nnz).astype(np.float32) / 4.0
    p_bits, g_bits = round_to_bits(p, dtype), round_to_bits(g, dtype)
    fmt = convert(fs, A, V, chunk=64)
    assert fmt.n_split_windows >= 3
    got = run_backward(fs, A, fmt, p_bits, g_bits, 0.5)
    ref, _ = oracle.edge_softmax_backward(A.M, A.rowptr, p_bits, g_bits, dtype, scale=0.5)
    # p g and the row sums are multiples of 2^-8 below 2^9 (17 bits), g - dot as well; times p = k/64 with k <= 4
    # and times the scale 1/2 that makes multiples of 2^-15 of at most 20 bits: exact in fp32 on the GPU as in fp64 here
    assert np.array_equal(ref * 2.0 ** 15, np.rint(ref * 2.0 ** 15)) and np.abs(ref).max() < 2.0 ** 5
    want = oracle.round_f64_to_bits(ref, dtype)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, "%d of %d differ, first at %d: gpu 0x%04x, expected 0x%04x (degree %d)" % (
        bad.size, got.size, bad[0], got[bad[0]], want[bad[0]], deg[np.searchsorted(A.rowptr, bad[0], side="right") - 1])


def test_softmax_backward_arguments_and_empty(fs):
    import torch
    A = random_csr(40, 30, 0.2, "f16", seed=3)
    fmt = convert(fs, A)
    v = fmt.vals_blk_t()
    for bad in (float("nan"), float("inf")):
        with pytest.raises(fs.FsError) as e:
            fs.fs_edge_softmax_backward(fmt, v, v, scale=bad)
        assert e.value.code == 1
    E = Csr(16, 16, np.zeros(17, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16), "f16")
    fe = convert(fs, E)
    z = torch.empty(0, dtype=torch.float16, device="cuda")
    fs.fs_edge_softmax_backward(fe, z, z)


def test_attention_backward_chain_matches_finite_differences(fs):
    """The calls compose into the backward pass of out = softmax_rows(scale * X Y^T at A's pattern) * H:
        P = fs_edge_softmax(fs_sddmm(X, Y)),  G = fs_sddmm(dOut, H),  dS = fs_edge_softmax_backward(P, G),
        dX = fs_spmm(values dS, Y),  dY = fs_spmm(A^T, values dS, X),  dH = fs_spmm(A^T, values P, dOut).
    Checked against central differences of the fp64 attention oracle for L = sum(out * dOut); the chain rounds
    P, G and dS to 16 bits on the way, hence the loose bar."""
    M, K, d, N, scale = 24, 40, 16, 16, 0.25
    A = random_csr(M, K, 0.2, "f16", seed=12, empty_rows=0.1)
    rng = np.random.default_rng(4)
    Xf = (np.round(rng.normal(size=(M, d)) * 8) / 8).astype(np.float32)
    Yf = (np.round(rng.normal(size=(K, d)) * 8) / 8).astype(np.float32)
    Hf = (np.round(rng.normal(size=(K, N)) * 8) / 8).astype(np.float32)
    Rf = (np.round(rng.normal(size=(M, N)) * 8) / 8).astype(np.float32)
    Xb, Yb, Hb, Rb = (round_to_bits(a, "f16") for a in (Xf, Yf, Hf, Rf))
    fmt = convert(fs, A)
    X, Y, H, R = (to_dev(b, "f16") for b in (Xb, Yb, Hb, Rb))
    P = fs.fs_edge_softmax(fmt, fs.fs_sddmm(fmt, X, Y), scale=scale)
    G = fs.fs_sddmm(fmt, R, H)
    dS = fs.fs_edge_softmax_backward(fmt, P, G, scale=scale)
    dX = bits_to_f64(from_dev_bits(fs.fs_spmm(fmt, Y, vals=dS)), "f16")

    def loss(Xv):
        out, _ = oracle.attention(M, K, A.rowptr, A.colidx, round_to_bits(Xv.astype(np.float32), "f16"), Yb, Hb, "f16", scale)
        return float((out * Rf.astype(np.float64)).sum())

    # X moves on the fp16 grid: steps of 2^-6 around values that are multiples of 1/8 stay exactly representable
    h = 2.0 ** -6
    fd = np.zeros((M, d))
    for i in range(M):
        for t in range(d):
            E = np.zeros((M, d)); E[i, t] = h
            fd[i, t] = (loss(Xf + E) - loss(Xf - E)) / (2 * h)
    scale_of = np.abs(fd).max()
    assert np.abs(dX - fd).max() <= 2e-2 * scale_of, (np.abs(dX - fd).max(), scale_of)

    # dY = dS^T X and dH = P^T dOut: the same products on the converted transpose, values carried over by the
    # permutation fs_csr_transpose returns
    import torch
    rp, ci, _ = upload_csr(A)
    rp_t, ci_t, perm = fs.fs_csr_transpose(rp, ci, M, K)
    P_t = fs.fs_gather16(fs.fs_blk_to_csr(fmt, P), perm)
    fmt_t = fs.fs_convert(rp_t, ci_t, P_t, K, M, torch_dtype=torch.float16)
    dH = bits_to_f64(from_dev_bits(fs.fs_spmm(fmt_t, R)), "f16")
    dS_t = fs.fs_csr_to_blk(fmt_t, fs.fs_gather16(fs.fs_blk_to_csr(fmt, dS), perm))
    dY = bits_to_f64(from_dev_bits(fs.fs_spmm(fmt_t, X, vals=dS_t)), "f16")

    def loss_yh(Yv, Hv):
        out, _ = oracle.attention(M, K, A.rowptr, A.colidx, Xb, round_to_bits(Yv.astype(np.float32), "f16"),
                                  round_to_bits(Hv.astype(np.float32), "f16"), "f16", scale)
        return float((out * Rf.astype(np.float64)).sum())

    fdY, fdH = np.zeros((K, d)), np.zeros((K, N))
    for k in range(K):
        for t in range(d):
            E = np.zeros((K, d)); E[k, t] = h
            fdY[k, t] = (loss_yh(Yf + E, Hf) - loss_yh(Yf - E, Hf)) / (2 * h)
        for t in range(N):
            E = np.zeros((K, N)); E[k, t] = h
            fdH[k, t] = (loss_yh(Yf, Hf + E) - loss_yh(Yf, Hf - E)) / (2 * h)
    assert np.abs(dY - fdY).max() <= 2e-2 * np.abs(fdY).max(), (np.abs(dY - fdY).max(), np.abs(fdY).max())
    assert np.abs(dH - fdH).max() <= 2e-2 * np.abs(fdH).max(), (np.abs(dH - fdH).max(), np.abs(fdH).max())
