"""The compute entry points only queue kernels on the caller's stream, so they can be recorded into a
HIP graph.  The attention chain is captured once and replayed with fresh inputs in the same buffers;
every replay must reproduce the eager result bit for bit."""
import numpy as np
import pytest

from gpu_util import from_dev_bits, to_dev, upload_csr
from workloads import dense, random_csr, stream

pytestmark = pytest.mark.gpu


def test_chain_replays_from_a_graph(tmp_path):
    import torch
    import paper_2412_11007_amd as fs
    fs.load_library()
    A = random_csr(700, 900, 0.04, "f16", seed=21, empty_rows=0.1)
    rp, ci, va = upload_csr(A)
    fmt = fs.fs_convert(rp, ci, None, A.M, A.K, torch_dtype=va.dtype, chunk=64)  # chunk=64: windows are cut
    assert fmt.n_split_windows > 0
    d, N = 32, 64
    X = torch.empty((A.M, d), dtype=torch.float16, device="cuda")
    Y = torch.empty((A.K, d), dtype=torch.float16, device="cuda")
    H = torch.empty((A.K, N), dtype=torch.float16, device="cuda")
    scores = torch.empty(fmt.V * fmt.nvec, dtype=torch.float16, device="cuda")
    C = torch.empty((A.M, N), dtype=torch.float16, device="cuda")
    work = torch.empty(max(fs.fs_spmm_workspace_bytes(fmt, N), 16), dtype=torch.uint8, device="cuda")
    swork = torch.empty(max(fs.fs_edge_softmax_workspace_bytes(fmt), 16), dtype=torch.uint8, device="cuda")
    C1 = torch.empty((A.M, N), dtype=torch.float16, device="cuda")
    awork = torch.empty(max(fs.fs_attention_workspace_bytes(fmt, N), 16), dtype=torch.uint8, device="cuda")

    def chain():
        fs.fs_sddmm(fmt, X, Y, out=scores)
        fs.fs_edge_softmax(fmt, scores, out=scores, scale=0.2, work=swork)
        fs.fs_spmm(fmt, H, vals=scores, out=C, work=work)
        fs.fs_attention(fmt, X, Y, H, scale=0.2, out=C1, work=awork)  # the same chain as one kernel

    def fill(seed):
        X.copy_(to_dev(dense(A.M, d, "n01", "f16", stream(seed, 98, 0)).bits, "f16"))
        Y.copy_(to_dev(dense(A.K, d, "n01", "f16", stream(seed, 98, 1)).bits, "f16"))
        H.copy_(to_dev(dense(A.K, N, "n01", "f16", stream(seed, 98, 2)).bits, "f16"))

    fill(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        chain()
    for seed in (1, 2, 3):
        fill(seed)
        chain()
        torch.cuda.synchronize()
        eager_C, eager_scores, eager_C1 = from_dev_bits(C).copy(), from_dev_bits(scores).copy(), from_dev_bits(C1).copy()
        # the two routes agree up to the 16-bit rounding of scores and probabilities in the three-call one
        assert (C.float() - C1.float()).abs().max().item() <= 2e-2
        C.zero_()
        C1.zero_()
        scores.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(from_dev_bits(C), eager_C), "replay %d differs from the eager run" % seed
        assert np.array_equal(from_dev_bits(scores), eager_scores)
        assert np.array_equal(from_dev_bits(C1), eager_C1)
