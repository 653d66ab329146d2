#!/usr/bin/env python3
"""Benchmark of the SpMM / SDDMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2_rmat16]

One step = one pass of the two operators over the workload, inputs resident in
HBM: fs_sddmm (where the workload has X, Y) followed by fs_spmm.  The format
conversion (fs_convert) runs once per sparsity pattern, so it is executed and
timed in the same run but reported separately (``convert``), not inside the
step.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes_spmm(nvec, M, W, V, N):
    """Bytes the method moves per SpMM: per nonzero vector a column index (4), its V values (2V)
    and one gathered row of B (2N); per output row 2N; per window one pointer (4)."""
    return nvec * (4 + 2 * V + 2 * N) + M * 2 * N + W * 4


def algorithmic_bytes_sddmm(nvec, M, W, V, d):
    """Per nonzero vector: index (4), mask (4), gathered Y row (2d), V written scores (2V);
    per window row 2d of X; per window one pointer (4)."""
    return nvec * (4 + 4 + 2 * d + 2 * V) + M * 2 * d + W * 4


def algorithmic_bytes_attention(nvec, M, W, V, d, N):
    """The fused chain: per nonzero vector an index (4), a mask (4), a gathered row of Y (2d) and of H (2N);
    per row 2d of X and 2N of output; per window one pointer (4).  No score or probability array."""
    return nvec * (4 + 4 + 2 * d + 2 * N) + M * (2 * d + 2 * N) + W * 4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg2_rmat16")
    ap.add_argument("--graph", action="store_true", help="also time the step replayed from a HIP graph")
    ap.add_argument("--packed", action="store_true", help="also time fs_spmm_packed (bitmap-packed values)")
    ap.add_argument("--V", type=int, default=0)
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--event-every", type=int, default=32,
                    help="record per-kernel HIP events on every n-th timed step (each pair costs a few us of stream time)")
    ap.add_argument("--operand", type=int, default=None, metavar="I",
                    help="which of the workload's dense SpMM operands to use (cfg3 has N=64 and N=256)")
    ap.add_argument("--softmax", action="store_true",
                    help="attention chain: fs_sddmm -> fs_edge_softmax -> fs_spmm on the softmaxed scores")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="only run the library's plain copy kernel on this many MiB, 10 times, and report GB/s "
                         "(gives a profiler's byte counters a kernel of known traffic)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path shards by row windows with no "
              "collective). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2412_11007_amd as fs
    from gpu_util import from_dev_bits, to_dev, upload_csr
    from workloads import bits_to_f64, make_config

    fs.load_library()
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.zeros(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fs.fs_copy_bytes(dst, src)
        e0.record()
        for _ in range(10):
            fs.fs_copy_bytes(dst, src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        print(json.dumps({"copy_MiB": args.calibrate_copy, "bytes_read": n, "bytes_written": n, "ms": ms,
                          "GBs_read_plus_write": 2 * n / ms / 1e6}))
        return
    cfg = make_config(args.workload)
    A = cfg["A"]
    if args.operand is not None:
        B = cfg["spmm"][args.operand]
    else:
        B = cfg["chain"] if "chain" in cfg else cfg["spmm"][-1 if args.workload != "cfg3_stencil" else 0]
    N = B.shape[1]
    has_sddmm = "sddmm" in cfg
    rp, ci, va = upload_csr(A)
    Bd = to_dev(B.bits, B.dtype)
    if has_sddmm:
        Xd, Yd = to_dev(cfg["sddmm"][0].bits, A.dtype), to_dev(cfg["sddmm"][1].bits, A.dtype)
        d = cfg["sddmm"][0].shape[1]

    # ---- conversion, timed separately (includes its host synchronisation)
    a_bytes, s_bytes = fs.fs_format_bytes(A.M, A.nnz, args.V, 0, 0 if A.dtype == "f16" else 1)
    arena = torch.empty(a_bytes, dtype=torch.uint8, device="cuda")
    scratch = torch.empty(s_bytes, dtype=torch.uint8, device="cuda")
    conv_ms = []
    for _ in range(5):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fmt = fs.fs_convert(rp, ci, va, A.M, A.K, V=args.V, chunk=args.chunk, arena=arena, scratch=scratch)
        torch.cuda.synchronize()
        conv_ms.append((time.perf_counter() - t0) * 1e3)
    # CSR of A^T (what a backward pass converts next), timed the same way
    tr_ms = []
    for _ in range(5):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tr = fs.fs_csr_transpose(rp, ci, A.M, A.K)
        torch.cuda.synchronize()
        tr_ms.append((time.perf_counter() - t0) * 1e3)
    del tr
    V = fmt.V
    chain = "chain" in cfg or args.softmax  # SDDMM scores feed SpMM as A's values
    if args.softmax and not has_sddmm:
        raise SystemExit("--softmax needs a workload with an SDDMM stage")

    C = torch.empty((A.M, N), dtype=Bd.dtype, device="cuda")
    work = torch.empty(max(fs.fs_spmm_workspace_bytes(fmt, N), 16), dtype=torch.uint8, device="cuda")
    scores = torch.empty(fmt.V * fmt.nvec, dtype=Bd.dtype, device="cuda") if has_sddmm else None
    sm_work = torch.empty(max(fs.fs_edge_softmax_workspace_bytes(fmt), 16), dtype=torch.uint8, device="cuda")
    sm_scale = 1.0 / float(np.sqrt(d)) if has_sddmm else 1.0

    K, Wm = args.steps, args.warmup
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(K)]
    for e4 in ev:  # create the underlying HIP events so that the library can record them
        for e in e4:
            e.record()

    every = max(1, min(args.event_every, args.steps // 16))  # at least sixteen timed samples

    def step(i, timed):
        timed = timed and (i % every == 0)
        if has_sddmm:
            if timed:
                ev[i][0].record()
            fs.fs_sddmm(fmt, Xd, Yd, out=scores)
            if timed:
                ev[i][1].record()
            if args.softmax:
                fs.fs_edge_softmax(fmt, scores, out=scores, scale=sm_scale, work=sm_work)
                if timed:
                    ev[i][4].record()
        vals = scores if chain else None
        evs = (ev[i][2].cuda_event, ev[i][3].cuda_event) if timed else None
        fs.fs_spmm(fmt, Bd, vals=vals, out=C, work=work, events=evs)

    for i in range(Wm):
        step(i % max(K, 1), False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(i, True)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K

    # ---- the same step replayed from a HIP graph (one capture, K replays): what a caller with a fixed
    # launch sequence gets; reported beside the eager figure, which stays the headline
    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0, False)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step(0, False)
        for _ in range(min(Wm, 20)):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / K

    sampled = range(0, K, every)
    spmm_ms = np.array([ev[i][2].elapsed_time(ev[i][3]) for i in sampled])
    sddmm_ms = np.array([ev[i][0].elapsed_time(ev[i][1]) for i in sampled]) if has_sddmm else None
    softmax_ms = np.array([ev[i][1].elapsed_time(ev[i][4]) for i in sampled]) if args.softmax else None

    # ---- the same attention chain as one fused kernel (fs_attention), timed beside the three calls
    fused = None
    if args.softmax:
        att_work = torch.empty(max(fs.fs_attention_workspace_bytes(fmt, N), 16), dtype=torch.uint8, device="cuda")
        C2 = torch.empty_like(C)
        n_f = max(5, min(K, 200))
        fe = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_f)]
        for _ in range(3):
            fs.fs_attention(fmt, Xd, Yd, Bd, scale=sm_scale, out=C2, work=att_work)
        for a, b in fe:
            a.record()
            fs.fs_attention(fmt, Xd, Yd, Bd, scale=sm_scale, out=C2, work=att_work)
            b.record()
        torch.cuda.synchronize()
        f_ms = np.array([a.elapsed_time(b) for a, b in fe])
        # the two paths round differently (the chain stores 16-bit scores and probabilities); report how far apart
        diff = (C2.float() - C.float()).abs().max().item()
        fused = {"us_avg": float(f_ms.mean()) * 1e3, "us_min": float(f_ms.min()) * 1e3,
                 "three_calls_us": ms_per_step * 1e3, "max_abs_diff_vs_three_calls": diff,
                 "algorithmic_GBs": algorithmic_bytes_attention(fmt.nvec, A.M, fmt.W, fmt.V, d, N) / (float(f_ms.mean()) * 1e-3) / 1e9,
                 "gflops": (2.0 * A.nnz * (d + N)) / (float(f_ms.mean()) * 1e-3) / 1e9}
        del C2, att_work

    # ---- SDDMM -> SpMM as one kernel (fs_sddmm_spmm), beside the two calls of the step, where the workload chains them
    fused_chain = None
    if chain and not args.softmax and fmt.V in (4, 8) and d <= 128:
        fc_work = torch.empty(max(fs.fs_attention_workspace_bytes(fmt, N), 16), dtype=torch.uint8, device="cuda")
        C3 = torch.empty_like(C)
        n_f = max(5, min(K, 200))
        fe = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_f)]
        for _ in range(3):
            fs.fs_sddmm_spmm(fmt, Xd, Yd, Bd, out=C3, work=fc_work)
        for a, b in fe:
            a.record()
            fs.fs_sddmm_spmm(fmt, Xd, Yd, Bd, out=C3, work=fc_work)
            b.record()
        torch.cuda.synchronize()
        f_ms = np.array([a.elapsed_time(b) for a, b in fe])
        fused_chain = {"us_avg": float(f_ms.mean()) * 1e3, "us_min": float(f_ms.min()) * 1e3,
                       "two_calls_us": ms_per_step * 1e3, "bit_identical_to_two_calls": bool(torch.equal(C3, C))}
        del C3, fc_work

    # ---- SpMM on bitmap-packed values beside the plain call (whole calls, cut-window merge included)
    packed = None
    if args.packed:
        t0 = time.perf_counter()
        pbuf = fs.fs_pack_values(fmt, vals=(scores if chain else None))
        torch.cuda.synchronize()
        pack_ms = (time.perf_counter() - t0) * 1e3
        n_p = max(5, min(K, 200))
        res = {}
        for name, call in (("plain", lambda: fs.fs_spmm(fmt, Bd, vals=(scores if chain else None), out=C, work=work)),
                           ("packed", lambda: fs.fs_spmm_packed(fmt, pbuf, Bd, out=C, work=work))):
            pe = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_p)]
            for _ in range(3):
                call()
            for a, b in pe:
                a.record()
                call()
                b.record()
            torch.cuda.synchronize()
            res[name] = np.array([a.elapsed_time(b) for a, b in pe])
        packed = {"us_avg": float(res["packed"].mean()) * 1e3, "us_min": float(res["packed"].min()) * 1e3,
                  "plain_call_us_avg": float(res["plain"].mean()) * 1e3, "plain_call_us_min": float(res["plain"].min()) * 1e3,
                  "pack_ms_first_call": pack_ms, "packed_bytes": int(pbuf.numel()),
                  "vals_blk_bytes": int(fmt.V * fmt.nvec * 2)}
        del pbuf

    # ---- context, outside the timed region: the box's plain streaming-copy rate (the ceiling a kernel
    # can actually reach) and SpMM right after 2 GiB of unrelated traffic has gone through the caches
    nb = 1 << 30
    src = torch.empty(nb, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nb, dtype=torch.uint8, device="cuda")
    ce = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    fs.fs_copy_bytes(dst, src)
    ce[0].record()
    for _ in range(5):
        fs.fs_copy_bytes(dst, src)
    ce[1].record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * nb * 5 / (ce[0].elapsed_time(ce[1]) * 1e-3) / 1e9
    cold_ms = []
    cold_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for e in cold_ev:
        e.record()
    for _ in range(5):
        fs.fs_copy_bytes(dst, src)
        fs.fs_spmm(fmt, Bd, vals=(scores if chain else None), out=C, work=work,
                   events=(cold_ev[0].cuda_event, cold_ev[1].cuda_event))
        torch.cuda.synchronize()
        cold_ms.append(cold_ev[0].elapsed_time(cold_ev[1]))
    del src, dst
    # the gather of fs_spmm alone (measurement aid): the floor under the main kernel's time on this matrix
    sink = torch.empty(1024 * 256, dtype=torch.int32, device="cuda")
    ge = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(3):
        fs.fs_gather_probe(fmt, Bd, sink=sink)
    n_g = max(5, min(K, 100))
    ge[0].record()
    for _ in range(n_g):
        fs.fs_gather_probe(fmt, Bd, sink=sink)
    ge[1].record()
    torch.cuda.synchronize()
    gather_us = ge[0].elapsed_time(ge[1]) * 1e3 / n_g

    flops_spmm = 2.0 * A.nnz * N
    flops_sddmm = 2.0 * A.nnz * d if has_sddmm else 0.0
    value = (flops_spmm + flops_sddmm) / (ms_per_step * 1e-3) / 1e9

    q_spmm = algorithmic_bytes_spmm(fmt.nvec, A.M, fmt.W, V, N)
    uniq_rows = int(np.unique(A.colidx).shape[0])
    q_min = fmt.nvec * (4 + 2 * V) + fmt.W * 4 + uniq_rows * 2 * N + A.M * 2 * N
    t_main = float(spmm_ms.mean()) * 1e-3
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s_spmm.json" % args.workload)
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
    roofline = {
        "bound": "hbm", "kernel": "k_spmm", "achieved": q_spmm / t_main / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": q_spmm / t_main / 1e9 / HBM_PEAK_GBS, "traffic": traffic,
        "algorithmic_bytes": q_spmm, "avg_launch_us": t_main * 1e6, "min_launch_us": float(spmm_ms.min()) * 1e3,
        "compulsory_bytes": q_min, "compulsory_frac": q_min / t_main / 1e9 / HBM_PEAK_GBS,
        # measured traffic (profiler counters, per launch) over this run's event-timed duration
        "traffic_GBs": (traffic / t_main / 1e9) if traffic else None,
        "traffic_frac": (traffic / t_main / 1e9 / HBM_PEAK_GBS) if traffic else None,
        # the same gather with nothing else around it (fs_gather_probe), back to back
        "gather_only_us": gather_us, "gather_only_over_kernel": gather_us / (t_main * 1e6),
    }

    # ---- a quick parity check of this run's output on sampled rows, and the CPU oracle leg
    cpu = None
    parity = None
    if not args.no_cpu:
        import oracle
        rows = np.unique(np.linspace(0, A.M - 1, 256).astype(np.int64))
        vals_bits = from_dev_bits(fs.fs_blk_to_csr(fmt, scores)) if chain else A.vals
        ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, vals_bits, B.bits, A.dtype, rows=rows)
        got = bits_to_f64(from_dev_bits(C[torch.from_numpy(rows).cuda()]), A.dtype)
        parity = float((np.maximum(np.abs(got - ref) - 2.0 ** -25, 0) / np.maximum(S, 1e-300)).max())
        # bounded sample: whole rows from the front of the matrix until ~4e9 fp64 MACs (a few seconds)
        budget = 4.0e9
        per_row = np.diff(A.rowptr).astype(np.float64) * N
        n_rows = int(min(A.M, np.searchsorted(np.cumsum(per_row), budget) + 1))
        srows = np.arange(n_rows, dtype=np.int64)
        times = []
        for _ in range(3 if n_rows == A.M else 1):
            t0 = time.perf_counter()
            oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, A.dtype, rows=srows, want_scale=False)
            times.append(time.perf_counter() - t0)
        macs = float(per_row[:n_rows].sum())
        cpu = {"value": 2.0 * macs / float(np.median(times)) / 1e9, "unit": "GFLOP/s", "cores": oracle.threads(),
               "kind": "oracle",
               "sample": "fp64 CSR SpMM N=%d on rows [0,%d) of %d (%.3g MACs), median of %d" % (
                   N, n_rows, A.M, macs, len(times))}

    out = {
        "metric": "SpMM & SDDMM effective GFLOP/s (2*nnz*N) at N=128; % of HBM roofline",
        "value": value, "unit": "GFLOP/s", "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": A.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "ops": (["sddmm d=%d" % d] if has_sddmm else []) + (["edge_softmax"] if args.softmax else []) + ["spmm N=%d" % N],
                   "M": A.M, "K": A.K, "nnz": A.nnz, "nvec": int(fmt.nvec), "V": int(V), "KB": int(fmt.KB),
                   "chunk": int(fmt.chunk), "items": int(fmt.n_items), "split_items": int(fmt.n_split_items),
                   "mfma": "16x16x32", "redundancy_VxKB": float(V * 32 * sum_blocks(fmt) / max(A.nnz, 1)),
                   "redundancy_mfma_16x32": float(16 * 32 * sum_blocks(fmt) / max(A.nnz, 1))},
        "spmm": {"gflops": flops_spmm / t_main / 1e9, "main_kernel_us_avg": t_main * 1e6,
                 "main_kernel_us_min": float(spmm_ms.min()) * 1e3, "main_kernel_us_median": float(np.median(spmm_ms)) * 1e3,
                 "main_kernel_us_cold_caches": float(np.median(cold_ms)) * 1e3},
        "stream_copy_GBs": copy_gbs,
        "sddmm": ({"gflops": flops_sddmm / (float(sddmm_ms.mean()) * 1e-3) / 1e9, "us_avg": float(sddmm_ms.mean()) * 1e3,
                   "us_min": float(sddmm_ms.min()) * 1e3,
                   "algorithmic_GBs": algorithmic_bytes_sddmm(fmt.nvec, A.M, fmt.W, V, d) / (float(sddmm_ms.mean()) * 1e-3) / 1e9}
                  if has_sddmm else None),
        "softmax": ({"us_avg": float(softmax_ms.mean()) * 1e3, "us_min": float(softmax_ms.min()) * 1e3,
                     "scale": sm_scale} if args.softmax else None),
        "ms_per_step_graph_replay": graph_ms,
        "attention_fused": fused,
        "sddmm_spmm_fused": fused_chain,
        "spmm_packed": packed,
        "convert": {"ms_median": float(np.median(conv_ms)), "ms_min": float(np.min(conv_ms)), "includes": "host sync",
                    "csr_transpose_ms_median": float(np.median(tr_ms)), "csr_transpose_ms_min": float(np.min(tr_ms))},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity_scaled_err_sampled_rows": parity,
    }
    print(json.dumps(out))


_blocks_cache = {}


def sum_blocks(fmt):
    """Number of 32-vector blocks the kernels issue (one matrix-core product per block and 16 columns)."""
    key = id(fmt)
    if key not in _blocks_cache:
        wp = fmt.win_ptr_t().cpu().numpy().astype(np.int64)
        n = np.diff(wp)
        _blocks_cache[key] = int(((n + 31) // 32).sum())
    return _blocks_cache[key]


if __name__ == "__main__":
    main()
