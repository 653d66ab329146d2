#!/usr/bin/env python3
"""Benchmark of the SpMM / SDDMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2_rmat16]

One step = one pass of the two operators over the workload, inputs resident in
HBM: fs_sddmm (where the workload has X, Y) followed by fs_spmm.  The format
conversion (fs_convert) runs once per sparsity pattern, so it is executed and
timed in the same run but reported separately (``convert``), not inside the
step.  Prints ONE JSON line.

Order of the run:
  1. before this process touches the GPU: two short child runs of this file under
     ``rocprofv3 --pmc`` (FETCH_SIZE, then WRITE_SIZE) read the bytes the SpMM kernel moves between L2
     and the fabric, per launch, calibrated on a plain copy of known size in the same child
     (``roofline.traffic``; skipped with --no-pmc or when rocprofv3 is missing);
  2. conversion, then a pass with HIP events around every kernel (per-kernel durations; it also
     brings the clocks up);
  3. the headline: W warm-up steps, then K bare steps -- no event is recorded inside the timed loop;
  4. context figures (gather-only probe, streaming copy, cold caches), the second power-law workload
     (``power_law``), and the CPU oracle on a bounded sample (``cpu_baseline``).

Byte figures, never mixed (each per launch of the SpMM main kernel):
  compulsory : every byte the method must move, once -- format arrays, the rows of B that are
               referenced at all, C.  ``roofline.frac`` = compulsory / time / 8 TB/s.
  hierarchy  : what the method asks of the memory hierarchy -- one row of B per nonzero vector,
               wherever it is served from.  May exceed the HBM peak; never called a fraction.
  fabric     : FETCH_SIZE + WRITE_SIZE, counted between L2 and the fabric; includes what the
               Infinity Cache serves, so it is an upper bound on HBM traffic, not HBM traffic.
"""
import argparse
import csv
import hashlib
import json
import os
import shutil
import subprocess
import sys
import tempfile
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
POWER_LAW = ("cfg2_rmat16", "cfg4_rmat20")
COPY_CAL_BYTES = 256 << 20


def log(msg):
    """Progress line on stderr (stdout carries the one JSON line)."""
    print("bench: " + msg, file=sys.stderr, flush=True)


def hierarchy_bytes_spmm(nvec, M, W, V, N):
    """Bytes the method asks for per SpMM: per nonzero vector a column index (4), its V values (2V)
    and one gathered row of B (2N); per output row 2N; per window one pointer (4)."""
    return nvec * (4 + 2 * V + 2 * N) + M * 2 * N + W * 4


def compulsory_bytes_spmm(nvec, M, W, V, N, unique_cols):
    """The same with every referenced row of B counted once."""
    return nvec * (4 + 2 * V) + W * 4 + unique_cols * 2 * N + M * 2 * N


def value_bytes_saved_by_packing(nvec, nnz, n_blocks, V):
    """Bitmap-packed values: per vector a mask byte (two for V = 16) instead of 2V value bytes, per stored entry
    2 bytes, per block slot a 4-byte offset."""
    return nvec * 2 * V - (nvec * (1 if V <= 8 else 2) + 2 * nnz + 4 * n_blocks)


def hierarchy_bytes_sddmm(nvec, M, W, V, d):
    """Per nonzero vector: index (4), mask (4), gathered Y row (2d), V written scores (2V);
    per window row 2d of X; per window one pointer (4)."""
    return nvec * (4 + 4 + 2 * d + 2 * V) + M * 2 * d + W * 4


def compulsory_bytes_sddmm(nvec, M, W, V, d, unique_cols):
    """The same with every referenced row of Y counted once."""
    return nvec * (4 + 4 + 2 * V) + W * 4 + unique_cols * 2 * d + M * 2 * d


def hierarchy_bytes_attention(nvec, M, W, V, d, N):
    """The fused chain: per nonzero vector an index (4), a mask (4), a gathered row of Y (2d) and of H (2N);
    per row 2d of X and 2N of output; per window one pointer (4).  No score or probability array."""
    return nvec * (4 + 4 + 2 * d + 2 * N) + M * (2 * d + 2 * N) + W * 4


def spmm_byte_model(fmt, A, N, unique_cols, packed):
    """(compulsory, hierarchy) bytes of one SpMM on this format, with the value stream the call really reads."""
    q_min = compulsory_bytes_spmm(fmt.nvec, A.M, fmt.W, fmt.V, N, unique_cols)
    q_hier = hierarchy_bytes_spmm(fmt.nvec, A.M, fmt.W, fmt.V, N)
    if packed:
        saved = value_bytes_saved_by_packing(fmt.nvec, A.nnz, fmt.n_blocks, fmt.V)
        q_min, q_hier = q_min - saved, q_hier - saved
    return q_min, q_hier


def source_stamp():
    """Hash of the library's sources: ties a stored counter reading to the code it was taken on."""
    h = hashlib.sha256()
    for d in (os.path.join(ROOT, "paper_2412_11007_amd", "csrc"), os.path.join(ROOT, "include")):
        for f in sorted(os.listdir(d)):
            if f.endswith((".hip", ".h")):
                h.update(f.encode())
                h.update(open(os.path.join(d, f), "rb").read())
    h.update(open(os.path.join(ROOT, "paper_2412_11007_amd", "build.py"), "rb").read())  # the compiler flags
    return h.hexdigest()[:16]


def spmm_kernel_pattern(dtype, V, packed=False):
    """Start of the SpMM main kernel's name for this element type and window height, as a profiler prints it."""
    return "k_spmm<%d, %d, " % (0 if dtype == "f16" else 1, V), (", true>" if packed else ", false>")


# ----------------------------------------------------------------------------- counter runs (children)
def save_workload(tmp, name, A, B):
    d = os.path.join(tmp, name)
    os.makedirs(d)
    for k, a in (("rowptr", A.rowptr), ("colidx", A.colidx), ("vals", A.vals), ("B", B.bits)):
        np.save(os.path.join(d, k + ".npy"), a)
    json.dump({"M": A.M, "K": A.K, "dtype": A.dtype}, open(os.path.join(d, "meta.json"), "w"))


def pmc_child(tmp, names):
    """Runs under rocprofv3: a plain copy of known size, then a few SpMM launches per workload."""
    import torch
    import paper_2412_11007_amd as fs
    from workloads import Csr
    from workloads.device import to_dev, upload_csr
    fs.load_library()
    torch.cuda.set_device(0)
    src = torch.zeros(COPY_CAL_BYTES, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        fs.fs_copy_bytes(dst, src)
    torch.cuda.synchronize()
    del src, dst
    for name in names:
        d = os.path.join(tmp, name)
        meta = json.load(open(os.path.join(d, "meta.json")))
        A = Csr(meta["M"], meta["K"], np.load(os.path.join(d, "rowptr.npy")), np.load(os.path.join(d, "colidx.npy")),
                np.load(os.path.join(d, "vals.npy")), meta["dtype"])
        Bd = to_dev(np.load(os.path.join(d, "B.npy")), A.dtype)
        rp, ci, va = upload_csr(A)
        fmt = fs.fs_convert(rp, ci, va, A.M, A.K)
        C = torch.empty((A.M, Bd.shape[1]), dtype=Bd.dtype, device="cuda")
        work = torch.empty(max(fs.fs_spmm_workspace_bytes(fmt, Bd.shape[1]), 16), dtype=torch.uint8, device="cuda")
        for _ in range(4):
            fs.fs_spmm(fmt, Bd, out=C, work=work)
        torch.cuda.synchronize()
        del fmt, C, work
        del Bd, rp, ci, va
        torch.cuda.empty_cache()


def read_counter(out_dir, counter):
    """{kernel name: mean counter value per dispatch, first dispatch of each kernel left out}."""
    per = {}
    for root, _, files in os.walk(out_dir):
        for f in files:
            if f.endswith("counter_collection.csv"):
                for r in csv.DictReader(open(os.path.join(root, f))):
                    if r["Counter_Name"] == counter:
                        per.setdefault(r["Kernel_Name"], []).append((int(r["Dispatch_Id"]), float(r["Counter_Value"])))
    out = {}
    for k, v in per.items():
        v.sort()
        vals = [x for _, x in v]
        out[k] = float(np.mean(vals[1:] if len(vals) > 1 else vals))
    return out


def measure_fabric_traffic(tmp, names, timeout_s=240):
    """Two child runs under rocprofv3 --pmc, before this process initialises the GPU.  Returns
    ({counter: {kernel: value}}, scale factors, note); empty on any failure."""
    if shutil.which("rocprofv3") is None:
        return {}, {}, "rocprofv3 not found"
    raw = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        out_dir = os.path.join(tmp, "pmc_" + counter)
        log("counter run %s (child under rocprofv3)" % counter)
        cmd = ["timeout", "-s", "KILL", str(timeout_s), "rocprofv3", "--output-format", "csv", "--pmc", counter,
               "--kernel-trace", "-d", out_dir, "-o", "x", "--", sys.executable, os.path.abspath(__file__),
               "--pmc-child", tmp, "--pmc-workloads", ",".join(names)]
        env = dict(os.environ, TMPDIR=tmp)
        try:
            res = subprocess.run(cmd, cwd=tmp, env=env, capture_output=True, text=True, timeout=timeout_s + 30)
        except subprocess.TimeoutExpired:
            return {}, {}, "counter run %s timed out" % counter
        if res.returncode != 0:
            return {}, {}, "counter run %s exited with %d: %s" % (counter, res.returncode, res.stderr[-300:])
        raw[counter] = read_counter(out_dir, counter)
        if not raw[counter]:
            return {}, {}, "counter run %s produced no %s rows" % (counter, counter)
    scale = {}
    for counter in raw:
        copy = [v for k, v in raw[counter].items() if k.startswith("k_copy16") or "::k_copy16" in k]
        if not copy or copy[0] <= 0:
            return {}, {}, "no reading for the calibration copy"
        scale[counter] = COPY_CAL_BYTES / copy[0]  # bytes per counter unit
    return raw, scale, "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE child runs of this bench run"


def fabric_bytes(raw, scale, dtype, V, packed=False):
    """FETCH_SIZE + WRITE_SIZE of the SpMM main kernel, in bytes per launch (None if not measured)."""
    if not raw:
        return None
    head, tail = spmm_kernel_pattern(dtype, V, packed)
    tot = 0.0
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        hit = [v for k, v in raw[counter].items() if head in k and (tail + "(") in k]
        if not hit:
            return None
        tot += hit[0] * scale[counter]
    return tot


# ----------------------------------------------------------------------------- timing helpers
def make_events(torch, n):
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
    for e in ev:  # create the underlying HIP events so that the library can record them
        e.record()
    return ev


def time_spmm_kernel(torch, fs, fmt, Bd, C, work, vals=None, n=20, warm=3):
    """(main-kernel durations, whole-call durations) in ms by HIP events on the launch stream."""
    for _ in range(warm):
        fs.fs_spmm(fmt, Bd, vals=vals, out=C, work=work)
    ev = [make_events(torch, 4) for _ in range(n)]
    for e in ev:
        e[0].record()
        fs.fs_spmm(fmt, Bd, vals=vals, out=C, work=work, events=(e[1].cuda_event, e[2].cuda_event))
        e[3].record()
    torch.cuda.synchronize()
    return (np.array([e[1].elapsed_time(e[2]) for e in ev]), np.array([e[0].elapsed_time(e[3]) for e in ev]))


def byte_figures(q_min, q_hier, q_fabric, t_s):
    out = {"compulsory_bytes": q_min, "compulsory_GBs": q_min / t_s / 1e9,
           "compulsory_frac": q_min / t_s / 1e9 / HBM_PEAK_GBS,
           "hierarchy_bytes": q_hier, "hierarchy_GBs": q_hier / t_s / 1e9,
           "fabric_bytes": q_fabric,
           "fabric_GBs": (q_fabric / t_s / 1e9) if q_fabric else None,
           "fabric_frac_of_8TBs": (q_fabric / t_s / 1e9 / HBM_PEAK_GBS) if q_fabric else None,
           "fabric_over_compulsory": (q_fabric / q_min) if q_fabric else None}
    return out


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
    ap.add_argument("--no-pmc", action="store_true", help="skip the rocprofv3 counter runs (use when this bench itself runs under a profiler)")
    ap.add_argument("--no-power-law", action="store_true", help="skip the second power-law workload")
    ap.add_argument("--event-steps", type=int, default=200, help="steps of the pass that records HIP events around every kernel")
    ap.add_argument("--operand", type=int, default=None, metavar="I",
                    help="which of the workload's dense SpMM operands to use (cfg3 has N=64 and N=256)")
    ap.add_argument("--softmax", action="store_true",
                    help="attention chain: fs_sddmm -> fs_edge_softmax -> fs_spmm on the softmaxed scores")
    ap.add_argument("--write-profiles", action="store_true",
                    help="store this run's counter readings under profiles/ (stamped with the source hash)")
    ap.add_argument("--profiles-dir", default=os.path.join(ROOT, "profiles"), help="where --write-profiles writes")
    ap.add_argument("--summarize", default=None, metavar="DIR",
                    help="print a short text summary of the rocprofv3 CSV output under DIR (kernel stats, mean counter "
                         "values per kernel) and exit: what the files under profiles/ are made from")
    ap.add_argument("--pmc-child", default=None, help=argparse.SUPPRESS)
    ap.add_argument("--pmc-workloads", default="", help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.summarize:
        summarize_profile(args.summarize)
        return
    if args.pmc_child:
        pmc_child(args.pmc_child, [n for n in args.pmc_workloads.split(",") if n])
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path shards by row windows with no "
              "collective). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    from workloads import bits_to_f64, make_config

    # ---- inputs (host side), and the counter runs, before anything in this process touches the GPU
    log("generating %s" % args.workload)
    cfg = make_config(args.workload)
    A = cfg["A"]
    if args.operand is not None:
        B = cfg["spmm"][args.operand]
    else:
        B = cfg["chain"] if "chain" in cfg else cfg["spmm"][-1 if args.workload != "cfg3_stencil" else 0]
    N = B.shape[1]
    has_sddmm = "sddmm" in cfg
    others = {}
    if not args.no_power_law and args.workload in POWER_LAW:
        for name in POWER_LAW:
            if name != args.workload:
                log("generating %s" % name)
                c2 = make_config(name)
                others[name] = (c2["A"], c2["spmm"][0])
                del c2
    tmp = tempfile.mkdtemp(prefix="fs_bench_")
    raw, scale, traffic_note = {}, {}, "not measured (--no-pmc)"
    try:
        if not args.no_pmc and not (has_sddmm and "chain" in cfg):
            save_workload(tmp, args.workload, A, B)
            for name, (A2, B2) in others.items():
                save_workload(tmp, name, A2, B2)
            raw, scale, traffic_note = measure_fabric_traffic(tmp, [args.workload] + list(others))
    finally:
        shutil.rmtree(tmp, ignore_errors=True)

    import torch
    import paper_2412_11007_amd as fs
    from workloads.device import from_dev_bits, to_dev, upload_csr

    fs.load_library()
    torch.cuda.set_device(0)
    log("counter runs: %s; now measuring %s" % (traffic_note, args.workload))
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

    # the two calls of a plain step with their arguments marshalled once (the binding's per-call checks cost
    # more host time than a 20-step run can hide behind the GPU)
    plain_step = not args.softmax
    call_spmm = fs.bind_spmm(fmt, Bd, C, work=work, vals=(scores if chain else None))
    call_sddmm = fs.bind_sddmm(fmt, Xd, Yd, out=scores) if has_sddmm else None

    def step(ev=None):
        """One pass of the hot path; with `ev` (seven events) every kernel is bracketed."""
        if ev is None and plain_step:
            if call_sddmm:
                call_sddmm()
            call_spmm()
            return
        if has_sddmm:
            if ev:
                ev[0].record()
            fs.fs_sddmm(fmt, Xd, Yd, out=scores)
            if ev:
                ev[1].record()
            if args.softmax:
                fs.fs_edge_softmax(fmt, scores, out=scores, scale=sm_scale, work=sm_work)
                if ev:
                    ev[2].record()
        vals = scores if chain else None
        if ev:
            ev[3].record()
            fs.fs_spmm(fmt, Bd, vals=vals, out=C, work=work, events=(ev[4].cuda_event, ev[5].cuda_event))
            ev[6].record()
        else:
            fs.fs_spmm(fmt, Bd, vals=vals, out=C, work=work)

    # ---- per-kernel durations: a pass of its own, HIP events on the launch stream around every kernel
    n_ev = max(5, args.event_steps if A.nnz < 4_000_000 else min(args.event_steps, 20))
    for _ in range(min(10, n_ev)):
        step()
    evs = [make_events(torch, 7) for _ in range(n_ev)]
    for e in evs:
        step(e)
    torch.cuda.synchronize()
    spmm_ms = np.array([e[4].elapsed_time(e[5]) for e in evs])
    spmm_call_ms = np.array([e[3].elapsed_time(e[6]) for e in evs])
    sddmm_ms = np.array([e[0].elapsed_time(e[1]) for e in evs]) if has_sddmm else None
    softmax_ms = np.array([e[1].elapsed_time(e[2]) for e in evs]) if args.softmax else None
    del evs

    # ---- the headline: W warm-up steps, K bare steps, nothing but the library calls in the loop
    log("event pass done; headline loop: %d warm-up + %d timed steps" % (Wm, K))
    for _ in range(Wm):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K

    # ---- the same step replayed from a HIP graph (one capture, K replays): what a caller with a fixed
    # launch sequence gets; reported beside the eager figure, which stays the headline
    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(min(Wm, 20)):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / K

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
                 "hierarchy_GBs": hierarchy_bytes_attention(fmt.nvec, A.M, fmt.W, fmt.V, d, N) / (float(f_ms.mean()) * 1e-3) / 1e9,
                 "gflops": (2.0 * A.nnz * (d + N)) / (float(f_ms.mean()) * 1e-3) / 1e9}
        del C2, att_work

    # ---- the gradient of the edge softmax (the operator a backward pass of the chain adds): the probabilities
    # the chain left in `scores`, and a gradient of the same shape (the SDDMM output layout; X, Y stand in for dOut, H)
    softmax_bwd = None
    if args.softmax:
        grad_in = fs.fs_sddmm(fmt, Xd, Yd)
        ds = torch.empty_like(scores)
        n_b = max(5, min(K, 200))
        be = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_b)]
        for _ in range(3):
            fs.fs_edge_softmax_backward(fmt, scores, grad_in, out=ds, scale=sm_scale, work=sm_work)
        for a, b in be:
            a.record()
            fs.fs_edge_softmax_backward(fmt, scores, grad_in, out=ds, scale=sm_scale, work=sm_work)
            b.record()
        torch.cuda.synchronize()
        b_ms = np.array([a.elapsed_time(b) for a, b in be])
        softmax_bwd = {"us_avg": float(b_ms.mean()) * 1e3, "us_min": float(b_ms.min()) * 1e3}
        del grad_in, ds

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

    # ---- SDDMM writing CSR-order output only (no blocked array), beside the blocked form of the step
    sddmm_csr_us = None
    if has_sddmm:
        out_csr = torch.empty(A.nnz, dtype=Bd.dtype, device="cuda")
        n_s = max(5, min(K, 200))
        se = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_s)]
        for _ in range(3):
            fs.fs_sddmm(fmt, Xd, Yd, out_csr=out_csr, blocked=False)
        for a, b in se:
            a.record()
            fs.fs_sddmm(fmt, Xd, Yd, out_csr=out_csr, blocked=False)
            b.record()
        torch.cuda.synchronize()
        sddmm_csr_us = float(np.mean([a.elapsed_time(b) for a, b in se])) * 1e3
        del out_csr

    # ---- SpMM on bitmap-packed values beside the plain call (whole calls, cut-window merge included)
    packed = None
    if args.packed:
        packed = time_packed(torch, fs, fmt, Bd, C, work, scores if chain else None, max(5, min(K, 200)))

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
    # what the L2s deliver to the CUs: 2048 workgroups re-reading 16 KiB chunks of a 16 MiB buffer (2 MiB per
    # XCD, L2-resident), 256 times in one kernel
    l2_sink = torch.empty(2048 * 256, dtype=torch.int32, device="cuda")
    le = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    fs.fs_read_bytes(src[: 16 << 20], repeats=256, sink=l2_sink)
    le[0].record()
    fs.fs_read_bytes(src[: 16 << 20], repeats=256, sink=l2_sink)
    le[1].record()
    torch.cuda.synchronize()
    l2_gbs = 2048.0 * 16384 * 256 / (le[0].elapsed_time(le[1]) * 1e-3) / 1e9
    del l2_sink
    cold_ms = []
    cold_ev = make_events(torch, 2)
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

    stamp = source_stamp()
    uniq_rows = int(np.unique(A.colidx).shape[0])
    reads_packed = bool(fmt.packed) and not chain  # the call reads the format's own values, packed by the conversion
    q_min, q_hier = spmm_byte_model(fmt, A, N, uniq_rows, reads_packed)
    t_main = float(spmm_ms.mean()) * 1e-3
    q_fabric = fabric_bytes(raw, scale, A.dtype, V, packed=reads_packed)
    traffic_source, traffic_stale = traffic_note, None
    if q_fabric is None:  # no live reading: the stored one, marked stale unless it was taken on these sources
        tpath = os.path.join(ROOT, "profiles", "fabric_traffic_%s_spmm.json" % args.workload)
        if os.path.exists(tpath):
            st = json.load(open(tpath))
            head, tail = spmm_kernel_pattern(A.dtype, V, packed=reads_packed)
            q_fabric = st.get("fabric_bytes_per_launch")
            traffic_stale = not (st.get("source_stamp") == stamp and head in st.get("kernel", ""))
            traffic_source = "stored reading profiles/%s (%s)" % (os.path.basename(tpath), traffic_note)
    figs = byte_figures(q_min, q_hier, q_fabric, t_main)
    roofline = {
        "bound": "hbm", "kernel": "k_spmm", "achieved": figs["compulsory_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": figs["compulsory_frac"], "traffic": q_fabric,
        "bytes_counted": "compulsory (format arrays + referenced rows of B once + C), per launch",
        "traffic_counts": "FETCH_SIZE + WRITE_SIZE between L2 and the fabric (includes Infinity Cache hits), per launch",
        "traffic_source": traffic_source, "traffic_stale": traffic_stale, "source_stamp": stamp,
        "avg_launch_us": t_main * 1e6, "min_launch_us": float(spmm_ms.min()) * 1e3,
        # the same gather with nothing else around it (fs_gather_probe), back to back
        "gather_only_us": gather_us, "gather_only_over_kernel": gather_us / (t_main * 1e6),
    }
    roofline.update({k: figs[k] for k in ("compulsory_bytes", "hierarchy_bytes", "hierarchy_GBs", "fabric_GBs",
                                          "fabric_frac_of_8TBs", "fabric_over_compulsory")})

    # ---- a quick parity check of this run's output on sampled rows, and the CPU oracle leg
    cpu = None
    parity = None
    if not args.no_cpu:
        import oracle
        log("CPU oracle leg")
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

    config = {"workload": args.workload, "ops": (["sddmm d=%d" % d] if has_sddmm else []) + (["edge_softmax"] if args.softmax else []) + ["spmm N=%d" % N],
              "M": A.M, "K": A.K, "nnz": A.nnz, "nvec": int(fmt.nvec), "V": int(V), "KB": int(fmt.KB),
              "chunk": int(fmt.chunk), "items": int(fmt.n_items), "split_items": int(fmt.n_split_items),
              "split_windows": int(fmt.n_split_windows),
              "mfma": "16x16x32", "redundancy_VxKB": float(V * 32 * sum_blocks(fmt) / max(A.nnz, 1)),
              "redundancy_mfma_16x32": float(16 * 32 * sum_blocks(fmt) / max(A.nnz, 1))}
    t_sddmm = float(sddmm_ms.mean()) * 1e-3 if has_sddmm else 0.0
    spmm_block = {"gflops": flops_spmm / t_main / 1e9, "main_kernel_us_avg": t_main * 1e6,
                  "main_kernel_us_min": float(spmm_ms.min()) * 1e3, "main_kernel_us_median": float(np.median(spmm_ms)) * 1e3,
                  # both launches of the call and the two event records inside it (a few us of stream time)
                  "whole_call_us_avg_with_inner_events": float(spmm_call_ms.mean()) * 1e3,
                  "main_kernel_us_cold_caches": float(np.median(cold_ms)) * 1e3}

    # ---- both power-law workloads side by side: this one from the figures above, the other measured now
    power_law = None
    if args.workload in POWER_LAW and not args.softmax and args.V == 0:
        power_law = {args.workload: dict(N=N, dtype=A.dtype, V=int(V), nnz=A.nnz, packed_values=reads_packed, kernel_us_avg=t_main * 1e6,
                                         kernel_us_min=float(spmm_ms.min()) * 1e3, whole_call_us_avg=float(spmm_call_ms.mean()) * 1e3,
                                         gflops=flops_spmm / t_main / 1e9, parity_scaled_err_sampled_rows=parity, **figs)}
        del Bd, C, work, scores, arena, scratch, fmt, rp, ci, va
        if has_sddmm:
            del Xd, Yd
        torch.cuda.empty_cache()
        for name, (A2, B2) in others.items():
            log("measuring %s" % name)
            power_law[name] = measure_power_law(torch, fs, name, A2, B2, raw, scale, not args.no_cpu)

    if args.write_profiles and raw:
        write_traffic_profiles(raw, scale, stamp, power_law, args)

    out = {
        "metric": "SpMM & SDDMM effective GFLOP/s (2*nnz*N) at N=128; % of HBM roofline",
        "value": value, "unit": "GFLOP/s", "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": A.dtype, "data": "synthetic",
        "config": config,
        "spmm": spmm_block,
        "stream_copy_GBs": copy_gbs, "l2_read_GBs": l2_gbs,
        "sddmm": ({"gflops": flops_sddmm / t_sddmm / 1e9, "us_avg": t_sddmm * 1e6,
                   "us_min": float(sddmm_ms.min()) * 1e3, "csr_order_output_only_us_avg": sddmm_csr_us,
                   "hierarchy_GBs": hierarchy_bytes_sddmm(config["nvec"], A.M, -(-A.M // V), V, d) / t_sddmm / 1e9,
                   "compulsory_bytes": compulsory_bytes_sddmm(config["nvec"], A.M, -(-A.M // V), V, d, uniq_rows),
                   "compulsory_frac": compulsory_bytes_sddmm(config["nvec"], A.M, -(-A.M // V), V, d, uniq_rows)
                                      / t_sddmm / 1e9 / HBM_PEAK_GBS}
                  if has_sddmm else None),
        "softmax": ({"us_avg": float(softmax_ms.mean()) * 1e3, "us_min": float(softmax_ms.min()) * 1e3,
                     "scale": sm_scale} if args.softmax else None),
        "softmax_backward": softmax_bwd,
        "ms_per_step_graph_replay": graph_ms,
        "attention_fused": fused,
        "sddmm_spmm_fused": fused_chain,
        "spmm_packed": packed,
        "convert": {"ms_median": float(np.median(conv_ms)), "ms_min": float(np.min(conv_ms)), "includes": "host sync",
                    "csr_transpose_ms_median": float(np.median(tr_ms)), "csr_transpose_ms_min": float(np.min(tr_ms))},
        "roofline": roofline,
        "power_law": power_law,
        "cpu_baseline": cpu,
        "parity_scaled_err_sampled_rows": parity,
    }
    print(json.dumps(out))


def time_packed(torch, fs, fmt, Bd, C, work, vals, n):
    t0 = time.perf_counter()
    pbuf = fs.fs_pack_values(fmt, vals=vals)
    torch.cuda.synchronize()
    pack_ms = (time.perf_counter() - t0) * 1e3
    res = {}
    for name, call in (("plain", lambda: fs.fs_spmm(fmt, Bd, vals=vals, out=C, work=work)),
                       ("packed", lambda: fs.fs_spmm_packed(fmt, pbuf, Bd, out=C, work=work))):
        pe = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n)]
        for _ in range(3):
            call()
        for a, b in pe:
            a.record()
            call()
            b.record()
        torch.cuda.synchronize()
        res[name] = np.array([a.elapsed_time(b) for a, b in pe])
    return {"us_avg": float(res["packed"].mean()) * 1e3, "us_min": float(res["packed"].min()) * 1e3,
            "plain_call_us_avg": float(res["plain"].mean()) * 1e3, "plain_call_us_min": float(res["plain"].min()) * 1e3,
            "pack_ms_first_call": pack_ms, "packed_bytes": int(pbuf.numel()),
            "vals_blk_bytes": int(fmt.V * fmt.nvec * 2), "V": int(fmt.V)}


def measure_power_law(torch, fs, name, A, B, raw, scale, with_cpu):
    """SpMM main-kernel time and the three byte figures for another workload, in this same process."""
    from workloads import bits_to_f64
    from workloads.device import from_dev_bits, to_dev, upload_csr
    N = B.shape[1]
    rp, ci, va = upload_csr(A)
    Bd = to_dev(B.bits, B.dtype)
    fmt = fs.fs_convert(rp, ci, va, A.M, A.K)
    V = fmt.V
    C = torch.empty((A.M, N), dtype=Bd.dtype, device="cuda")
    work = torch.empty(max(fs.fs_spmm_workspace_bytes(fmt, N), 16), dtype=torch.uint8, device="cuda")
    n = 200 if A.nnz < 4_000_000 else 20
    k_ms, call_ms = time_spmm_kernel(torch, fs, fmt, Bd, C, work, n=n)
    t = float(k_ms.mean()) * 1e-3
    uniq = int(np.unique(A.colidx).shape[0])
    packed = bool(fmt.packed)  # large matrices: the conversion packed the values and fs_spmm reads those
    q_min, q_hier = spmm_byte_model(fmt, A, N, uniq, packed)
    figs = byte_figures(q_min, q_hier, fabric_bytes(raw, scale, A.dtype, V, packed=packed), t)
    parity = None
    if with_cpu:
        import oracle
        rows = np.unique(np.linspace(0, A.M - 1, 256).astype(np.int64))
        ref, S = oracle.spmm(A.M, A.K, A.rowptr, A.colidx, A.vals, B.bits, A.dtype, rows=rows)
        got = bits_to_f64(from_dev_bits(C[torch.from_numpy(rows).cuda()]), A.dtype)
        floor = 2.0 ** -25 if A.dtype == "f16" else 2.0 ** -134
        parity = float((np.maximum(np.abs(got - ref) - floor, 0) / np.maximum(S, 1e-300)).max())
    out = dict(N=N, dtype=A.dtype, V=int(V), nnz=A.nnz, packed_values=packed, kernel_us_avg=t * 1e6,
               kernel_us_min=float(k_ms.min()) * 1e3, whole_call_us_avg=float(call_ms.mean()) * 1e3,
               gflops=2.0 * A.nnz * N / t / 1e9, parity_scaled_err_sampled_rows=parity, **figs)
    if packed:  # the same call on the unpacked value array, for comparison
        k2, c2 = time_spmm_kernel(torch, fs, fmt, Bd, C, work, vals=fmt.vals_blk_t(), n=n)
        out["unpacked_values_kernel_us_avg"] = float(k2.mean()) * 1e3
        out["unpacked_values_whole_call_us_avg"] = float(c2.mean()) * 1e3
    del rp, ci, va, Bd, C, work
    torch.cuda.empty_cache()
    return out


def write_traffic_profiles(raw, scale, stamp, power_law, args):
    """profiles/fabric_traffic_<workload>_spmm.{txt,json} from this run's counter readings."""
    cmd = "python3 bench.py --write-profiles" + ("" if args.workload == "cfg2_rmat16" else " --workload " + args.workload)
    for name, p in (power_law or {}).items():
        if not p.get("fabric_bytes"):
            continue
        head, tail = spmm_kernel_pattern(p["dtype"], p["V"], packed=p.get("packed_values", False))
        kern = [k[k.index("k_spmm<"):k.index(">(") + 1] for k in raw["FETCH_SIZE"] if head in k and (tail + "(") in k]
        lines = ["L2<->fabric traffic of the SpMM main kernel per launch, workload %s (one MI355X)" % name,
                 "command: %s" % cmd,
                 "  (the bench starts two children of itself under `rocprofv3 --output-format csv --pmc FETCH_SIZE|WRITE_SIZE",
                 "   --kernel-trace`; each child runs fs_copy_bytes on %d MiB three times, then four fs_spmm launches per workload;" % (COPY_CAL_BYTES >> 20),
                 "   the first dispatch of every kernel is left out of the mean)",
                 "calibration: one counter unit = %.2f bytes (FETCH_SIZE), %.2f bytes (WRITE_SIZE), from the copy of known size" % (
                     scale["FETCH_SIZE"], scale["WRITE_SIZE"]),
                 "these counters sit between L2 and the fabric: they include what the Infinity Cache serves, so they bound HBM traffic from above",
                 "", "kernel: %s" % (kern[0] if kern else "?"),
                 "  fabric bytes %.2f MB   compulsory bytes %.2f MB (x%.2f)   hierarchy (method) bytes %.2f MB" % (
                     p["fabric_bytes"] / 1e6, p["compulsory_bytes"] / 1e6, p["fabric_over_compulsory"], p["hierarchy_bytes"] / 1e6),
                 "  kernel time by HIP events in the same run: %.1f us avg (%.1f min)" % (p["kernel_us_avg"], p["kernel_us_min"]),
                 "  fabric %.0f GB/s (%.3f of 8 TB/s)   compulsory %.0f GB/s (roofline frac %.3f)   hierarchy %.0f GB/s   %.0f GFLOP/s" % (
                     p["fabric_GBs"], p["fabric_frac_of_8TBs"], p["compulsory_GBs"], p["compulsory_frac"], p["hierarchy_GBs"], p["gflops"]),
                 "source stamp (sha256 of csrc/ and include/, first 16 hex digits): %s" % stamp]
        os.makedirs(args.profiles_dir, exist_ok=True)
        base = os.path.join(args.profiles_dir, "fabric_traffic_%s_spmm" % name)
        open(base + ".txt", "w").write("\n".join(lines) + "\n")
        json.dump({"kernel": kern[0] if kern else "", "fabric_bytes_per_launch": p["fabric_bytes"], "source_stamp": stamp,
                   "bytes_per_unit": scale, "command": cmd}, open(base + ".json", "w"), indent=1)


def short_kernel_name(name):
    n = name.replace("(anonymous namespace)::", "")
    if n.startswith("void "):
        n = n[5:]
    return n.split("(")[0]


def summarize_profile(root):
    """Text summary of rocprofv3 --output-format csv output: per-kernel durations from the kernel trace (or the
    stats file) and, where counters were collected, their mean per dispatch and kernel."""
    stats, trace, counters = [], {}, {}
    for d, _, files in os.walk(root):
        for f in sorted(files):
            path = os.path.join(d, f)
            if f.endswith("kernel_stats.csv"):
                stats += list(csv.DictReader(open(path)))
            elif f.endswith("kernel_trace.csv"):
                for r in csv.DictReader(open(path)):
                    trace.setdefault(short_kernel_name(r["Kernel_Name"]), []).append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
            elif f.endswith("counter_collection.csv"):
                seen = set()
                for r in csv.DictReader(open(path)):
                    k = short_kernel_name(r["Kernel_Name"])
                    key = (r["Dispatch_Id"], r["Counter_Name"])
                    if key in seen:
                        continue
                    seen.add(key)
                    counters.setdefault(k, {}).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    if trace:
        print("kernel                                              calls    avg us     min us     max us   total ms")
        tot = sum(sum(v) for v in trace.values())
        for k, v in sorted(trace.items(), key=lambda kv: -sum(kv[1]))[:24]:
            print("%-50s %6d %9.1f  %9.1f  %9.1f  %9.2f  %5.1f%%" % (k[:50], len(v), np.mean(v) / 1e3, min(v) / 1e3, max(v) / 1e3,
                                                                     sum(v) / 1e6, 100.0 * sum(v) / max(tot, 1)))
    elif stats:
        for r in stats[:24]:
            print("%-50s calls %6s avg %10.1f us" % (short_kernel_name(r["Name"])[:50], r["Calls"], float(r["AverageNs"]) / 1e3))
    if counters:
        print()
        print("mean counter values per dispatch (first dispatch of each kernel left out where there are several)")
        for k, cs in sorted(counters.items()):
            if not k.startswith("k_"):
                continue
            print(k)
            for c, v in sorted(cs.items()):
                vv = v[1:] if len(v) > 1 else v
                print("    %-34s %18.1f   (%d dispatches)" % (c, float(np.mean(vv)), len(vv)))


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
