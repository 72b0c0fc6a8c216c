#!/usr/bin/env python3
"""Benchmark of the LightKV compression step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: every stage of the
workload's hierarchical schedule, each stage = window partition -> per-window counts -> scores (FD + xi)
-> selection -> message passing + compaction.  All inputs are resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 3] [--mode graph|eager] [--pass all|...]

Prints ONE JSON line: metric "vision tokens compressed/sec per layer" (tokens entering the compression
stages of one step / time of the step), the roofline of the dominant kernel (message passing +
compaction, HBM bound, quoted with caches flushed in front of every launch), the same kernel as it runs
inside the step and on the batched workload, the two dense contractions (bipartite and full pairwise
feature divergence of the 2880-token window) against the bf16 matrix-core peak, and the CPU oracle
timed on the host cores.

Passes (--pass): "all" (default) runs everything; "step", "cold", "hbm_primary", "similarity", "pairwise"
run the set-up and that measurement alone, so that a kernel trace of the command holds the launches of
one regime (the summaries under profiles/ are made that way).  Two maintenance modes need no workload:
--calibrate-counters (plain device copies of known size, to scale FETCH_SIZE / WRITE_SIZE) and
--summarize DB [COMMAND] (a rocprofv3 kernel-trace database as the short text kept under profiles/).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published
PASSES = ("all", "step", "cold", "hbm_primary", "similarity", "pairwise", "ceilings")


def _parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="3", help="1..5, halving, global (default 3: the N=2880 LLaVA-NeXT-shaped layer)")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"])
    ap.add_argument("--pass", dest="only", default="all", choices=PASSES,
                    help="run one measurement only (after the set-up it needs); default: all of them")
    ap.add_argument("--match", default="best_per_a", choices=["best_per_a", "edge_topk", "full_pairwise"],
                    help="edge_topk: Step 2 read literally, floor(rho v / 2) lowest-FD edges per window; full_pairwise: "
                         "the appendix ablation, at most floor(rho v) tokens leave a window (token counts depend on the "
                         "data in both: eager, small read-backs per stage)")
    ap.add_argument("--rho", type=float, default=None, help="edge_topk / full_pairwise: the ratio rho (defaults 0.36 / 0.18: "
                    "about the tokens per stage the default schedule of config 3 removes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-repeats", type=int, default=4, help="oracle steps timed per cpu_baseline leg")
    ap.add_argument("--calibrate-counters", action="store_true")
    ap.add_argument("--summarize", nargs="+", metavar=("DB", "COMMAND"))
    return ap.parse_args()


def _elem_bytes(dtype):
    return 2 if dtype == "bf16" else 4


def rows_bytes(wl, n_in, n_out):
    """Algorithmic HBM bytes of message passing + compaction for one stage: X, K, V rows read once
    (batch * n_in rows) and written once (batch * n_out rows)."""
    return 3 * _elem_bytes(wl.dtype) * wl.d * wl.batch * (n_in + n_out)


def measured_traffic(workload_name):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE, scaled by a copy-kernel calibration); None where no such summary exists for the workload.  The
    figure is read from the file: this run does not measure it."""
    path = os.path.join(ROOT, "profiles", "rows_kernel_hbm_traffic_%s.txt" % {"llava_next": "llava_next_n2880"}.get(workload_name, workload_name))
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return int(line.split("=")[1]), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def summarize(db_path: str, command: str) -> str:
    """rocprofv3 --kernel-trace database -> per-kernel text summary."""
    import sqlite3
    con = sqlite3.connect(db_path)
    rows = list(con.execute(
        "select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
        "from kernels group by name order by 6 desc"))
    total = sum(r[5] for r in rows) or 1
    lines = ["command: " + command, "source : rocprofv3 --kernel-trace (rocpd database), durations in microseconds", "",
             "%-78s %7s %10s %10s %10s %7s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "share")]
    for name, n, avg, mn, mx, tot in rows:
        lines.append("%-78s %7d %10.2f %10.2f %10.2f %6.1f%%" % (name[:78], n, avg / 1e3, mn / 1e3, mx / 1e3, 100.0 * tot / total))
    return "\n".join(lines) + "\n"


def calibrate_counters():
    """Plain device-to-device copies of known size (64 MiB and 512 MiB, four each).  Run under
    `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`: what those counters report for a kernel whose HBM traffic is
    known (reads N bytes, writes N bytes) scales the counters of the LightKV kernels."""
    import torch
    for mib in (64, 512):
        a = torch.empty(mib * 1024 * 1024 // 2, dtype=torch.bfloat16, device="cuda").normal_()
        b = torch.empty_like(a)
        for _ in range(4):
            b.copy_(a)
        torch.cuda.synchronize()
    print(json.dumps({"calibration": "copies of 64 MiB and 512 MiB, four each"}))


def _probe_lib():
    import ctypes as C
    lib = C.CDLL(os.path.join(ROOT, "paper_2605_00789_amd", "liblightkv_probe.so"))
    lib.lightkv_probe_operand_delivery.restype = C.c_int
    lib.lightkv_probe_operand_delivery.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                                   C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_double), C.c_void_p]
    lib.lightkv_probe_mfma.restype = C.c_int
    lib.lightkv_probe_mfma.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_float), C.c_void_p]
    return lib


class _Timer:
    """HIP events on the launch stream; the interval of an empty event pair is measured the same way and removed.  What
    is left of an interval around one kernel is its dispatch latency plus its execution: an upper bound of the duration a
    kernel trace reports for it."""

    def __init__(self, stream):
        import torch
        self.torch, self.stream = torch, stream
        nulls = []
        for _ in range(20):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda._sleep(200_000)
            a.record(stream); b.record(stream)
            stream.synchronize()
            nulls.append(a.elapsed_time(b) * 1e3)
        self.null_us = sorted(nulls)[len(nulls) // 2]

    def pair(self):
        return self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)

    def us(self, a, b):
        return max(a.elapsed_time(b) * 1e3 - self.null_us, 0.0)


def _pipeline(wl, dev):
    import torch
    from paper_2605_00789_amd import CompressionPipeline, to_device as to_dev
    pipe = CompressionPipeline(dtype=wl.dtype, batch=wl.batch, d=wl.d, heads=wl.heads, head_dim=wl.head_dim,
                               tiles=wl.tiles, grid_h=wl.grid_h, grid_w=wl.grid_w, cu_txt=wl.cu_txt,
                               windows_per_axis=wl.windows_per_axis, targets=wl.targets, fused=True)
    X, K, V, Q = (to_dev(t, wl.dtype) for t in (wl.X, wl.K, wl.V, wl.Q))
    pos = torch.from_numpy(wl.pos).to(dev)
    return pipe, (X, K, V, Q, pos)


def rows_cold_pass(wl, pipe, tensors, stream, timer, n_inst):
    """The merge kernel of every stage with L2 and Infinity Cache holding none of its inputs: a 1 GiB buffer is READ in
    front of every launch (clean lines: a flush by writing would leave the caches full of dirty lines whose write-back
    then competes with the kernel).  Stage inputs and index structures are those a run of the schedule left behind.
    Returns microseconds per stage (mean over n_inst launches); the single launches are kept in `rows_cold_pass.samples`
    (a list per stage) for the spread that goes into the line."""
    import torch
    from paper_2605_00789_amd import binding as B
    X, K, V, Q, pos = tensors
    dev = X.device
    flush = torch.zeros(1 << 27, dtype=torch.int64, device=dev)
    sink = torch.zeros((), dtype=torch.int64, device=dev)
    per_stage = [0.0] * wl.stages
    samples = [[] for _ in range(wl.stages)]
    with torch.cuda.stream(stream):
        pipe.run(X, K, V, Q, pos)
        stream.synchronize()
        for _ in range(n_inst):
            Xi, Ki, Vi, pi = X, K, V, pos
            evs = []
            for s in range(wl.stages):
                st = pipe.stages[s]
                torch.sum(flush, dim=(0,), out=sink)
                a, b = timer.pair()
                a.record(stream)
                B.lightkv_aggregate_compact(st.problem, st.new_index, st.grp_offsets, st.grp_src, st.xi, Xi, Ki, Vi, pi,
                                            st.X_out, st.K_out, st.V_out, st.pos_out)
                b.record(stream)
                evs.append((a, b))
                Xi, Ki, Vi, pi = st.X_out, st.K_out, st.V_out, st.pos_out
            stream.synchronize()
            for s, (a, b) in enumerate(evs):
                us = timer.us(a, b)
                per_stage[s] += us / n_inst
                samples[s].append(us)
    del flush, sink
    rows_cold_pass.samples = samples
    return per_stage


def _rows_roofline(wl, per_stage_us, n_ins, regime, samples=None):
    rows_b = [rows_bytes(wl, n_ins[s], wl.targets[s]) for s in range(wl.stages)]
    tot_us, tot_b = sum(per_stage_us), sum(rows_b)
    ach = tot_b / (tot_us * 1e-6) / 1e9 if tot_us > 0 else 0.0
    spread = {}
    if samples:   # per stage: 10th percentile, median, 90th percentile of the single launches
        def pct(v, q):
            v = sorted(v)
            return round(v[min(len(v) - 1, int(q * len(v)))], 2)
        spread = {"launch_us_p10_p50_p90_per_stage": [[pct(v, 0.1), pct(v, 0.5), pct(v, 0.9)] for v in samples]}
    return {**_rows_roofline_core(wl, regime, ach, tot_us, per_stage_us, tot_b), **spread}


def _rows_roofline_core(wl, regime, ach, tot_us, per_stage_us, tot_b):
    return {"kernel": "rows_kernel (lightkv_aggregate_compact)", "bound": "hbm", "regime": regime,
            "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
            "launches_per_step": wl.stages, "avg_launch_us": round(tot_us / wl.stages, 2),
            "launch_us_per_stage": [round(u, 2) for u in per_stage_us],
            "algorithmic_bytes_per_launch": int(tot_b / wl.stages), "workload": wl.name}


def similarity_pass(stream, timer, n_inst, full_pairwise):
    """The dense contraction on the 2880-token window of config 3's tensors: the FD half of lightkv_score, bipartite
    (1440 x 1440 x 4096) or full pairwise (2880 x 2880 x 4096), i.e. squared norms + tiled MFMA kernel + key unpacking in
    one call.  The profiles under profiles/ isolate the MFMA kernel."""
    import torch
    from workloads import make_workload
    from paper_2605_00789_amd import binding as B
    from paper_2605_00789_amd import to_device as to_dev
    wl = make_workload("global")
    dev = torch.device("cuda:0")
    n = wl.n_per_seq
    h_cu = wl.cu_vis.astype("int32")
    cu = torch.from_numpy(h_cu).to(dev)
    X = to_dev(wl.X, wl.dtype)
    pos = torch.from_numpy(wl.pos).to(dev)
    wo = torch.empty(2, dtype=torch.int32, device=dev)
    wt = torch.empty(n, dtype=torch.int32, device=dev)
    rem = torch.zeros(1, dtype=torch.int32, device=dev)
    prob = B.Problem(batch=1, d=wl.d, heads=wl.heads, head_dim=wl.head_dim, dtype=wl.dtype, h_cu_vis=h_cu, cu_vis=cu,
                     n_windows=1, max_window_tokens=n, win_offsets=wo, win_tokens=wt, win_remove=rem,
                     match=B.MATCH_FULL_PAIRWISE if full_pairwise else B.MATCH_BEST_PER_A)
    ws = torch.empty(B.lightkv_workspace_size(prob), dtype=torch.uint8, device=dev)
    xi = torch.ones(n, dtype=torch.float32, device=dev)
    best_fd = torch.empty(n, dtype=torch.float32, device=dev)
    best_dst = torch.empty(n, dtype=torch.int32, device=dev)
    us = 0.0
    with torch.cuda.stream(stream):
        B.lightkv_build_windows(1, h_cu, cu, pos, wl.tiles, wl.grid_h, wl.grid_w, 0, wo, wt)
        for _ in range(3):
            B.lightkv_score(prob, X, None, None, xi, best_fd, best_dst, ws, xi_mode=B.XI_GIVEN)
        stream.synchronize()
        for _ in range(n_inst):
            torch.cuda._sleep(1_000_000)
            a, b = timer.pair()
            a.record(stream)
            B.lightkv_score(prob, X, None, None, xi, best_fd, best_dst, ws, xi_mode=B.XI_GIVEN)
            b.record(stream)
            stream.synchronize()
            us += timer.us(a, b) / n_inst
    flops = 2.0 * n * n * wl.d if full_pairwise else 2.0 * ((n + 1) // 2) * (n // 2) * wl.d
    tf = flops / (us * 1e-6) / 1e12
    return {"call": "lightkv_score, FD half, " + ("full pairwise: row_norms + fd_pair + finalize, 2880 x 2880 x 4096"
                                                   if full_pairwise else "bipartite: row_norms + fd_big + finalize, 1440 x 1440 x 4096"),
            "bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "flops_per_call": int(flops), "avg_call_us": round(us, 2),
            "workload": wl.name}


def copy_ceiling(stream, timer, total_mb_list=(107, 342, 824), n_inst=20):
    """A plain device-to-device copy (torch's copy kernel) whose read + write traffic equals that of a launch of the merge
    kernel, timed the same way as the cold pass: 1 GiB read in front of every launch, HIP events around the one kernel.
    What a copy reaches is what "HBM bound" can mean at that size on this chip."""
    import torch
    dev = torch.device("cuda:0")
    flush = torch.zeros(1 << 27, dtype=torch.int64, device=dev)
    sink = torch.zeros((), dtype=torch.int64, device=dev)
    out = []
    with torch.cuda.stream(stream):
        for mb in total_mb_list:
            n = mb * 1000 * 1000 // 2 // 2          # bf16 elements per side: read n, write n
            a = torch.empty(n, dtype=torch.bfloat16, device=dev).normal_()
            b = torch.empty_like(a)
            b.copy_(a)
            stream.synchronize()
            us = 0.0
            for _ in range(n_inst):
                torch.sum(flush, dim=(0,), out=sink)
                e0, e1 = timer.pair()
                e0.record(stream)
                b.copy_(a)
                e1.record(stream)
                stream.synchronize()
                us += timer.us(e0, e1) / n_inst
            gbs = 4.0 * n / (us * 1e-6) / 1e9
            out.append({"traffic_MB": round(4.0 * n / 1e6, 1), "us": round(us, 2), "GBps": round(gbs, 1),
                        "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)})
            del a, b
    del flush, sink
    return out


def _copy_reference(stream, timer, roof, n_inst):
    """The achievable ceiling beside a cold roofline object: a plain device-to-device copy with the kernel's algorithmic
    bytes per launch as its traffic, flushed and timed exactly like the kernel; frac_of_copy = copy time / kernel time."""
    mb = int(round(roof["algorithmic_bytes_per_launch"] / 1e6))
    c = copy_ceiling(stream, timer, total_mb_list=(mb,), n_inst=max(5, min(n_inst, 20)))[0]
    c["kernel_frac_of_copy"] = round(c["us"] / roof["avg_launch_us"], 4)
    return c


def ceilings_pass(stream):
    """What the chip delivers to the dense contractions, measured with the probe library (no method arithmetic): the
    operand loads of the tiled FD kernels alone (every byte comes out of L2: nothing is reused through L1), and bare
    loops of independent 32x32x16 bf16 MFMAs on constant and on random operands (the sustained clocks depend on the
    switching activity of the operands)."""
    import ctypes as C
    import numpy as np
    import torch
    from workloads import make_workload
    from paper_2605_00789_amd import to_device as to_dev
    lib = _probe_lib()
    wl = make_workload("global")
    X = to_dev(wl.X, wl.dtype)
    n, row_bytes = X.shape[0], X.shape[1] * 2
    sp = C.c_void_p(stream.cuda_stream)
    out = {"operand_delivery": [], "mfma_bare_loop": []}
    for name, pairwise, tile, splits, piece in (("bipartite 1440 x 1440, 96 x 96 tiles (fd_big_kernel's loads)", 0, 96, 1, 256),
                                                ("bipartite, 96 x 96 tiles, 128-byte pieces", 0, 96, 1, 128),
                                                ("bipartite, 192 x 192 tiles, hidden axis split 4 ways", 0, 192, 4, 128),
                                                ("full pairwise 2880 x 2880, 192 x 192 tiles (fd_pair_kernel's loads)", 1, 192, 1, 128),
                                                ("full pairwise, 96 x 96 tiles", 1, 96, 1, 256)):
        us, nbytes = C.c_float(0), C.c_double(0)
        rc = lib.lightkv_probe_operand_delivery(C.c_void_p(X.data_ptr()), n, row_bytes, pairwise, tile, splits, piece, 20,
                                                C.byref(us), C.byref(nbytes), sp)
        if rc != 0:
            raise RuntimeError("lightkv_probe_operand_delivery failed: %d" % rc)
        out["operand_delivery"].append({"case": name, "us": round(us.value, 2), "MB_to_CUs": round(nbytes.value / 1e6, 1),
                                        "TBps": round(nbytes.value / (us.value * 1e-6) / 1e12, 2)})
    iters_mfma = 500
    for name, data in (("constant operands (all lanes 1.0)", torch.ones(1024 * 6 * 256 * 8, dtype=torch.bfloat16, device=X.device)),
                       ("random operands (N(0,1) bf16)", torch.randn(1024 * 6 * 256 * 8, device=X.device).to(torch.bfloat16))):
        for wgs in (225, 256, 1024):
            us = C.c_float(0)
            rc = lib.lightkv_probe_mfma(C.c_void_p(data.data_ptr()), wgs, iters_mfma, 5, C.byref(us), sp)
            if rc != 0:
                raise RuntimeError("lightkv_probe_mfma failed: %d" % rc)
            flops = wgs * 4 * 9 * iters_mfma * 32768.0
            out["mfma_bare_loop"].append({"case": name, "workgroups": wgs, "us": round(us.value, 2),
                                          "TFLOPs": round(flops / (us.value * 1e-6) / 1e12, 1),
                                          "frac_of_published_peak": round(flops / (us.value * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 3)})
    return out


def cpu_baseline(run_once, tokens_per_step, repeats, sample):
    """The oracle as it stands on the host cores: all threads the BLAS behind numpy takes, and one thread."""
    out = {}
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:   # noqa: BLE001
        threadpool_limits, cores = None, os.cpu_count() or 1
    t0 = time.perf_counter()
    for _ in range(repeats):
        run_once()
    dt = (time.perf_counter() - t0) / repeats
    out["cpu_baseline"] = {"value": round(tokens_per_step / dt, 1), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                           "sample": "%d %s, numpy fp64, %.2f s each" % (repeats, sample, dt)}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            for _ in range(repeats):
                run_once()
            dt1 = (time.perf_counter() - t0) / repeats
        out["cpu_baseline_1thread"] = {"value": round(tokens_per_step / dt1, 1), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                       "sample": "%d %s, numpy fp64, %.2f s each" % (repeats, sample, dt1)}
    return out


def bench_variant(args):
    """The schedules whose token counts depend on the data (the k lowest edges per window; full pairwise matching):
    eager, host read-backs included in the timed region (they are part of the step: the next stage cannot be sized
    without them)."""
    import numpy as np
    import torch
    from workloads import make_workload
    from paper_2605_00789_amd import EdgeTopKSchedule, to_device as to_dev, max_window_cells
    from paper_2605_00789_amd import binding as B
    cfg = int(args.workload) if args.workload.isdigit() else args.workload
    wl = make_workload(cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    pairwise = args.match == "full_pairwise"
    rho = args.rho if args.rho is not None else (0.18 if pairwise else 0.36)
    ws_axis = list(wl.windows_per_axis)
    sched = EdgeTopKSchedule(dtype=wl.dtype, batch=wl.batch, d=wl.d, heads=wl.heads, head_dim=wl.head_dim, tiles=wl.tiles,
                             grid_h=wl.grid_h, grid_w=wl.grid_w, cu_txt=wl.cu_txt, windows_per_axis=ws_axis,
                             rho=[rho] * len(ws_axis), match=args.match)
    X, K, V, Q = (to_dev(t, wl.dtype) for t in (wl.X, wl.K, wl.V, wl.Q))
    pos = torch.from_numpy(wl.pos).to(dev)
    for _ in range(max(args.warmup, 1)):
        res = sched.run(wl.cu_vis, X, K, V, Q, pos)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = sched.run(wl.cu_vis, X, K, V, Q, pos)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    acc = {}
    n_inst = max(5, min(args.steps, 30))
    for _ in range(n_inst):
        marks = []
        sched.run(wl.cu_vis, X, K, V, Q, pos, marks=marks)
        torch.cuda.synchronize()
        stage = 0
        for (na, ea), (nb, eb) in zip(marks[0::2], marks[1::2]):
            if na == "build_windows":
                stage += 1
            acc.setdefault("stage%d.%s" % (stage, na), []).append(ea.elapsed_time(eb) * 1e3)
    calls_us = {k: round(sorted(v)[len(v) // 2], 2) for k, v in acc.items()}
    n_in = [int(wl.cu_vis[-1])] + [int(r.h_cu_vis_out[-1]) for r in res[:-1]]
    n_out = [int(r.h_cu_vis_out[-1]) for r in res]
    eb_ = _elem_bytes(wl.dtype)
    rows_b = sum(3 * (a + b) * wl.d * eb_ for a, b in zip(n_in, n_out))
    rows_us = sum(v for k, v in calls_us.items() if k.endswith("aggregate_compact"))
    ach = rows_b / (rows_us * 1e-6) / 1e9
    out = {
        "metric": "vision tokens compressed/sec per layer", "value": round(sum(n_in) / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "match": args.match, "rho": rho, "batch": wl.batch, "stages": len(ws_axis),
                   "windows_per_axis": ws_axis, "tokens_in_per_stage": n_in, "tokens_out_per_stage": n_out,
                   "counts_per_stage": [int(r.h_win_edges.sum()) for r in res], "launch": "one library call (lightkv_compress_schedule_ratio): eager, buffers allocated once, counts on the device, one read-back per stage (the batch + 1 sequence offsets); calls_us from the same stages driven call by call"},
        "roofline": {"kernel": "rows_kernel (lightkv_aggregate_compact)", "bound": "hbm", "regime": "in the step",
                     "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                     "traffic": None, "launches_per_step": len(ws_axis), "avg_launch_us": round(rows_us / len(ws_axis), 2),
                     "algorithmic_bytes_per_launch": rows_b // len(ws_axis),
                     "note": "call interval from events around the call (includes launch overhead of an eager call)"},
        "calls_us": calls_us,
    }
    if not args.no_cpu_baseline:
        from oracle import lightkv_oracle as O

        def once():
            Xc, Kc, Vc, posc, cu = wl.X, wl.K, wl.V, wl.pos, wl.cu_vis
            Q64 = O.widen(wl.Q, wl.dtype)
            for s, w in enumerate(ws_axis):
                wo, wt = O.build_windows(posc, cu, wl.tiles, wl.grid_h, wl.grid_w, w)
                args_ = (O.widen(Xc, wl.dtype), O.widen(Kc, wl.dtype), O.widen(Vc, wl.dtype), Q64, posc, cu, wl.cu_txt,
                         wl.heads, wl.head_dim, wo, wt)
                if pairwise:
                    r = O.compress_stage_full_pairwise(*args_, O.removal_counts_ratio(wo, rho))
                else:
                    r = O.compress_stage_edges(*args_, O.edge_counts_ratio(wo, rho))
                Xc, Kc, Vc = (O.round_to_storage(t, wl.dtype) for t in (r.X, r.K, r.V))
                posc, cu = r.pos, r.cu_vis
        out.update(cpu_baseline(once, sum(n_in), max(1, args.cpu_repeats // 2), "full schedules of the same workload"))
    print(json.dumps(out))


def main():
    args = _parse()
    if args.summarize:
        sys.stdout.write(summarize(args.summarize[0], args.summarize[1] if len(args.summarize) > 1 else ""))
        return
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the step has no cross-GPU part); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.calibrate_counters:
        return calibrate_counters()
    if args.match != "best_per_a":
        return bench_variant(args)
    import numpy as np
    from workloads import make_workload
    from paper_2605_00789_amd import binding as B

    cfg = int(args.workload) if args.workload.isdigit() else args.workload
    wl = make_workload(cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    pipe, tensors = _pipeline(wl, dev)
    X, K, V, Q, pos = tensors
    n_ins = [wl.n_per_seq] + list(wl.targets[:-1])
    tokens_per_step = wl.batch * sum(n_ins)
    only = args.only
    want = lambda name: only in ("all", name)   # noqa: E731
    main_workload = cfg == 3                    # the extra objects of the default line belong to the default workload

    stream = torch.cuda.Stream()
    out = {
        "metric": "vision tokens compressed/sec per layer", "value": None, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": None, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "description": wl.notes, "batch": wl.batch, "stages": wl.stages,
                   "tokens_in_per_stage": [wl.batch * n for n in n_ins], "windows_per_axis": wl.windows_per_axis,
                   "launch": args.mode, "pass": only},
    }
    with torch.cuda.stream(stream):
        for _ in range(max(args.warmup, 1)):
            pipe.run(X, K, V, Q, pos)
        stream.synchronize()
        status = [int(st.status.sum().item()) for st in pipe.stages]
        if any(status):
            print("bench.py: a stage's token budget could not be met (status %s)" % status, file=sys.stderr)
            sys.exit(1)
        timer = _Timer(stream)
        out["event_overhead_us"] = round(timer.null_us, 2)
        n_inst = max(5, min(args.steps, 50))

        if want("step"):
            graph = None
            if args.mode == "graph":
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    pipe.run(X, K, V, Q, pos)
                for _ in range(3):
                    graph.replay()
                stream.synchronize()
            # ---- timed region: exactly K steps, synchronised on both sides
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                if graph is not None:
                    graph.replay()
                else:
                    pipe.run(X, K, V, Q, pos)
            torch.cuda.synchronize()
            ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
            out["ms_per_step"] = round(ms_per_step, 5)
            out["value"] = round(tokens_per_step / (ms_per_step * 1e-3), 1)

            # ---- per-call durations with HIP events on the launch stream.  A sleep kernel in front lets the host enqueue
            # the whole step before the GPU starts it, so event intervals hold GPU time only.
            names = ("build_windows", "score", "select", "aggregate_compact")
            acc = {(s, n): 0.0 for s in range(wl.stages) for n in names}
            for _ in range(n_inst):
                evs = []
                torch.cuda._sleep(2_000_000)
                Xi, Ki, Vi, pi = X, K, V, pos
                for s in range(wl.stages):
                    st = pipe.stages[s]
                    p = st.problem
                    e = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
                    e[0].record(stream)
                    B.lightkv_build_windows(pipe.batch, st.h_cu_vis, st.cu_vis, pi, pipe.tiles, pipe.grid_h, pipe.grid_w,
                                            st.w, st.win_offsets, st.win_tokens)
                    B.lightkv_window_counts(pipe.batch, p.c.n_windows, st.win_offsets, B.COUNT_TARGET, st.win_remove,
                                            cu_vis=st.cu_vis, cu_vis_target=st.cu_target, status=st.status)
                    e[1].record(stream)
                    B.lightkv_score(p, Xi, Q, Ki, st.xi, st.best_fd, st.best_dst, pipe.ws)
                    e[2].record(stream)
                    B.lightkv_select(p, st.best_fd, st.best_dst, st.dst, st.new_index, st.grp_offsets, st.grp_src,
                                     st.cu_vis_out, pipe.ws)
                    e[3].record(stream)
                    B.lightkv_aggregate_compact(p, st.new_index, st.grp_offsets, st.grp_src, st.xi, Xi, Ki, Vi, pi,
                                                st.X_out, st.K_out, st.V_out, st.pos_out)
                    e[4].record(stream)
                    evs.append(e)
                    Xi, Ki, Vi, pi = st.X_out, st.K_out, st.V_out, st.pos_out
                stream.synchronize()
                for s, e in enumerate(evs):
                    for k, n in enumerate(names):
                        acc[(s, n)] += timer.us(e[k], e[k + 1]) / n_inst
            out["calls_us"] = {"stage%d.%s" % (s + 1, n): round(acc[(s, n)], 2) for s in range(wl.stages) for n in names}
            # per call: algorithmic bytes and flops over the event interval of the call
            #   score             reads X once (feature divergence) and Q, K once (xi): e d (N + T + N) bytes;
            #                     2 d sum_w |A_w| |B_w| flops for FD (window sizes read back) + 2 d sum_b T_b N_b for xi
            #   aggregate_compact 3 e d (N + n') bytes
            eb_ = _elem_bytes(wl.dtype)
            sum_t = int(wl.cu_txt[-1])
            t_b = np.diff(np.asarray(wl.cu_txt, dtype=np.int64))
            calls_roofline = {}
            for s in range(wl.stages):
                st = pipe.stages[s]
                n_s = wl.batch * n_ins[s]
                v = np.diff(st.win_offsets.cpu().numpy().astype(np.int64))
                fd_flops = 2.0 * wl.d * float((((v + 1) // 2) * (v // 2)).sum())
                xi_flops = 2.0 * wl.d * float((t_b * n_ins[s]).sum())
                sc_bytes = eb_ * wl.d * (2 * n_s + sum_t)
                sc_us, rw_us = acc[(s, "score")], acc[(s, "aggregate_compact")]
                rw_bytes = rows_bytes(wl, n_ins[s], wl.targets[s])
                st_us = sum(acc[(s, n)] for n in names)
                calls_roofline["stage%d" % (s + 1)] = {
                    "tokens_in": n_s,
                    "tokens_per_s_eager": round(n_s / (st_us * 1e-6), 1) if st_us > 0 else None,
                    "score": {"bytes": int(sc_bytes), "GBps": round(sc_bytes / (sc_us * 1e-6) / 1e9, 1) if sc_us > 0 else None,
                              "fd_flops": int(fd_flops), "xi_flops": int(xi_flops),
                              "TFLOPs": round((fd_flops + xi_flops) / (sc_us * 1e-6) / 1e12, 2) if sc_us > 0 else None,
                              "mfma_frac": round((fd_flops + xi_flops) / (sc_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 5) if sc_us > 0 else None},
                    "select": {"us": round(acc[(s, "select")], 2), "share_of_stage": round(acc[(s, "select")] / st_us, 3) if st_us > 0 else None},
                    "aggregate_compact": {"bytes": int(rw_bytes), "GBps": round(rw_bytes / (rw_us * 1e-6) / 1e9, 1) if rw_us > 0 else None,
                                          "hbm_frac": round(rw_bytes / (rw_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if rw_us > 0 else None}}
            out["calls_roofline"] = calls_roofline
            warm = _rows_roofline(wl, [acc[(s, "aggregate_compact")] for s in range(wl.stages)], n_ins,
                                  "in the step (inputs just read by the score kernels: cache resident where they fit)")
            out["roofline_warm"] = warm

    # ---- the dominant kernel with caches flushed in front of every launch: the regime the fractions are quoted from
    if want("cold"):
        cold_us = rows_cold_pass(wl, pipe, tensors, stream, timer, n_inst)
        cold = _rows_roofline(wl, cold_us, n_ins, "cold: 1 GiB read in front of every launch", samples=rows_cold_pass.samples)
        traffic, src = measured_traffic(wl.name)
        cold["traffic"] = traffic
        cold["traffic_source"] = ("committed profile %s (not measured by this run)" % src) if src else None
        cold["copy_reference"] = _copy_reference(stream, timer, cold, n_inst)
        out["roofline"] = cold
    elif "roofline_warm" in out:
        out["roofline"] = dict(out["roofline_warm"], traffic=None)

    # ---- the same kernel on the batched workload (does not fit the caches: the primary HBM datapoint)
    if main_workload and want("hbm_primary"):
        wl5 = make_workload(5)
        pipe5, tensors5 = _pipeline(wl5, dev)
        n_ins5 = [wl5.n_per_seq] + list(wl5.targets[:-1])
        cold5_us = rows_cold_pass(wl5, pipe5, tensors5, stream, timer, max(5, n_inst // 2))
        out["roofline_hbm_primary"] = _rows_roofline(wl5, cold5_us, n_ins5, "cold: 1 GiB read in front of every launch",
                                                     samples=rows_cold_pass.samples)
        out["roofline_hbm_primary"]["copy_reference"] = _copy_reference(stream, timer, out["roofline_hbm_primary"], n_inst)
        del pipe5, tensors5, wl5

    # ---- the dense contractions of the 2880-token window against the matrix-core peak
    if (main_workload or cfg == "global") and want("similarity"):
        out["roofline_similarity"] = similarity_pass(stream, timer, n_inst, full_pairwise=False)
    if (main_workload or cfg == "global") and want("pairwise"):
        out["roofline_similarity_full_pairwise"] = similarity_pass(stream, timer, n_inst, full_pairwise=True)

    if only == "ceilings":
        with torch.cuda.stream(stream):
            out["ceilings"] = ceilings_pass(stream)
        out["ceilings"]["plain_copy_cold"] = copy_ceiling(stream, timer)

    if not args.no_cpu_baseline and only == "all":
        from oracle import lightkv_oracle as O
        out.update(cpu_baseline(lambda: O.compress_schedule(wl), tokens_per_step, args.cpu_repeats,
                                "full steps of the same workload (all %d stages)" % wl.stages))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
