#!/usr/bin/env python3
"""Benchmark of the LightKV compression step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: every stage of the
workload's hierarchical schedule, each stage = window partition -> scores (FD + xi) -> selection ->
message passing + compaction.  All inputs are resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 3] [--mode graph|eager]

Prints ONE JSON line: metric "vision tokens compressed/sec per layer" (tokens entering the compression
stages of one step / time of the step), the roofline of the dominant kernel and the CPU oracle timed
on the host cores.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def _parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="3", help="1..5, halving, global (default 3: the N=2880 LLaVA-NeXT-shaped layer)")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"])
    ap.add_argument("--match", default="best_per_a", choices=["best_per_a", "edge_topk"],
                    help="edge_topk: Step 2 read literally, floor(rho v / 2) lowest-FD edges per window (token counts "
                         "depend on the data: eager, two small read-backs per stage)")
    ap.add_argument("--rho", type=float, default=0.36, help="edge_topk: ratio rho of Step 2 (0.36: as many edges per "
                    "window as the default schedule of config 3 removes tokens)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-repeats", type=int, default=20, help="oracle steps timed for cpu_baseline (about 10 s)")
    ap.add_argument("--cold", action="store_true",
                    help="also time the dominant kernel with L2 and Infinity Cache flushed before every launch "
                         "(extra object roofline_cold; the headline figures are unchanged).  Not part of the default "
                         "run, so that a kernel trace of the default command holds the launches of the step only")
    ap.add_argument("--no-cold", dest="cold", action="store_false", help="(the default)")
    return ap.parse_args()


def _elem_bytes(dtype):
    return 2 if dtype == "bf16" else 4


def rows_bytes(wl, n_in, n_out):
    """Algorithmic HBM bytes of message passing + compaction for one stage: X, K, V rows read once
    (batch * n_in rows) and written once (batch * n_out rows)."""
    return 3 * _elem_bytes(wl.dtype) * wl.d * wl.batch * (n_in + n_out)


def measured_traffic(workload_name):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE, scaled by a copy-kernel calibration); None where no such summary exists for the workload."""
    path = os.path.join(ROOT, "profiles", "rows_kernel_hbm_traffic_%s.txt" % {"llava_next": "llava_next_n2880"}.get(workload_name, workload_name))
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return int(line.split("=")[1])
    except OSError:
        pass
    return None


def bench_edge_topk(args):
    """The schedule with the k lowest edges per window: stages whose windows fit the variant's limit, eager, host
    read-backs included in the timed region (they are part of the step: the next stage cannot be sized without them)."""
    import numpy as np
    import torch
    from workloads import make_workload
    from paper_2605_00789_amd import EdgeTopKSchedule, to_device as to_dev, max_window_cells
    from paper_2605_00789_amd import binding as B
    cfg = int(args.workload) if args.workload.isdigit() else args.workload
    wl = make_workload(cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ws_axis = [w for w in wl.windows_per_axis
               if w > 0 and max_window_cells(wl.tiles, wl.grid_h, wl.grid_w, w) <= B.EDGE_MAX_WINDOW_TOKENS]
    sched = EdgeTopKSchedule(dtype=wl.dtype, batch=wl.batch, d=wl.d, heads=wl.heads, head_dim=wl.head_dim, tiles=wl.tiles,
                             grid_h=wl.grid_h, grid_w=wl.grid_w, cu_txt=wl.cu_txt, windows_per_axis=ws_axis,
                             rho=[args.rho] * len(ws_axis))
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
    # per-call GPU time from events around the calls (a pass of its own)
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
        "config": {"workload": wl.name, "match": "edge_topk", "rho": args.rho, "batch": wl.batch, "stages": len(ws_axis),
                   "windows_per_axis": ws_axis, "tokens_in_per_stage": n_in, "tokens_out_per_stage": n_out,
                   "edges_per_stage": [int(r.h_win_edges.sum()) for r in res], "launch": "eager + 2 read-backs per stage"},
        "roofline": {"kernel": "rows_kernel (lightkv_aggregate_compact)", "bound": "hbm", "achieved": round(ach, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None,
                     "launches_per_step": len(ws_axis), "avg_launch_us": round(rows_us / len(ws_axis), 2),
                     "algorithmic_bytes_per_launch": rows_b // len(ws_axis),
                     "note": "call interval from events around the call (includes launch overhead of an eager call)"},
        "calls_us": calls_us,
    }
    if not args.no_cpu_baseline:
        from oracle import lightkv_oracle as O
        t0 = time.perf_counter()
        reps = max(1, args.cpu_repeats // 4)
        for _ in range(reps):
            Xc, Kc, Vc, posc, cu = wl.X, wl.K, wl.V, wl.pos, wl.cu_vis
            Q64 = O.widen(wl.Q, wl.dtype)
            for s, w in enumerate(ws_axis):
                wo, wt = O.build_windows(posc, cu, wl.tiles, wl.grid_h, wl.grid_w, w)
                v = np.diff(wo)
                k = np.minimum(np.floor(args.rho * v / 2.0 + 1e-9).astype(np.int64), ((v + 1) // 2) * (v // 2))
                r = O.compress_stage_edges(O.widen(Xc, wl.dtype), O.widen(Kc, wl.dtype), O.widen(Vc, wl.dtype), Q64, posc, cu,
                                           wl.cu_txt, wl.heads, wl.head_dim, wo, wt, k)
                Xc, Kc, Vc = (O.round_to_storage(t, wl.dtype) for t in (r.X, r.K, r.V))
                posc, cu = r.pos, r.cu_vis
        dt = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": round(sum(n_in) / dt, 1), "unit": "tokens/s", "cores": os.cpu_count() or 1,
                               "kind": "oracle", "sample": "%d full schedules of the same workload, numpy fp64, %.2f s each" % (reps, dt)}
    print(json.dumps(out))


def main():
    args = _parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the step has no cross-GPU part); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if args.match == "edge_topk":
        import torch
        if not torch.cuda.is_available():
            print("bench.py: no GPU visible", file=sys.stderr)
            sys.exit(1)
        return bench_edge_topk(args)
    import numpy as np
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from workloads import make_workload
    from paper_2605_00789_amd import CompressionPipeline, to_device as to_dev

    cfg = int(args.workload) if args.workload.isdigit() else args.workload
    wl = make_workload(cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    pipe = CompressionPipeline(dtype=wl.dtype, batch=wl.batch, d=wl.d, heads=wl.heads, head_dim=wl.head_dim,
                               tiles=wl.tiles, grid_h=wl.grid_h, grid_w=wl.grid_w, cu_txt=wl.cu_txt,
                               windows_per_axis=wl.windows_per_axis, targets=wl.targets, fused=True)
    X, K, V, Q = (to_dev(t, wl.dtype) for t in (wl.X, wl.K, wl.V, wl.Q))
    pos = torch.from_numpy(wl.pos).to(dev)
    n_ins = [wl.n_per_seq] + list(wl.targets[:-1])
    tokens_per_step = wl.batch * sum(n_ins)

    stream = torch.cuda.Stream()
    graph = None
    with torch.cuda.stream(stream):
        for _ in range(max(args.warmup, 1)):
            pipe.run(X, K, V, Q, pos)
        stream.synchronize()
        if args.mode == "graph":
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                pipe.run(X, K, V, Q, pos)
            for _ in range(3):
                graph.replay()
            stream.synchronize()

        def step():
            if graph is not None:
                graph.replay()
            else:
                pipe.run(X, K, V, Q, pos)

        # ---- timed region: exactly K steps, synchronised on both sides
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / args.steps

        # ---- per-call durations with HIP events on the launch stream.  A sleep kernel in front lets the
        # host enqueue the whole step before the GPU starts it, so event intervals hold GPU time only.
        # interval of an empty event pair on this stream (event bookkeeping), removed from every call interval
        nulls = []
        for _ in range(20):
            a, b2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda._sleep(200_000)
            a.record(stream); b2.record(stream)
            stream.synchronize()
            nulls.append(a.elapsed_time(b2) * 1e3)
        null_us = sorted(nulls)[len(nulls) // 2]
        names = ("build_windows", "score", "select", "aggregate_compact")
        n_inst = max(5, min(args.steps, 50))
        acc = {(s, n): 0.0 for s in range(wl.stages) for n in names}
        from paper_2605_00789_amd import binding as B
        for it in range(n_inst):
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
                    acc[(s, n)] += max(e[k].elapsed_time(e[k + 1]) * 1e3 - null_us, 0.0) / n_inst   # microseconds
    calls_us = {"stage%d.%s" % (s + 1, n): round(acc[(s, n)], 2) for s in range(wl.stages) for n in names}

    cold_us = None
    if args.cold:
        # every launch starts from caches that hold none of its inputs: a 1 GiB buffer is READ in front of it (clean
        # lines: a flush by writing would leave the caches full of dirty lines whose write-back then competes with the
        # kernel).  Stage inputs and index structures are the ones the eager pass above left behind.
        flush = torch.zeros(1 << 27, dtype=torch.int64, device=dev)
        sink = torch.zeros((), dtype=torch.int64, device=dev)
        cold_us = 0.0
        with torch.cuda.stream(stream):
            for it in range(n_inst):
                Xi, Ki, Vi, pi = X, K, V, pos
                evs = []
                for s in range(wl.stages):
                    st = pipe.stages[s]
                    torch.sum(flush, dim=(0,), out=sink)
                    a, b2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record(stream)
                    B.lightkv_aggregate_compact(st.problem, st.new_index, st.grp_offsets, st.grp_src, st.xi, Xi, Ki, Vi, pi,
                                                st.X_out, st.K_out, st.V_out, st.pos_out)
                    b2.record(stream)
                    evs.append((a, b2))
                    Xi, Ki, Vi, pi = st.X_out, st.K_out, st.V_out, st.pos_out
                stream.synchronize()
                cold_us += sum(max(a.elapsed_time(b2) * 1e3 - null_us, 0.0) for a, b2 in evs) / n_inst
        del flush, sink

    # ---- per call: algorithmic bytes and flops over the event interval of the call (eager pass above)
    #   score             reads X once (feature divergence) and Q, K once (xi): e d (N + T + N) bytes;
    #                     2 d sum_w |A_w| |B_w| flops for FD (window sizes read back from the device) + 2 d sum_b T_b N_b for xi
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
        sc_us = acc[(s, "score")]
        rw_bytes = rows_bytes(wl, n_ins[s], wl.targets[s])
        rw_us = acc[(s, "aggregate_compact")]
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

    # ---- roofline of the dominant kernel: message passing + compaction (one kernel per stage, HBM bound)
    rows_us = sum(acc[(s, "aggregate_compact")] for s in range(wl.stages))
    rows_b = sum(rows_bytes(wl, n_ins[s], wl.targets[s]) for s in range(wl.stages))
    achieved = rows_b / (rows_us * 1e-6) / 1e9 if rows_us > 0 else 0.0
    roofline = {"kernel": "rows_kernel (lightkv_aggregate_compact)", "bound": "hbm",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(wl.name),
                "launches_per_step": wl.stages,
                "avg_launch_us": round(rows_us / wl.stages, 2),
                "algorithmic_bytes_per_launch": int(rows_b / wl.stages)}

    # the dense-contraction case: FD half of lightkv_score on single-window stages (row norms + tiled MFMA kernel + key
    # unpacking in one call; the profile under profiles/ isolates the MFMA kernel)
    roofline_fd = None
    if all(w == 0 for w in wl.windows_per_axis) and wl.dtype == "bf16":
        fd_us = 0.0
        with torch.cuda.stream(stream):
            for it in range(n_inst):
                torch.cuda._sleep(2_000_000)
                st = pipe.stages[0]
                a, b2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                B.lightkv_score(st.problem, X, None, None, st.xi, st.best_fd, st.best_dst, pipe.ws, xi_mode=B.XI_GIVEN)
                b2.record(stream)
                stream.synchronize()
                fd_us += max(a.elapsed_time(b2) * 1e3 - null_us, 0.0) / n_inst
        nA, nB = (wl.n_per_seq + 1) // 2, wl.n_per_seq // 2
        flops = 2.0 * wl.batch * nA * nB * wl.d
        tf = flops / (fd_us * 1e-6) / 1e12
        roofline_fd = {"call": "lightkv_score, FD half (row_norms + fd_big + finalize)", "bound": "mfma",
                       "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "flops_per_call": int(flops),
                       "avg_call_us": round(fd_us, 2)}

    roofline_cold = None
    if cold_us:
        ach = rows_b / (cold_us * 1e-6) / 1e9
        roofline_cold = {"achieved": round(ach, 1), "frac": round(ach / HBM_PEAK_GBS, 4), "unit": "GB/s",
                         "avg_launch_us": round(cold_us / wl.stages, 2)}
    value = tokens_per_step / (ms_per_step * 1e-3)
    out = {
        "metric": "vision tokens compressed/sec per layer",
        "value": round(value, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": wl.name, "description": wl.notes, "batch": wl.batch, "stages": wl.stages,
                   "tokens_in_per_stage": [wl.batch * n for n in n_ins], "windows_per_axis": wl.windows_per_axis,
                   "launch": args.mode},
        "roofline": roofline,
        "calls_us": calls_us,
        "calls_roofline": calls_roofline,
        "event_overhead_us": round(null_us, 2),
    }
    if roofline_cold:
        out["roofline_cold"] = roofline_cold
    if roofline_fd:
        out["roofline_similarity"] = roofline_fd

    if not args.no_cpu_baseline:
        from oracle import lightkv_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        t0 = time.perf_counter()
        for _ in range(args.cpu_repeats):
            O.compress_schedule(wl)
        dt = (time.perf_counter() - t0) / args.cpu_repeats
        out["cpu_baseline"] = {"value": round(tokens_per_step / dt, 1), "unit": "tokens/s", "cores": int(cores),
                               "kind": "oracle",
                               "sample": "%d full steps of the same workload (all %d stages), numpy fp64, %.2f s each"
                                         % (args.cpu_repeats, wl.stages, dt)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
