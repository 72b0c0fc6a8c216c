"""Buffer ownership and call order for the hierarchical schedule (paper Sec. 3.2.2): every stage calls
lightkv_build_windows -> lightkv_score -> lightkv_select -> lightkv_aggregate_compact (or the separate
lightkv_aggregate + lightkv_compact) on one stream, without host synchronisation.  All device buffers are
allocated once in the constructor; `run` only enqueues kernels."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from .schedule import max_window_cells, windows_per_sequence


def to_device(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """Storage array of a tensor (bf16 carried as uint16 bit patterns, or float32) -> device tensor of that dtype."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def from_device(t: torch.Tensor, dtype: str) -> np.ndarray:
    """Device tensor -> storage array (uint16 bit patterns for bf16)."""
    t = t.detach().cpu().contiguous()
    if dtype == "bf16":
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


@dataclass
class StageBuffers:
    n_in: int
    n_out: int
    w: int
    problem: B.Problem
    h_cu_vis: np.ndarray
    cu_vis: torch.Tensor
    win_offsets: torch.Tensor
    win_tokens: torch.Tensor
    win_remove: torch.Tensor       # written on the device by lightkv_window_counts (from the stage's token budget)
    cu_target: torch.Tensor        # sequence offsets the stage must leave
    status: torch.Tensor           # [batch]: 1 where the budget of a sequence could not be met
    xi: torch.Tensor
    best_fd: torch.Tensor
    best_dst: torch.Tensor
    dst: torch.Tensor
    new_index: torch.Tensor
    grp_offsets: torch.Tensor
    grp_src: torch.Tensor
    cu_vis_out: torch.Tensor
    X_out: torch.Tensor
    K_out: torch.Tensor
    V_out: torch.Tensor
    pos_out: torch.Tensor
    x_sq_out: torch.Tensor     # |x|^2 of the rows of X_out: the next stage's feature divergence takes it as given


class CompressionPipeline:
    def __init__(self, *, dtype: str, batch: int, d: int, heads: int, head_dim: int, tiles: int, grid_h: int,
                 grid_w: int, cu_txt: np.ndarray, windows_per_axis: Sequence[int], targets: Sequence[int],
                 device="cuda:0", fused: bool = True, metric: str = "cosine", direction: str = "a_to_b"):
        self.dtype, self.batch, self.d, self.heads, self.head_dim = dtype, batch, d, heads, head_dim
        self.direction = direction   # "b_to_a": the reverse direction (LIGHTKV_DIRECTION_B_TO_A)
        self._dir = {"a_to_b": B.DIRECTION_A_TO_B, "b_to_a": B.DIRECTION_B_TO_A}[direction]
        self.tiles, self.grid_h, self.grid_w = tiles, grid_h, grid_w
        self.device = torch.device(device)
        self.fused = fused
        self.metric = metric
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.h_cu_txt = np.ascontiguousarray(cu_txt, dtype=np.int32)
        self.cu_txt = torch.from_numpy(self.h_cu_txt).to(self.device)
        dev = self.device
        i32 = dict(dtype=torch.int32, device=dev)
        n_in = tiles * grid_h * grid_w
        self.stages: List[StageBuffers] = []
        ws_bytes = 0
        for w, n_out in zip(windows_per_axis, targets):
            sum_in, sum_out = batch * n_in, batch * n_out
            wps = windows_per_sequence(tiles, w)
            n_windows = batch * wps
            h_cu = (np.arange(batch + 1, dtype=np.int32) * n_in).astype(np.int32)
            cu = torch.from_numpy(h_cu).to(dev)
            if n_out > n_in:
                raise ValueError("a stage cannot add tokens")
            win_offsets = torch.empty(n_windows + 1, **i32)
            win_tokens = torch.empty(max(sum_in, 1), **i32)
            win_remove = torch.zeros(max(n_windows, 1), **i32)
            cu_target = torch.from_numpy((np.arange(batch + 1, dtype=np.int32) * n_out).astype(np.int32)).to(dev)
            status = torch.zeros(batch, **i32)
            bound = min(max_window_cells(tiles, grid_h, grid_w, w), n_in)
            prob = B.Problem(batch=batch, d=d, heads=heads, head_dim=head_dim, dtype=dtype, h_cu_vis=h_cu,
                             cu_vis=cu, h_cu_txt=self.h_cu_txt, cu_txt=self.cu_txt, n_windows=n_windows,
                             max_window_tokens=bound, win_offsets=win_offsets, win_tokens=win_tokens,
                             win_remove=win_remove, h_win_remove=None, metric=metric, direction=self._dir)
            ws_bytes = max(ws_bytes, B.lightkv_workspace_size(prob))
            st = StageBuffers(
                n_in=n_in, n_out=n_out, w=w, problem=prob, h_cu_vis=h_cu, cu_vis=cu, win_offsets=win_offsets,
                win_tokens=win_tokens, win_remove=win_remove, cu_target=cu_target, status=status,
                xi=torch.empty(sum_in, dtype=torch.float32, device=dev),
                best_fd=torch.empty(sum_in, dtype=torch.float32, device=dev),
                best_dst=torch.empty(sum_in, **i32), dst=torch.empty(sum_in, **i32),
                new_index=torch.empty(sum_in, **i32), grp_offsets=torch.empty(sum_in + 1, **i32),
                grp_src=torch.empty(max(sum_in - sum_out, 1), **i32), cu_vis_out=torch.empty(batch + 1, **i32),
                X_out=torch.empty(sum_out, d, dtype=self.tdtype, device=dev),
                K_out=torch.empty(sum_out, d, dtype=self.tdtype, device=dev),
                V_out=torch.empty(sum_out, d, dtype=self.tdtype, device=dev),
                pos_out=torch.empty(sum_out, **i32),
                x_sq_out=torch.empty(max(sum_out, 1), dtype=torch.float32, device=dev))
            self.stages.append(st)
            n_in = n_out
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        # the whole schedule as one library call (lightkv_compress_schedule): the stages' descriptors and buffers as a C array
        self.c_stages = B.StageArray([dict(problem=st.problem, w=st.w, win_offsets=st.win_offsets, win_tokens=st.win_tokens,
                                           xi=st.xi, best_fd=st.best_fd, best_dst=st.best_dst, dst=st.dst,
                                           new_index=st.new_index, grp_offsets=st.grp_offsets, grp_src=st.grp_src,
                                           cu_vis_out=st.cu_vis_out, X_out=st.X_out, K_out=st.K_out, V_out=st.V_out,
                                           pos_out=st.pos_out, x_sqnorm_out=st.x_sq_out, cu_vis_target=st.cu_target,
                                           win_remove=st.win_remove, status=st.status) for st in self.stages])
        # xi needs neither the windows nor the FD scores and is only consumed by the merge, so it is enqueued on a
        # second stream (default priority) that forks at the start of a stage and joins before aggregate/compact
        self.side = torch.cuda.Stream(device=dev)
        self.side2 = torch.cuda.Stream(device=dev)   # builds the next stage's windows during the merge
        # scratch copies for the unfused path (aggregate works in place)
        if not fused:
            s0 = self.stages[0]
            n0 = batch * s0.n_in
            self.tmp = [torch.empty(n0, d, dtype=self.tdtype, device=dev) for _ in range(3)]

    # one stage; inputs are device tensors of this stage's shape
    def run_stage(self, s: int, X, K, V, Q, pos, *, xi_mode=B.XI_TEXT_QUERY, lse=None, softmax_scale=0.0,
                  xi_given: Optional[torch.Tensor] = None, score_K=None, stream=None, windows_ready=False,
                  prepare_next=False, x_sqnorm: Optional[torch.Tensor] = None):
        """score_K: keys of the xi contraction when they are not the K rows being merged
        (vision-query mode: Q holds the vision queries, score_K the prompt keys).
        windows_ready: the window lists of this stage were already built on the second helper stream
        (by the previous stage's prepare_next); prepare_next: build the next stage's windows while this
        stage's rows are being merged (they only need pos and new_index, not the merged rows).
        x_sqnorm: |x|^2 of the rows of X when X is the previous stage's X_out (that stage's x_sq_out)."""
        st = self.stages[s]
        p = st.problem
        main = torch.cuda.current_stream() if stream is None else stream
        xi = st.xi
        # small steps with windows of at most 64 tokens: lightkv_score_select runs the xi passes inside the launches of
        # the FD chain, all on the caller's stream; otherwise xi gets the helper stream
        one_stream = (self.fused and xi_given is None and 0 < p.c.max_window_tokens <= 64
                      and X.shape[0] <= B.ONE_STREAM_MAX_TOKENS)
        if xi_given is not None:
            xi = xi_given
        elif not one_stream:
            self.side.wait_stream(main)                                   # fork
            B.lightkv_score(p, None, Q, K if score_K is None else score_K, xi, None, None, self.ws, xi_mode=xi_mode,
                            lse=lse, softmax_scale=softmax_scale, stream=self.side)          # xi half only
        if windows_ready:
            main.wait_stream(self.side2)
        else:
            B.lightkv_build_windows(self.batch, st.h_cu_vis, st.cu_vis, pos, self.tiles, self.grid_h, self.grid_w, st.w,
                                    st.win_offsets, st.win_tokens, stream=main)
            B.lightkv_window_counts(self.batch, p.c.n_windows, st.win_offsets, B.COUNT_TARGET, st.win_remove,
                                    direction=self._dir, cu_vis=st.cu_vis, cu_vis_target=st.cu_target, status=st.status, stream=main)
        if one_stream:
            B.lightkv_score_select(p, X, Q, K if score_K is None else score_K, xi, st.best_fd, st.best_dst, st.dst,
                                   st.new_index, st.grp_offsets, st.grp_src, st.cu_vis_out, self.ws, xi_mode=xi_mode,
                                   lse=lse, softmax_scale=softmax_scale, x_sqnorm=x_sqnorm, stream=main)
        elif self.fused:   # FD half + selection
            B.lightkv_score_select(p, X, None, None, xi, st.best_fd, st.best_dst, st.dst, st.new_index, st.grp_offsets,
                                   st.grp_src, st.cu_vis_out, self.ws, xi_mode=B.XI_GIVEN, x_sqnorm=x_sqnorm, stream=main)
        else:
            B.lightkv_score(p, X, None, None, xi, st.best_fd, st.best_dst, self.ws, xi_mode=B.XI_GIVEN,
                            x_sqnorm=x_sqnorm, stream=main)
            B.lightkv_select(p, st.best_fd, st.best_dst, st.dst, st.new_index, st.grp_offsets, st.grp_src,
                             st.cu_vis_out, self.ws, stream=main)
        if prepare_next and self.fused and s + 1 < len(self.stages):
            # the next stage's windows follow from pos and new_index alone: they are built on the second helper stream
            # while the rows are merged on this one
            nx = self.stages[s + 1]
            self.side2.wait_stream(main)                                  # fork after select
            B.lightkv_build_windows_next(self.batch, st.h_cu_vis, st.cu_vis, pos, st.new_index, st.cu_vis_out, self.tiles,
                                         self.grid_h, self.grid_w, nx.w, nx.win_offsets, nx.win_tokens,
                                         stream=self.side2)
            B.lightkv_window_counts(self.batch, nx.problem.c.n_windows, nx.win_offsets, B.COUNT_TARGET, nx.win_remove,
                                    direction=self._dir, cu_vis=st.cu_vis_out, cu_vis_target=nx.cu_target, status=nx.status, stream=self.side2)
        if xi_given is None and not one_stream:
            main.wait_stream(self.side)                                   # join: the merge needs xi
        stream = main
        if self.fused:
            B.lightkv_aggregate_compact(p, st.new_index, st.grp_offsets, st.grp_src, xi, X, K, V, pos, st.X_out,
                                        st.K_out, st.V_out, st.pos_out, x_sqnorm_out=st.x_sq_out, stream=stream)
        else:
            n = X.shape[0]
            tx, tk, tv = (t[:n] for t in self.tmp)
            tx.copy_(X); tk.copy_(K); tv.copy_(V)
            B.lightkv_aggregate(p, st.grp_offsets, st.grp_src, xi, tx, tk, tv, stream=stream)
            B.lightkv_compact(p, st.new_index, tx, tk, tv, pos, st.X_out, st.K_out, st.V_out, st.pos_out,
                              x_sqnorm_out=st.x_sq_out, stream=stream)
        return st

    def run(self, X, K, V, Q, pos, stream=None):
        """All stages back to back; returns the last stage's buffers (its *_out tensors hold the result).  The fused
        pipeline is one call of lightkv_compress_schedule; the unfused one (separate lightkv_aggregate and
        lightkv_compact, kept for comparison) is driven stage by stage from here."""
        if self.fused:
            B.lightkv_compress_schedule(self.c_stages, self.tiles, self.grid_h, self.grid_w, X, K, V, pos, Q, self.ws,
                                        stream=stream)
            return self.stages[-1]
        st = None
        main = torch.cuda.current_stream() if stream is None else stream
        for s in range(len(self.stages)):
            st = self.run_stage(s, X, K, V, Q, pos, stream=main, windows_ready=(s > 0 and self.fused),
                                prepare_next=True, x_sqnorm=(st.x_sq_out if st is not None else None))
            X, K, V, pos = st.X_out, st.K_out, st.V_out, st.pos_out
        main.wait_stream(self.side2)   # nothing is left running on a helper stream when run() returns
        return st


@dataclass
class EdgeStepResult:
    """Outputs of one step whose token count depends on the data; every tensor is cut to the rows the step really wrote.
    The tensors are views of buffers the schedule owns: those of a step stay valid until the step after next runs (X, K,
    V, pos: two sets in turn) or until the next step runs (everything else)."""
    h_cu_vis_out: np.ndarray
    X: torch.Tensor
    K: torch.Tensor
    V: torch.Tensor
    pos: torch.Tensor
    xi: torch.Tensor
    best_fd: torch.Tensor
    best_dst: torch.Tensor
    dst: torch.Tensor
    new_index: torch.Tensor
    grp_offsets: torch.Tensor
    grp_src: torch.Tensor
    win_offsets: torch.Tensor
    win_tokens: torch.Tensor
    win_remove: torch.Tensor     # per-window counts as the step used them (device)
    cu_vis_out: torch.Tensor     # device copy of h_cu_vis_out

    @property
    def h_win_edges(self) -> np.ndarray:
        """The per-window counts on the host (a read-back: call it outside timed regions)."""
        return self.win_remove.cpu().numpy()


class EdgeTopKSchedule:
    """The hierarchical schedule for the matchings whose token counts depend on the data:
      match="edge_topk"      the k lowest-FD edges per window (LIGHTKV_MATCH_EDGE_TOPK, k = floor(rho v / 2) as
                             Sec. 3.2.1 counts the pairs), windows of any size the library takes;
      match="full_pairwise"  every token against every other token of its window (LIGHTKV_MATCH_FULL_PAIRWISE, the
                             appendix ablation), at most floor(rho v) tokens leave a window;
      match="best_per_a"     the default matching with r_w = floor(rho v_w) taken from the windows as they are
                             (Sec. 3.2.2's ratio instead of fixed token budgets).
    Every buffer is allocated once, here, for the largest step (the first); the per-window counts are computed and
    consumed on the device.  The one thing the host reads back per step is cu_vis_out, the batch + 1 sequence offsets
    after the step: the next step's descriptor needs them.  Nothing here is captured in a graph (the sizes of a step
    depend on the data of the one before).  run() is one library call (lightkv_compress_schedule_ratio); run_step() and
    run_steps() drive the same stages call by call."""

    def __init__(self, *, dtype: str, batch: int, d: int, heads: int, head_dim: int, tiles: int, grid_h: int,
                 grid_w: int, cu_txt: np.ndarray, windows_per_axis: Sequence[int], rho: Sequence[float],
                 device="cuda:0", metric: str = "cosine", match: str = "edge_topk"):
        self.dtype, self.batch, self.d, self.heads, self.head_dim = dtype, batch, d, heads, head_dim
        self.tiles, self.grid_h, self.grid_w = tiles, grid_h, grid_w
        self.windows_per_axis, self.rho = list(windows_per_axis), list(rho)
        self.device = torch.device(device)
        self.metric = metric
        if match not in ("edge_topk", "full_pairwise", "best_per_a"):
            raise ValueError(match)
        self.match = match
        self.h_cu_txt = np.ascontiguousarray(cu_txt, dtype=np.int32)
        self.cu_txt = torch.from_numpy(self.h_cu_txt).to(self.device)
        dev, i32 = self.device, dict(dtype=torch.int32, device=self.device)
        n0 = tiles * grid_h * grid_w
        cap = max(batch * n0, 1)
        self.capacity = cap
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        f32 = dict(dtype=torch.float32, device=dev)
        self._win_tokens = torch.empty(cap, **i32)
        self._xi, self._best_fd = torch.empty(cap, **f32), torch.empty(cap, **f32)
        self._best_dst, self._dst, self._new_index = (torch.empty(cap, **i32) for _ in range(3))
        self._grp_offsets, self._grp_src = torch.empty(cap + 1, **i32), torch.empty(cap, **i32)
        self._cu = [torch.empty(batch + 1, **i32) for _ in range(2)]          # in turn: a step's cu_vis and cu_vis_out
        self._out = [tuple(torch.empty(cap, d, dtype=tdt, device=dev) for _ in range(3)) + (torch.empty(cap, **i32),)
                     for _ in range(2)]
        self._win_offsets, self._win_remove, self._bound = [], [], []
        h_full = (np.arange(batch + 1, dtype=np.int32) * n0).astype(np.int32)
        ws_bytes = 0
        for w in self.windows_per_axis:
            n_windows = batch * windows_per_sequence(tiles, w)
            self._win_offsets.append(torch.empty(n_windows + 1, **i32))
            self._win_remove.append(torch.empty(max(n_windows, 1), **i32))
            self._bound.append(min(max_window_cells(tiles, grid_h, grid_w, w), max(n0, 1)))
            ws_bytes = max(ws_bytes, B.lightkv_workspace_size(self._problem(len(self._bound) - 1, h_full, self._cu[0])))
        self._ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self._call = None        # buffers and descriptors of the one-call form, made on first use

    def _match_code(self):
        return {"edge_topk": B.MATCH_EDGE_TOPK, "full_pairwise": B.MATCH_FULL_PAIRWISE, "best_per_a": B.MATCH_BEST_PER_A}[self.match]

    def _count_mode(self):
        return B.COUNT_EDGES if self.match == "edge_topk" else B.COUNT_RATIO

    def _problem(self, s, h_cu_vis, cu_vis, h_win_offsets=None, h_k=None):
        n_windows = self.batch * windows_per_sequence(self.tiles, self.windows_per_axis[s])
        bound = min(self._bound[s], max(int(np.diff(h_cu_vis).max()), 1))
        return B.Problem(batch=self.batch, d=self.d, heads=self.heads, head_dim=self.head_dim, dtype=self.dtype,
                         h_cu_vis=h_cu_vis, cu_vis=cu_vis, h_cu_txt=self.h_cu_txt, cu_txt=self.cu_txt, n_windows=n_windows,
                         max_window_tokens=0 if h_win_offsets is not None else bound, win_offsets=self._win_offsets[s],
                         win_tokens=self._win_tokens, win_remove=self._win_remove[s], h_win_offsets=h_win_offsets,
                         h_win_remove=h_k, metric=self.metric, match=self._match_code())

    def run_step(self, s: int, h_cu_vis: np.ndarray, X, K, V, Q, pos, *, xi_given=None, h_win_edges=None,
                 marks: Optional[list] = None, cu_vis=None, host_mirror: bool = True) -> EdgeStepResult:
        """marks: if a list, (name, event) pairs are appended around the three library calls (current stream).
        cu_vis: the device copy of h_cu_vis if the caller has one (run() hands on the previous step's cu_vis_out).
        h_win_edges: per-window counts given by the caller instead of the ratio (then they and the window sizes are
        validated on the host, which costs a read-back of the window offsets; host_mirror=False hands them to the
        device only, as the ratio's counts are)."""
        def mark(name):
            if marks is not None:
                ev = torch.cuda.Event(enable_timing=True)
                ev.record()
                marks.append((name, ev))

        batch, w = self.batch, self.windows_per_axis[s]
        h_cu_vis = np.ascontiguousarray(h_cu_vis, dtype=np.int32)
        sum_n = int(h_cu_vis[-1])
        if sum_n > self.capacity:
            raise ValueError("more tokens than the schedule was built for")
        if cu_vis is None:
            cu_vis = self._cu[0]
            cu_vis.copy_(torch.from_numpy(h_cu_vis))
        cu_vis_out = self._cu[1] if cu_vis is self._cu[0] else self._cu[0]
        n_windows = batch * windows_per_sequence(self.tiles, w)
        win_offsets, win_tokens, win_remove = self._win_offsets[s], self._win_tokens, self._win_remove[s]
        mark("build_windows")
        B.lightkv_build_windows(batch, h_cu_vis, cu_vis, pos, self.tiles, self.grid_h, self.grid_w, w, win_offsets,
                                win_tokens)
        mark("end")
        if h_win_edges is None:                              # k_w = floor(rho v_w / 2) (r_w = floor(rho v_w)), on the device
            B.lightkv_window_counts(batch, n_windows, win_offsets, self._count_mode(), win_remove, rho=self.rho[s])
            prob = self._problem(s, h_cu_vis, cu_vis)
        else:
            h_k = np.ascontiguousarray(h_win_edges, dtype=np.int32)
            win_remove[:n_windows].copy_(torch.from_numpy(h_k))
            mirror = host_mirror and self.match == "edge_topk"
            prob = self._problem(s, h_cu_vis, cu_vis, win_offsets.cpu().numpy() if mirror else None, h_k if mirror else None)
            # with the host's counts the library sizes the edge list from them -- up to every pair of a window -- and
            # writes that many group entries; counts known to the device only are clamped to one per token
            if mirror and int(h_k.sum()) > self._grp_src.numel():
                self._grp_src = torch.empty(int(h_k.sum()), dtype=torch.int32, device=self.device)
        need = B.lightkv_workspace_size(prob)
        if need > self._ws.numel():                          # (the plans are not monotone in the sizes: a rare regrow)
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        xi = self._xi[:sum_n] if xi_given is None else xi_given
        best_fd, best_dst, dst, new_index = (t[:max(sum_n, 1)] for t in (self._best_fd, self._best_dst, self._dst, self._new_index))
        grp_offsets, grp_src = self._grp_offsets[:sum_n + 1], self._grp_src
        mark("score_select")
        B.lightkv_score_select(prob, X, Q, K, xi, best_fd, best_dst, dst, new_index, grp_offsets, grp_src, cu_vis_out,
                               self._ws, xi_mode=B.XI_TEXT_QUERY if xi_given is None else B.XI_GIVEN)
        mark("end")
        X_out, K_out, V_out, pos_out = self._out[0] if X.data_ptr() != self._out[0][0].data_ptr() else self._out[1]
        mark("aggregate_compact")
        B.lightkv_aggregate_compact(prob, new_index, grp_offsets, grp_src, xi, X, K, V, pos, X_out, K_out, V_out, pos_out)
        mark("end")
        h_out = cu_vis_out.cpu().numpy()                     # the one read-back: the sequence lengths after the step
        n_out = int(h_out[-1])
        res = EdgeStepResult(h_out, X_out[:n_out], K_out[:n_out], V_out[:n_out], pos_out[:n_out], xi, best_fd, best_dst,
                             dst, new_index, grp_offsets, grp_src, win_offsets, win_tokens, win_remove[:n_windows], cu_vis_out)
        return res

    def _call_buffers(self, h_cu_vis):
        """Per-stage index buffers and descriptors for lightkv_compress_schedule_ratio (the row tensors are the two sets
        the steps use in turn)."""
        i32, f32 = dict(dtype=torch.int32, device=self.device), dict(dtype=torch.float32, device=self.device)
        cap, batch = self.capacity, self.batch
        cu_in = torch.from_numpy(h_cu_vis).to(self.device)
        stages, bufs = [], []
        for s, w in enumerate(self.windows_per_axis):
            n_windows = batch * windows_per_sequence(self.tiles, w)
            b = dict(win_offsets=self._win_offsets[s], win_tokens=torch.empty(cap, **i32), win_remove=self._win_remove[s],
                     xi=torch.empty(cap, **f32), best_fd=torch.empty(cap, **f32), best_dst=torch.empty(cap, **i32),
                     dst=torch.empty(cap, **i32), new_index=torch.empty(cap, **i32), grp_offsets=torch.empty(cap + 1, **i32),
                     grp_src=torch.empty(cap, **i32), cu_vis_out=torch.empty(batch + 1, **i32))
            X_out, K_out, V_out, pos_out = self._out[s % 2]
            prob = B.Problem(batch=batch, d=self.d, heads=self.heads, head_dim=self.head_dim, dtype=self.dtype,
                             h_cu_vis=h_cu_vis, cu_vis=cu_in, h_cu_txt=self.h_cu_txt, cu_txt=self.cu_txt,
                             n_windows=n_windows, max_window_tokens=self._bound[s], win_offsets=b["win_offsets"],
                             win_tokens=b["win_tokens"], win_remove=b["win_remove"], metric=self.metric,
                             match=self._match_code())
            need = B.lightkv_workspace_size(prob)
            if need > self._ws.numel():
                self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
            stages.append(dict(problem=prob, w=w, X_out=X_out, K_out=K_out, V_out=V_out, pos_out=pos_out, **b))
            bufs.append(b)
        return dict(h_cu_vis=h_cu_vis.copy(), cu_in=cu_in, bufs=bufs, stages=B.StageArray(stages))

    def run(self, h_cu_vis: np.ndarray, X, K, V, Q, pos, marks: Optional[list] = None) -> List[EdgeStepResult]:
        """Every stage in one library call.  X, K, V, pos must not be the schedule's own output sets.  With marks the
        stages are driven call by call instead (run_steps), so that every call can be timed."""
        if marks is not None:
            return self.run_steps(h_cu_vis, X, K, V, Q, pos, marks=marks)
        h_cu_vis = np.ascontiguousarray(h_cu_vis, dtype=np.int32)
        if int(h_cu_vis[-1]) > self.capacity:
            raise ValueError("more tokens than the schedule was built for")
        c = self._call
        if c is None or not np.array_equal(c["h_cu_vis"], h_cu_vis):
            c = self._call = self._call_buffers(h_cu_vis)
        h_out = B.lightkv_compress_schedule_ratio(c["stages"], self.rho, self.tiles, self.grid_h, self.grid_w, X, K, V,
                                                  pos, Q, self._ws)
        out, n_in = [], int(h_cu_vis[-1])
        for s, b in enumerate(c["bufs"]):
            X_out, K_out, V_out, pos_out = self._out[s % 2]
            n_out = int(h_out[s, -1])
            n_windows = self.batch * windows_per_sequence(self.tiles, self.windows_per_axis[s])
            out.append(EdgeStepResult(h_out[s], X_out[:n_out], K_out[:n_out], V_out[:n_out], pos_out[:n_out],
                                      b["xi"][:n_in], b["best_fd"][:max(n_in, 1)], b["best_dst"][:max(n_in, 1)],
                                      b["dst"][:max(n_in, 1)], b["new_index"][:max(n_in, 1)], b["grp_offsets"][:n_in + 1],
                                      b["grp_src"], b["win_offsets"], b["win_tokens"], b["win_remove"][:n_windows],
                                      b["cu_vis_out"]))
            n_in = n_out
        return out

    def run_steps(self, h_cu_vis: np.ndarray, X, K, V, Q, pos, marks: Optional[list] = None) -> List[EdgeStepResult]:
        """The same stages call by call (one read-back per stage, here on the host side of the binding)."""
        out, cu_vis = [], None
        for s in range(len(self.windows_per_axis)):
            r = self.run_step(s, h_cu_vis, X, K, V, Q, pos, marks=marks, cu_vis=cu_vis)
            out.append(r)
            h_cu_vis, X, K, V, pos, cu_vis = r.h_cu_vis_out, r.X, r.K, r.V, r.pos, r.cu_vis_out
        return out
