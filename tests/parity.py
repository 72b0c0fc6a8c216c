"""Stage-by-stage comparison of the HIP path with the CPU oracle (used by the GPU tests, the smoke
check and nothing else).  Every stage is "teacher forced": the oracle gets exactly the tensors the
GPU stage consumed, so storage rounding of earlier stages cannot fork the selection.

Tolerances (stated by the task's parity bar):
  index sets       bit exact, except where the oracle's own fp64 scores are tied within 1e-6
                   (relative on the cosine); such cases are verified by score, and counted
  xi               relative 1e-3 (bf16 inputs) / 1e-5 (fp32)
  best_fd          absolute 1e-5 (bf16 inputs) / 1e-6 (fp32)
                   (distance metrics: the same figures relative to the window's largest |a|^2 + |b|^2, the scale of
                   the terms whose difference the distance is, and compared on the squared distance -- the square
                   root is monotone, so selection is unaffected, but it has no bounded error near zero)
  X, K, V rows     per-row |delta|_2/|ref|_2 and max|delta|/max|ref| <= 2e-2 (bf16 I/O) / 1e-5 (fp32)
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

from oracle import lightkv_oracle as O

TIE_BAND = 1e-6


def to_dev(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    from paper_2605_00789_amd import to_device
    return to_device(a, dtype, device)


def from_dev(t: torch.Tensor, dtype: str) -> np.ndarray:
    from paper_2605_00789_amd import from_device
    return from_device(t, dtype)


@dataclass
class StageReport:
    stage: int
    n_in: int
    n_out: int
    edge_ties: int = 0          # A rows whose GPU partner differs from the oracle's but ties within the band
    window_ties: int = 0        # windows whose merged set differs but ties within the band
    max_xi_rel: float = 0.0
    max_fd_abs: float = 0.0
    max_row_rel: float = 0.0
    max_elem_rel: float = 0.0
    notes: list = field(default_factory=list)


def check_stage(pipe, s: int, Xs, Ks, Vs, Qs, pos, dtype: str, *, xi_mode=0, lse=None, xi_given=None,
                softmax_scale=None, Qdev=None, score_K=None, extra_run_kwargs=None) -> tuple:
    """Runs stage s of `pipe` on the storage arrays (numpy) and checks every output against the oracle.
    Returns (report, outputs as storage arrays)."""
    st_cfg = pipe.stages[s]
    batch = pipe.batch
    dX, dK, dV = to_dev(Xs, dtype), to_dev(Ks, dtype), to_dev(Vs, dtype)
    dQ = Qdev if Qdev is not None else (to_dev(Qs, dtype) if Qs is not None else None)
    dpos = torch.from_numpy(np.ascontiguousarray(pos, dtype=np.int32)).to(dX.device)
    kw = dict(extra_run_kwargs or {})
    if lse is not None:
        kw["lse"] = torch.from_numpy(np.ascontiguousarray(lse, dtype=np.float32)).to(dX.device)
    if xi_given is not None:
        kw["xi_given"] = torch.from_numpy(np.ascontiguousarray(xi_given, dtype=np.float32)).to(dX.device)
    if softmax_scale is not None:
        kw["softmax_scale"] = float(softmax_scale)
    if score_K is not None:
        kw["score_K"] = to_dev(score_K, dtype)
    st = pipe.run_stage(s, dX, dK, dV, dQ, dpos, xi_mode=xi_mode, **kw)
    torch.cuda.synchronize()

    g = {k: getattr(st, k).cpu().numpy() for k in ("win_offsets", "win_tokens", "best_fd", "best_dst", "dst",
                                                     "new_index", "grp_offsets", "grp_src", "cu_vis_out", "pos_out")}
    g_xi = (st.xi.cpu().numpy() if xi_given is None else np.asarray(xi_given, dtype=np.float32))
    rep = StageReport(stage=s, n_in=st_cfg.n_in, n_out=st_cfg.n_out)
    bf16 = dtype == "bf16"
    metric = getattr(pipe, "metric", "cosine")
    direction = getattr(pipe, "direction", "a_to_b")   # "b_to_a": A below is the proposing set B, Bn the receiving set A

    # ---- windows: exact
    cu_vis = st_cfg.h_cu_vis
    wo, wt = O.build_windows(pos, cu_vis, pipe.tiles, pipe.grid_h, pipe.grid_w, st_cfg.w)
    np.testing.assert_array_equal(g["win_offsets"], wo, err_msg="win_offsets")
    np.testing.assert_array_equal(g["win_tokens"][:len(wt)], wt, err_msg="win_tokens")
    # per-window counts: the stage's token budget spread over the windows as they are (exact)
    n_seq = np.diff(np.asarray(cu_vis, dtype=np.int64))
    rem, infeasible = O.removal_counts_target(wo, batch, n_seq - st_cfg.n_out, direction)
    assert not infeasible.any(), "the stage's budget cannot be met by these windows"
    np.testing.assert_array_equal(st.win_remove.cpu().numpy()[:len(rem)], rem, err_msg="win_remove")
    np.testing.assert_array_equal(st.status.cpu().numpy(), np.zeros(batch, dtype=np.int32), err_msg="status")

    X64, K64, V64 = O.widen(Xs, dtype), O.widen(Ks, dtype), O.widen(Vs, dtype)
    # ---- xi
    if xi_given is None:
        Q64 = O.widen(Qs, dtype)
        lse64 = None if lse is None else np.asarray(lse, dtype=np.float32).astype(np.float64)
        if xi_mode == 0:
            xi_ref = O.xi_text_query(Q64, K64, cu_vis, pipe.h_cu_txt, pipe.heads, pipe.head_dim, scale=softmax_scale,
                                     lse=lse64)
        else:
            xi_ref = O.xi_vision_query(Q64, O.widen(score_K, dtype), lse64, cu_vis, pipe.h_cu_txt, pipe.heads, pipe.head_dim,
                                       scale=softmax_scale)
        rel = np.abs(g_xi - xi_ref) / np.maximum(np.abs(xi_ref), 1e-300)
        rep.max_xi_rel = float(rel.max()) if len(rel) else 0.0
        assert rep.max_xi_rel <= (1e-3 if bf16 else 1e-5), "xi relative error %.3g" % rep.max_xi_rel
    else:
        xi_ref = np.asarray(xi_given, dtype=np.float64)

    # ---- best edge per A node, then the merged set per window
    n = X64.shape[0]
    exp_new_removed = 0
    for w in range(len(wo) - 1):
        toks = wt[wo[w]:wo[w + 1]]
        A, Bn = O.split_window(toks, direction)
        if len(Bn) == 0 or len(A) == 0:
            assert np.all(g["best_dst"][toks] == -1) and np.all(np.isinf(g["best_fd"][toks]))
            assert np.all(g["dst"][toks] == -1)
            continue
        fd = O.feature_divergence(X64[A], X64[Bn], metric)        # oracle's dense FD block (fp64)
        g_fd = g["best_fd"][A].astype(np.float64)
        scale = 1.0
        if metric != "cosine":
            if metric == "euclidean":
                fd, g_fd = fd * fd, g_fd * g_fd
            scale = float((X64[A] ** 2).sum(axis=1).max() + (X64[Bn] ** 2).sum(axis=1).max())
        band = TIE_BAND * scale
        j_ref = np.argmin(fd, axis=1)
        f_ref = fd[np.arange(len(A)), j_ref]
        assert np.all(g["best_dst"][Bn] == -1) and np.all(np.isinf(g["best_fd"][Bn]))
        # partner: same index, or a score tie inside the band
        b_gpu = g["best_dst"][A]
        local = {int(t): k for k, t in enumerate(Bn)}
        for la in np.nonzero(b_gpu != Bn[j_ref])[0]:
            assert int(b_gpu[la]) in local, "partner of token %d is outside its window's B set" % A[la]
            f_g = fd[la, local[int(b_gpu[la])]]
            assert f_g <= f_ref[la] + band, "window %d row %d: partner FD %.9g vs best %.9g" % (w, la, f_g, f_ref[la])
            rep.edge_ties += 1
        err = np.abs(g_fd - f_ref) / scale
        rep.max_fd_abs = max(rep.max_fd_abs, float(err.max()))
        # merged set
        r = int(rem[w])
        order = sorted(range(len(A)), key=lambda la: (f_ref[la], la))
        ref_set = set(int(A[la]) for la in order[:r])
        gpu_set = set(int(a) for a in A if g["dst"][a] >= 0)
        assert len(gpu_set) == r, "window %d: %d merged, expected %d" % (w, len(gpu_set), r)
        exp_new_removed += r
        if gpu_set != ref_set:
            tau = f_ref[order[r - 1]]
            for la, a in enumerate(A):
                if int(a) in gpu_set:
                    assert f_ref[la] <= tau + band, "window %d: merged token %d has FD %.9g > threshold %.9g" % (w, a, f_ref[la], tau)
                else:
                    assert f_ref[la] >= tau - band, "window %d: kept token %d has FD %.9g < threshold %.9g" % (w, a, f_ref[la], tau)
            rep.window_ties += 1
        # a merged token goes to the partner the score step reported
        for a in gpu_set:
            assert g["dst"][a] == g["best_dst"][a]
        assert np.all(g["dst"][Bn] == -1)
    assert rep.max_fd_abs <= (1e-5 if bf16 else 1e-6), "best_fd abs error %.3g" % rep.max_fd_abs

    # ---- index structures follow from dst: exact
    dst = g["dst"]
    np.testing.assert_array_equal(g["new_index"], O.kept_index(dst), err_msg="new_index")
    go, gs = O.groups_csr(dst)
    np.testing.assert_array_equal(g["grp_offsets"], go, err_msg="grp_offsets")
    np.testing.assert_array_equal(g["grp_src"][:len(gs)], gs, err_msg="grp_src")
    keep = dst < 0
    cu_out = np.zeros(batch + 1, dtype=np.int32)
    for b in range(batch):
        cu_out[b + 1] = cu_out[b] + int(keep[cu_vis[b]:cu_vis[b + 1]].sum())
    np.testing.assert_array_equal(g["cu_vis_out"], cu_out, err_msg="cu_vis_out")
    n_out = int(keep.sum())
    assert n_out == n - exp_new_removed == batch * st_cfg.n_out                  # kept + merged = N
    np.testing.assert_array_equal(g["pos_out"][:n_out], np.asarray(pos)[keep], err_msg="pos_out")

    # ---- values: oracle message passing on the GPU's (verified) selection
    outs = {}
    tol = 2e-2 if bf16 else 1e-5
    for name, Y64, dev_out in (("X", X64, st.X_out), ("K", K64, st.K_out), ("V", V64, st.V_out)):
        ref = O.compact(O.message_passing(Y64, xi_ref, dst), dst)
        got_store = from_dev(dev_out[:n_out], dtype)
        got = O.widen(got_store, dtype)
        num = np.linalg.norm(got - ref, axis=1)
        den = np.maximum(np.linalg.norm(ref, axis=1), 1e-300)
        row_rel = float((num / den).max()) if n_out else 0.0
        elem_rel = float((np.abs(got - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-300)).max()) if n_out else 0.0
        rep.max_row_rel = max(rep.max_row_rel, row_rel)
        rep.max_elem_rel = max(rep.max_elem_rel, elem_rel)
        assert row_rel <= tol and elem_rel <= tol, "%s rows: rel %.3g / %.3g" % (name, row_rel, elem_rel)
        # rows that were only copied are bit exact
        untouched = (go[1:] - go[:-1])[keep] == 0
        src_store = {"X": Xs, "K": Ks, "V": Vs}[name]
        np.testing.assert_array_equal(got_store[untouched], np.asarray(src_store)[keep][untouched],
                                      err_msg=name + " copied rows")
        outs[name] = got_store
    outs["pos"] = g["pos_out"][:n_out].copy()
    outs["cu_vis"] = cu_out
    outs["dst"] = dst
    outs["xi"] = g_xi
    return rep, outs


def check_workload(wl, pipe=None, stages=None, fused=True, metric="cosine", direction="a_to_b"):
    """Runs all stages of a workload teacher-forced; returns the per-stage reports."""
    from paper_2605_00789_amd import CompressionPipeline
    if pipe is None:
        pipe = CompressionPipeline(dtype=wl.dtype, batch=wl.batch, d=wl.d, heads=wl.heads, head_dim=wl.head_dim,
                                   tiles=wl.tiles, grid_h=wl.grid_h, grid_w=wl.grid_w, cu_txt=wl.cu_txt,
                                   windows_per_axis=wl.windows_per_axis, targets=wl.targets, fused=fused, metric=metric,
                                   direction=direction)
    X, K, V, pos = wl.X, wl.K, wl.V, wl.pos
    reports = []
    for s in range(wl.stages if stages is None else stages):
        rep, out = check_stage(pipe, s, X, K, V, wl.Q, pos, wl.dtype)
        reports.append(rep)
        X, K, V, pos = out["X"], out["K"], out["V"], out["pos"]
    return reports


# ---------------------------------------------------------------------------------------------------------------
# Step 2 read literally: the k lowest-FD edges of every window (LIGHTKV_MATCH_EDGE_TOPK)
# ---------------------------------------------------------------------------------------------------------------
@dataclass
class EdgeReport:
    stage: int
    n_in: int
    n_out: int
    edges: int = 0
    window_ties: int = 0        # windows whose edge set differs from the oracle's but ties within the band
    max_xi_rel: float = 0.0
    max_row_rel: float = 0.0


def check_edge_step(sched, s: int, h_cu_vis, Xs, Ks, Vs, Qs, pos, dtype: str, *, xi_given=None, h_win_edges=None,
                    host_mirror=True):
    """Runs step s of an EdgeTopKSchedule on storage arrays and checks every output against the oracle, which gets
    exactly the tensors the GPU step consumed.  Edge sets are compared exactly; where they differ every edge the GPU
    took must lie within TIE_BAND of the oracle's k-th lowest FD and every edge it left out not below it."""
    batch = sched.batch
    dX, dK, dV = to_dev(Xs, dtype), to_dev(Ks, dtype), to_dev(Vs, dtype)
    dQ = to_dev(Qs, dtype)
    dpos = torch.from_numpy(np.ascontiguousarray(pos, dtype=np.int32)).to(dX.device)
    dxi = None if xi_given is None else torch.from_numpy(np.ascontiguousarray(xi_given, dtype=np.float32)).to(dX.device)
    r = sched.run_step(s, h_cu_vis, dX, dK, dV, dQ, dpos, xi_given=dxi, h_win_edges=h_win_edges, host_mirror=host_mirror)
    torch.cuda.synchronize()
    g = {k: getattr(r, k).cpu().numpy() for k in ("win_offsets", "win_tokens", "best_fd", "best_dst", "dst", "new_index",
                                                  "grp_offsets", "grp_src", "pos")}
    g_xi = r.xi.cpu().numpy()
    bf16 = dtype == "bf16"
    metric = sched.metric
    n = int(h_cu_vis[-1])
    rep = EdgeReport(stage=s, n_in=n, n_out=int(r.h_cu_vis_out[-1]))

    wo, wt = O.build_windows(pos, h_cu_vis, sched.tiles, sched.grid_h, sched.grid_w, sched.windows_per_axis[s])
    np.testing.assert_array_equal(g["win_offsets"], wo, err_msg="win_offsets")
    np.testing.assert_array_equal(g["win_tokens"][:len(wt)], wt, err_msg="win_tokens")
    h_k = r.h_win_edges
    v_all = np.diff(wo)
    h_k = np.minimum(h_k, ((v_all + 1) // 2) * (v_all // 2))          # a count above the window's pairs takes them all
    if h_win_edges is None or not host_mirror:
        h_k = np.minimum(h_k, v_all)                                  # counts known to the device only: also at most v_w

    X64, K64, V64 = O.widen(Xs, dtype), O.widen(Ks, dtype), O.widen(Vs, dtype)
    if xi_given is None:
        xi_ref = O.xi_text_query(O.widen(Qs, dtype), K64, h_cu_vis, sched.h_cu_txt, sched.heads, sched.head_dim)
        rel = np.abs(g_xi - xi_ref) / np.maximum(np.abs(xi_ref), 1e-300)
        rep.max_xi_rel = float(rel.max()) if len(rel) else 0.0
        assert rep.max_xi_rel <= (1e-3 if bf16 else 1e-5), "xi relative error %.3g" % rep.max_xi_rel
    else:
        xi_ref = np.asarray(xi_given, dtype=np.float64)

    go, gs = g["grp_offsets"], g["grp_src"]
    assert go[0] == 0 and go[n] == int(h_k.sum()) and np.all(np.diff(go[:n + 1]) >= 0)
    gpu_edges = []
    gone = np.zeros(n, dtype=bool)
    for w in range(len(wo) - 1):
        toks = wt[wo[w]:wo[w + 1]]
        A, Bn = O.split_window(toks)
        k = int(h_k[w])
        assert np.all(go[A + 1] - go[A] == 0), "an A token has sources"
        if len(Bn) == 0:
            assert k == 0 and np.all(g["dst"][toks] == -1)
            continue
        fd = O.feature_divergence(X64[A], X64[Bn], metric)
        scale = 1.0
        fd_cmp = fd
        if metric != "cosine":
            if metric == "euclidean":
                fd_cmp = fd * fd
            scale = float((X64[A] ** 2).sum(axis=1).max() + (X64[Bn] ** 2).sum(axis=1).max())
        band = TIE_BAND * scale
        la_of = {int(t): i for i, t in enumerate(A)}
        mine = []
        for j, b in enumerate(Bn):
            src = gs[go[b]:go[b + 1]]
            assert np.all(np.diff(src) > 0), "sources of token %d are not ascending and distinct" % b
            for a in src:
                assert int(a) in la_of, "source %d of token %d is not an A node of its window" % (a, b)
                mine.append((la_of[int(a)], j))
        assert len(mine) == k, "window %d: %d edges, expected %d" % (w, len(mine), k)
        # the k lowest pairs, ties by (A position, B position): a stable sort of the row-major block
        order = np.argsort(fd.ravel(), kind="stable")[:k]
        ref_set = set((int(e) // len(Bn), int(e) % len(Bn)) for e in order)
        mine_set = set(mine)
        assert len(mine_set) == k, "window %d: an edge is listed twice" % w
        if mine_set != ref_set:
            tau = fd_cmp.ravel()[order[-1]]
            taken = np.zeros(fd.shape, dtype=bool)
            taken[[i for i, _ in mine], [j for _, j in mine]] = True
            assert np.all(fd_cmp[taken] <= tau + band), "window %d: an edge above the threshold %.9g was taken" % (w, tau)
            assert np.all(fd_cmp[~taken] >= tau - band), "window %d: an edge below the threshold %.9g was left out" % (w, tau)
            rep.window_ties += 1
        # dst: the lowest selected edge of every A node that owns one; best_fd / best_dst: its lowest edge of all
        own = {}
        for i, j in mine:
            own.setdefault(i, []).append(j)
        for i, a in enumerate(A):
            if i in own:
                gone[a] = True
                jd = int(np.nonzero(Bn == g["dst"][a])[0][0])
                assert jd in own[i] and fd_cmp[i, jd] <= min(fd_cmp[i, j] for j in own[i]) + band
            else:
                assert g["dst"][a] == -1
            jb = int(np.nonzero(Bn == g["best_dst"][a])[0][0])
            assert fd_cmp[i, jb] <= fd_cmp[i].min() + band
            got = float(g["best_fd"][a]) ** (2 if metric == "euclidean" else 1)
            assert abs(got - fd_cmp[i].min()) / scale <= (1e-5 if bf16 else 1e-6)
        assert np.all(g["dst"][Bn] == -1) and np.all(g["best_dst"][Bn] == -1)
        gpu_edges += [(int(A[i]), int(Bn[j])) for i, j in mine]
        rep.edges += k

    keep = ~gone
    np.testing.assert_array_equal(g["new_index"], np.where(keep, np.cumsum(keep) - 1, -1), err_msg="new_index")
    cu_out = np.zeros(batch + 1, dtype=np.int32)
    for b in range(batch):
        cu_out[b + 1] = cu_out[b] + int(keep[h_cu_vis[b]:h_cu_vis[b + 1]].sum())
    np.testing.assert_array_equal(r.h_cu_vis_out, cu_out, err_msg="cu_vis_out")
    n_out = int(keep.sum())
    np.testing.assert_array_equal(g["pos"], np.asarray(pos)[keep], err_msg="pos_out")
    ego, egs = O.edges_csr(n, gpu_edges)
    np.testing.assert_array_equal(go[:n + 1], ego, err_msg="grp_offsets")
    np.testing.assert_array_equal(gs[:len(egs)], egs, err_msg="grp_src")

    outs = {}
    tol = 2e-2 if bf16 else 1e-5
    for name, Y64, dev_out, src_store in (("X", X64, r.X, Xs), ("K", K64, r.K, Ks), ("V", V64, r.V, Vs)):
        ref = O.message_passing_edges(Y64, xi_ref, gpu_edges)[keep]
        got_store = from_dev(dev_out, dtype)
        got = O.widen(got_store, dtype)
        assert got.shape[0] == n_out
        num = np.linalg.norm(got - ref, axis=1)
        den = np.maximum(np.linalg.norm(ref, axis=1), 1e-300)
        row_rel = float((num / den).max()) if n_out else 0.0
        elem_rel = float((np.abs(got - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-300)).max()) if n_out else 0.0
        rep.max_row_rel = max(rep.max_row_rel, row_rel)
        assert row_rel <= tol and elem_rel <= tol, "%s rows: rel %.3g / %.3g" % (name, row_rel, elem_rel)
        untouched = (ego[1:] - ego[:-1])[keep] == 0
        np.testing.assert_array_equal(got_store[untouched], np.asarray(src_store)[keep][untouched], err_msg=name + " copied rows")
        outs[name] = got_store
    outs["pos"] = g["pos"].copy()
    outs["cu_vis"] = cu_out
    return rep, outs


def check_edge_workload(wl, rho, stages=None, metric="cosine"):
    from paper_2605_00789_amd import EdgeTopKSchedule
    n_st = wl.stages if stages is None else stages
    sched = EdgeTopKSchedule(dtype=wl.dtype, batch=wl.batch, d=wl.d, heads=wl.heads, head_dim=wl.head_dim, tiles=wl.tiles,
                             grid_h=wl.grid_h, grid_w=wl.grid_w, cu_txt=wl.cu_txt,
                             windows_per_axis=wl.windows_per_axis[:n_st], rho=list(rho)[:n_st], metric=metric)
    X, K, V, pos, cu = wl.X, wl.K, wl.V, wl.pos, wl.cu_vis
    reports = []
    for s in range(n_st):
        rep, out = check_edge_step(sched, s, cu, X, K, V, wl.Q, pos, wl.dtype)
        reports.append(rep)
        X, K, V, pos, cu = out["X"], out["K"], out["V"], out["pos"], out["cu_vis"]
    return reports


# ---------------------------------------------------------------------------------------------------------------
# Full pairwise matching (appendix ablation, LIGHTKV_MATCH_FULL_PAIRWISE)
# ---------------------------------------------------------------------------------------------------------------
@dataclass
class PairwiseReport:
    stage: int
    n_in: int
    n_out: int
    tie_rows: int = 0           # tokens whose GPU neighbour differs from the oracle's but ties within the band
    differs_from_oracle_selection: int = 0   # information: tokens decided differently by the all-fp64 selection
    max_xi_rel: float = 0.0
    max_fd_abs: float = 0.0
    max_row_rel: float = 0.0


def check_pairwise_step(sched, s: int, h_cu_vis, Xs, Ks, Vs, Qs, pos, dtype: str, *, xi_given=None, h_win_remove=None):
    """One step of full pairwise matching against the oracle, which gets exactly the tensors the GPU step consumed.
    Scores: every token's nearest-neighbour FD within the stated FD tolerance, its neighbour the oracle's or one that
    ties with it within TIE_BAND.  Selection: the visit is sequential, so a near-tie in the scores may legitimately
    change everything after it; it is therefore checked exactly against the oracle's rule applied to the scores the
    GPU reported (integer work on given keys), and how far the all-fp64 selection differs is reported as information.
    Rows: oracle message passing on the GPU's (verified) selection."""
    batch = sched.batch
    dX, dK, dV = to_dev(Xs, dtype), to_dev(Ks, dtype), to_dev(Vs, dtype)
    dQ = to_dev(Qs, dtype)
    dpos = torch.from_numpy(np.ascontiguousarray(pos, dtype=np.int32)).to(dX.device)
    dxi = None if xi_given is None else torch.from_numpy(np.ascontiguousarray(xi_given, dtype=np.float32)).to(dX.device)
    r = sched.run_step(s, h_cu_vis, dX, dK, dV, dQ, dpos, xi_given=dxi, h_win_edges=h_win_remove)
    torch.cuda.synchronize()
    g = {k: getattr(r, k).cpu().numpy() for k in ("win_offsets", "win_tokens", "best_fd", "best_dst", "dst", "new_index",
                                                  "grp_offsets", "grp_src", "pos")}
    g_xi = r.xi.cpu().numpy()
    bf16 = dtype == "bf16"
    metric = sched.metric
    n = int(h_cu_vis[-1])
    rep = PairwiseReport(stage=s, n_in=n, n_out=int(r.h_cu_vis_out[-1]))

    wo, wt = O.build_windows(pos, h_cu_vis, sched.tiles, sched.grid_h, sched.grid_w, sched.windows_per_axis[s])
    np.testing.assert_array_equal(g["win_offsets"], wo, err_msg="win_offsets")
    np.testing.assert_array_equal(g["win_tokens"][:len(wt)], wt, err_msg="win_tokens")
    rem = O.removal_counts_ratio(wo, sched.rho[s]) if h_win_remove is None else np.asarray(h_win_remove, dtype=np.int32)
    np.testing.assert_array_equal(r.h_win_edges, rem, err_msg="win_remove")

    X64, K64, V64 = O.widen(Xs, dtype), O.widen(Ks, dtype), O.widen(Vs, dtype)
    if xi_given is None:
        xi_ref = O.xi_text_query(O.widen(Qs, dtype), K64, h_cu_vis, sched.h_cu_txt, sched.heads, sched.head_dim)
        rel = np.abs(g_xi - xi_ref) / np.maximum(np.abs(xi_ref), 1e-300)
        rep.max_xi_rel = float(rel.max()) if len(rel) else 0.0
        assert rep.max_xi_rel <= (1e-3 if bf16 else 1e-5), "xi relative error %.3g" % rep.max_xi_rel
    else:
        xi_ref = np.asarray(xi_given, dtype=np.float64)

    # ---- scores
    for w in range(len(wo) - 1):
        toks = wt[wo[w]:wo[w + 1]]
        if len(toks) < 2:
            assert np.all(g["best_dst"][toks] == -1) and np.all(np.isinf(g["best_fd"][toks]))
            continue
        fd = O.feature_divergence(X64[toks], X64[toks], metric)
        np.fill_diagonal(fd, np.inf)
        g_fd = g["best_fd"][toks].astype(np.float64)
        scale = 1.0
        if metric != "cosine":
            if metric == "euclidean":
                fd, g_fd = fd * fd, g_fd * g_fd
            scale = 2.0 * float((X64[toks] ** 2).sum(axis=1).max())
        band = TIE_BAND * scale
        j_ref = np.argmin(fd, axis=1)
        f_ref = fd[np.arange(len(toks)), j_ref]
        local = {int(t): k for k, t in enumerate(toks)}
        b_gpu = g["best_dst"][toks]
        for l in np.nonzero(b_gpu != toks[j_ref])[0]:
            assert int(b_gpu[l]) in local and int(b_gpu[l]) != int(toks[l]), "neighbour of token %d is not another token of its window" % toks[l]
            f_g = fd[l, local[int(b_gpu[l])]]
            assert f_g <= f_ref[l] + band, "window %d token %d: neighbour FD %.9g vs best %.9g" % (w, toks[l], f_g, f_ref[l])
            rep.tie_rows += 1
        rep.max_fd_abs = max(rep.max_fd_abs, float((np.abs(g_fd - f_ref) / scale).max()))
    assert rep.max_fd_abs <= (1e-5 if bf16 else 1e-6), "nearest-neighbour FD abs error %.3g" % rep.max_fd_abs

    # ---- selection: the oracle's visit on the scores the GPU reported -> exact
    dst = g["dst"]
    want = O.select_full_pairwise(g["best_fd"].astype(np.float64), g["best_dst"], wo, wt, rem)
    np.testing.assert_array_equal(dst, want, err_msg="dst")
    nf, nd = O.nearest_neighbours(X64, wo, wt, metric)
    rep.differs_from_oracle_selection = int((O.select_full_pairwise(nf, nd, wo, wt, rem) != dst).sum())
    gone = dst >= 0
    assert not gone[dst[gone]].any(), "a destination was merged away"
    for w in range(len(wo) - 1):
        toks = wt[wo[w]:wo[w + 1]]
        assert int(gone[toks].sum()) <= int(rem[w])

    # ---- index structures follow from dst: exact
    np.testing.assert_array_equal(g["new_index"], O.kept_index(dst), err_msg="new_index")
    go, gs = O.groups_csr(dst)
    np.testing.assert_array_equal(g["grp_offsets"][:n + 1], go, err_msg="grp_offsets")
    np.testing.assert_array_equal(g["grp_src"][:len(gs)], gs, err_msg="grp_src")
    keep = ~gone
    cu_out = np.zeros(batch + 1, dtype=np.int32)
    for b in range(batch):
        cu_out[b + 1] = cu_out[b] + int(keep[h_cu_vis[b]:h_cu_vis[b + 1]].sum())
    np.testing.assert_array_equal(r.h_cu_vis_out, cu_out, err_msg="cu_vis_out")
    n_out = int(keep.sum())
    np.testing.assert_array_equal(g["pos"], np.asarray(pos)[keep], err_msg="pos_out")

    outs = {}
    tol = 2e-2 if bf16 else 1e-5
    for name, Y64, dev_out, src_store in (("X", X64, r.X, Xs), ("K", K64, r.K, Ks), ("V", V64, r.V, Vs)):
        ref = O.compact(O.message_passing(Y64, xi_ref, dst), dst)
        got_store = from_dev(dev_out, dtype)
        got = O.widen(got_store, dtype)
        assert got.shape[0] == n_out
        num = np.linalg.norm(got - ref, axis=1)
        den = np.maximum(np.linalg.norm(ref, axis=1), 1e-300)
        row_rel = float((num / den).max()) if n_out else 0.0
        elem_rel = float((np.abs(got - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-300)).max()) if n_out else 0.0
        rep.max_row_rel = max(rep.max_row_rel, row_rel)
        assert row_rel <= tol and elem_rel <= tol, "%s rows: rel %.3g / %.3g" % (name, row_rel, elem_rel)
        untouched = (go[1:] - go[:-1])[keep] == 0
        np.testing.assert_array_equal(got_store[untouched], np.asarray(src_store)[keep][untouched], err_msg=name + " copied rows")
        outs[name] = got_store
    outs["pos"] = g["pos"].copy()
    outs["cu_vis"] = cu_out
    return rep, outs


def check_pairwise_workload(wl, rho, stages=None, metric="cosine"):
    from paper_2605_00789_amd import EdgeTopKSchedule
    n_st = wl.stages if stages is None else stages
    sched = EdgeTopKSchedule(dtype=wl.dtype, batch=wl.batch, d=wl.d, heads=wl.heads, head_dim=wl.head_dim, tiles=wl.tiles,
                             grid_h=wl.grid_h, grid_w=wl.grid_w, cu_txt=wl.cu_txt,
                             windows_per_axis=wl.windows_per_axis[:n_st], rho=list(rho)[:n_st], metric=metric,
                             match="full_pairwise")
    X, K, V, pos, cu = wl.X, wl.K, wl.V, wl.pos, wl.cu_vis
    reports = []
    for s in range(n_st):
        rep, out = check_pairwise_step(sched, s, cu, X, K, V, wl.Q, pos, wl.dtype)
        reports.append(rep)
        X, K, V, pos, cu = out["X"], out["K"], out["V"], out["pos"], out["cu_vis"]
    return reports
