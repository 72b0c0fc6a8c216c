"""ctypes binding of liblightkv.so: same names as the C ABI (include/lightkv.h),
argument marshalling only.  torch tensors supply device memory and the stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

XI_TEXT_QUERY, XI_VISION_QUERY, XI_GIVEN = 0, 1, 2
F32, BF16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "liblightkv.so")


class LightKVError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: status %d (%s)" % (where, status, lightkv_status_string(status)))


class _CProblem(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("d", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32),
        ("dtype", C.c_int32), ("n_windows", C.c_int32), ("max_window_tokens", C.c_int32), ("metric", C.c_int32),
        ("match", C.c_int32), ("direction", C.c_int32),
        ("h_cu_vis", C.c_void_p), ("h_cu_txt", C.c_void_p), ("cu_vis", C.c_void_p), ("cu_txt", C.c_void_p),
        ("win_offsets", C.c_void_p), ("win_tokens", C.c_void_p), ("win_remove", C.c_void_p),
        ("h_win_offsets", C.c_void_p), ("h_win_remove", C.c_void_p),
    ]


class _CStage(C.Structure):
    _fields_ = [
        ("problem", _CProblem), ("w", C.c_int32), ("reserved", C.c_int32),
        ("win_offsets", C.c_void_p), ("win_tokens", C.c_void_p), ("xi", C.c_void_p), ("best_fd", C.c_void_p),
        ("best_dst", C.c_void_p), ("dst", C.c_void_p), ("new_index", C.c_void_p), ("grp_offsets", C.c_void_p),
        ("grp_src", C.c_void_p), ("cu_vis_out", C.c_void_p), ("X_out", C.c_void_p), ("K_out", C.c_void_p),
        ("V_out", C.c_void_p), ("pos_out", C.c_void_p), ("x_sqnorm_out", C.c_void_p), ("out_rows", C.c_int64),
        ("cu_vis_target", C.c_void_p), ("win_remove", C.c_void_p), ("status", C.c_void_p),
    ]


def _load():
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(
            "liblightkv.so is not built (%s). Run `python -c 'import __graft_entry__ as g; g.build()'` "
            "or `python paper_2605_00789_amd/build.py`; there is no fallback path." % path)
    lib = C.CDLL(path)
    P = C.POINTER(_CProblem)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    lib.lightkv_status_string.restype = C.c_char_p
    lib.lightkv_status_string.argtypes = [C.c_int]
    lib.lightkv_version.restype = C.c_int
    lib.lightkv_version.argtypes = []
    lib.lightkv_workspace_size.restype = C.c_int
    lib.lightkv_workspace_size.argtypes = [P, C.POINTER(sz)]
    lib.lightkv_build_windows.restype = C.c_int
    lib.lightkv_build_windows.argtypes = [i32, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
    lib.lightkv_build_windows_next.restype = C.c_int
    lib.lightkv_build_windows_next.argtypes = [i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
    lib.lightkv_score.restype = C.c_int
    lib.lightkv_score.argtypes = [P, vp, i64, vp, vp, i64, i64, vp, i64, i64, i32, vp, f32, vp, vp, vp, vp, i64, vp, sz, vp]
    lib.lightkv_score_select.restype = C.c_int
    lib.lightkv_score_select.argtypes = [P, vp, i64, vp, vp, i64, i64, vp, i64, i64, i32, vp, f32, vp, vp, vp,
                                         vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lightkv_select.restype = C.c_int
    lib.lightkv_select.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lightkv_windows_per_sequence.restype = C.c_int32
    lib.lightkv_windows_per_sequence.argtypes = [i32, i32]
    lib.lightkv_max_window_cells.restype = C.c_int32
    lib.lightkv_max_window_cells.argtypes = [i32, i32, i32, i32]
    lib.lightkv_window_counts.restype = C.c_int
    lib.lightkv_window_counts.argtypes = [i32, i32, vp, i32, i32, C.c_double, vp, vp, vp, vp, vp]
    lib.lightkv_select_static.restype = C.c_int
    lib.lightkv_select_static.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.lightkv_aggregate.restype = C.c_int
    lib.lightkv_aggregate.argtypes = [P, vp, vp, vp, vp, i64, vp, i64, vp, i64, vp]
    lib.lightkv_compact.restype = C.c_int
    lib.lightkv_compact.argtypes = [P, vp, vp, i64, vp, i64, vp, i64, vp, vp, vp, vp, vp, vp, i64, i64, vp, vp]
    lib.lightkv_aggregate_compact.restype = C.c_int
    lib.lightkv_aggregate_compact.argtypes = [P, vp, vp, vp, vp, vp, i64, vp, i64, vp, i64, vp, vp, vp, vp, vp, vp, i64, i64, vp, vp]
    lib.lightkv_compress_schedule.restype = C.c_int
    lib.lightkv_compress_schedule.argtypes = [C.POINTER(_CStage), i32, i32, i32, i32, vp, i64, vp, i64, vp, i64, vp,
                                              vp, i64, i64, f32, vp, sz, vp]
    lib.lightkv_compress_schedule_ratio.restype = C.c_int
    lib.lightkv_compress_schedule_ratio.argtypes = [C.POINTER(_CStage), i32, C.POINTER(C.c_double), i32, i32, i32, vp, i64,
                                                    vp, i64, vp, i64, vp, vp, i64, i64, f32, vp, sz, vp, vp]
    return lib


_lib = _load()

EXPORTS = ("lightkv_status_string", "lightkv_version", "lightkv_workspace_size", "lightkv_build_windows", "lightkv_compress_schedule",
           "lightkv_compress_schedule_ratio",
           "lightkv_build_windows_next", "lightkv_windows_per_sequence", "lightkv_max_window_cells", "lightkv_window_counts",
           "lightkv_score", "lightkv_score_select", "lightkv_select", "lightkv_select_static", "lightkv_aggregate", "lightkv_compact", "lightkv_aggregate_compact")


def _dptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    return C.c_void_p(t.data_ptr())


def _hptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    if a.dtype != np.int32 or not a.flags["C_CONTIGUOUS"]:
        raise ValueError("host arrays must be contiguous int32")
    return C.c_void_p(a.ctypes.data)


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise LightKVError(status, where)


def _out_rows(*outs) -> int:
    rows = [int(t.shape[0]) for t in outs if t is not None]
    return min(rows) if rows else 0


def _ld(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else int(t.stride(0))


METRICS = {"cosine": 0, "euclidean": 1, "l2sq": 2}
MATCH_BEST_PER_A, MATCH_EDGE_TOPK, MATCH_FULL_PAIRWISE = 0, 1, 2
DIRECTION_A_TO_B, DIRECTION_B_TO_A = 0, 1   # lightkv_direction
EDGE_MAX_WINDOW_TOKENS = 4096   # LIGHTKV_EDGE_MAX_WINDOW_TOKENS
SELECT_STATIC_MAX_TOKENS = 65536   # LIGHTKV_SELECT_STATIC_MAX_TOKENS
ONE_STREAM_MAX_TOKENS = 1024   # LIGHTKV_ONE_STREAM_MAX_TOKENS


class Problem:
    """Python mirror of `lightkv_problem`; keeps the host arrays and device tensors it points to alive."""

    def __init__(self, *, batch, d, heads, head_dim, dtype, h_cu_vis, cu_vis, h_cu_txt=None, cu_txt=None,
                 n_windows=0, max_window_tokens=0, win_offsets=None, win_tokens=None, win_remove=None,
                 h_win_offsets=None, h_win_remove=None, metric="cosine", match=MATCH_BEST_PER_A,
                 direction=DIRECTION_A_TO_B):
        self.refs = dict(h_cu_vis=h_cu_vis, cu_vis=cu_vis, h_cu_txt=h_cu_txt, cu_txt=cu_txt,
                         win_offsets=win_offsets, win_tokens=win_tokens, win_remove=win_remove,
                         h_win_offsets=h_win_offsets, h_win_remove=h_win_remove)
        self.c = _CProblem()
        self.c.batch, self.c.d, self.c.heads, self.c.head_dim = batch, d, heads, head_dim
        self.c.dtype = {"f32": F32, "bf16": BF16, F32: F32, BF16: BF16}[dtype]
        self.c.n_windows, self.c.max_window_tokens = n_windows, max_window_tokens
        self.c.metric = METRICS[metric] if isinstance(metric, str) else int(metric)
        self.c.match, self.c.direction = int(match), int(direction)
        for name in ("h_cu_vis", "h_cu_txt", "h_win_offsets", "h_win_remove"):
            setattr(self.c, name, _hptr(self.refs[name]))
        for name in ("cu_vis", "cu_txt", "win_offsets", "win_tokens", "win_remove"):
            setattr(self.c, name, _dptr(self.refs[name]))

    def ref(self):
        return C.byref(self.c)


def lightkv_status_string(status: int) -> str:
    return _lib.lightkv_status_string(int(status)).decode()


def lightkv_version() -> int:
    return int(_lib.lightkv_version())


def lightkv_workspace_size(p: Problem) -> int:
    out = C.c_size_t(0)
    _check(_lib.lightkv_workspace_size(p.ref(), C.byref(out)), "lightkv_workspace_size")
    return int(out.value)


def lightkv_build_windows(batch, h_cu_vis, cu_vis, pos, tiles, grid_h, grid_w, w, win_offsets, win_tokens,
                          stream=None):
    _check(_lib.lightkv_build_windows(batch, _hptr(h_cu_vis), _dptr(cu_vis), _dptr(pos), tiles, grid_h, grid_w, w,
                                      _dptr(win_offsets), _dptr(win_tokens), _stream(stream)),
           "lightkv_build_windows")


def lightkv_build_windows_next(batch, h_cu_vis, cu_vis, pos, new_index, cu_vis_out, tiles, grid_h, grid_w, w,
                               win_offsets, win_tokens, stream=None):
    _check(_lib.lightkv_build_windows_next(batch, _hptr(h_cu_vis), _dptr(cu_vis), _dptr(pos), _dptr(new_index),
                                           _dptr(cu_vis_out), tiles, grid_h, grid_w, w, _dptr(win_offsets),
                                           _dptr(win_tokens), _stream(stream)), "lightkv_build_windows_next")


COUNT_RATIO, COUNT_EDGES, COUNT_TARGET = 0, 1, 2


def lightkv_windows_per_sequence(tiles: int, w: int) -> int:
    n = int(_lib.lightkv_windows_per_sequence(tiles, w))
    if n < 0:
        raise ValueError("invalid tiles / w")
    return n


def lightkv_max_window_cells(tiles: int, grid_h: int, grid_w: int, w: int) -> int:
    n = int(_lib.lightkv_max_window_cells(tiles, grid_h, grid_w, w))
    if n < 0:
        raise ValueError("invalid grid")
    return n


def lightkv_window_counts(batch, n_windows, win_offsets, mode, win_remove, *, direction=DIRECTION_A_TO_B, rho=0.0,
                          cu_vis=None, cu_vis_target=None, status=None, stream=None):
    _check(_lib.lightkv_window_counts(batch, n_windows, _dptr(win_offsets), int(mode), int(direction), float(rho), _dptr(cu_vis),
                                      _dptr(cu_vis_target), _dptr(win_remove), _dptr(status), _stream(stream)),
           "lightkv_window_counts")


def lightkv_score(p: Problem, X, Q, K, xi, best_fd, best_dst, ws, *, heads_major=False, xi_mode=XI_TEXT_QUERY,
                  lse=None, softmax_scale=0.0, x_sqnorm=None, fd_dump=None, stream=None):
    """X [sumN, d]; Q, K token-major [tokens, heads*head_dim] (or [heads, tokens, head_dim] with heads_major);
    x_sqnorm: optional fp32 [sumN], |x|^2 of the rows of X (from lightkv_compact / lightkv_aggregate_compact)."""
    hd = p.c.head_dim

    def strides(t):
        if t is None:
            return 0, 0
        if heads_major:
            return int(t.stride(1)), int(t.stride(0))
        return int(t.stride(0)), hd

    qts, qhs = strides(Q)
    kts, khs = strides(K)
    _check(_lib.lightkv_score(p.ref(), _dptr(X), _ld(X), _dptr(x_sqnorm), _dptr(Q), qts, qhs, _dptr(K), kts, khs, xi_mode,
                              _dptr(lse), float(softmax_scale), _dptr(xi), _dptr(best_fd), _dptr(best_dst),
                              _dptr(fd_dump), 0 if fd_dump is None else fd_dump.numel(),
                              _dptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "lightkv_score")


def lightkv_score_select(p: Problem, X, Q, K, xi, best_fd, best_dst, dst, new_index, grp_offsets, grp_src, cu_vis_out,
                         ws, *, heads_major=False, xi_mode=XI_TEXT_QUERY, lse=None, softmax_scale=0.0, x_sqnorm=None,
                         stream=None):
    hd = p.c.head_dim

    def strides(t):
        if t is None:
            return 0, 0
        if heads_major:
            return int(t.stride(1)), int(t.stride(0))
        return int(t.stride(0)), hd

    qts, qhs = strides(Q)
    kts, khs = strides(K)
    if p.c.match == MATCH_EDGE_TOPK:
        # the C call takes plain pointers: the one size the library cannot check is checked here.  With the host's
        # counts the group list holds one entry per edge, without them at most one per token of the batch.
        h_k, h_cu = p.refs.get("h_win_remove"), p.refs["h_cu_vis"]
        need = int(np.asarray(h_k, dtype=np.int64).sum()) if h_k is not None else int(h_cu[-1])
        if grp_src.numel() < need:
            raise ValueError("grp_src holds %d entries, this step may write %d" % (grp_src.numel(), need))
    _check(_lib.lightkv_score_select(p.ref(), _dptr(X), _ld(X), _dptr(x_sqnorm), _dptr(Q), qts, qhs, _dptr(K), kts, khs, xi_mode,
                                     _dptr(lse), float(softmax_scale), _dptr(xi), _dptr(best_fd), _dptr(best_dst),
                                     _dptr(dst), _dptr(new_index), _dptr(grp_offsets), _dptr(grp_src),
                                     _dptr(cu_vis_out), _dptr(ws), ws.numel() * ws.element_size(), _stream(stream)),
           "lightkv_score_select")


def lightkv_select(p: Problem, best_fd, best_dst, dst, new_index, grp_offsets, grp_src, cu_vis_out, ws, stream=None):
    _check(_lib.lightkv_select(p.ref(), _dptr(best_fd), _dptr(best_dst), _dptr(dst), _dptr(new_index),
                               _dptr(grp_offsets), _dptr(grp_src), _dptr(cu_vis_out), _dptr(ws),
                               ws.numel() * ws.element_size(), _stream(stream)), "lightkv_select")


def lightkv_select_static(p: Problem, best_fd, best_dst, dst, new_index, grp_offsets, grp_src, cu_vis_out, stream=None):
    _check(_lib.lightkv_select_static(p.ref(), _dptr(best_fd), _dptr(best_dst), _dptr(dst), _dptr(new_index),
                                      _dptr(grp_offsets), _dptr(grp_src), _dptr(cu_vis_out), _stream(stream)),
           "lightkv_select_static")


def lightkv_aggregate(p: Problem, grp_offsets, grp_src, xi, X, K, V, stream=None):
    _check(_lib.lightkv_aggregate(p.ref(), _dptr(grp_offsets), _dptr(grp_src), _dptr(xi), _dptr(X), _ld(X),
                                  _dptr(K), _ld(K), _dptr(V), _ld(V), _stream(stream)), "lightkv_aggregate")


def lightkv_compact(p: Problem, new_index, X, K, V, pos, X_out, K_out, V_out, pos_out, x_sqnorm_out=None, tail_rows=0,
                    cu_vis_out=None, stream=None):
    _check(_lib.lightkv_compact(p.ref(), _dptr(new_index), _dptr(X), _ld(X), _dptr(K), _ld(K), _dptr(V), _ld(V),
                                _dptr(pos), _dptr(X_out), _dptr(K_out), _dptr(V_out), _dptr(pos_out),
                                _dptr(x_sqnorm_out), _out_rows(X_out, K_out, V_out, pos_out), int(tail_rows),
                                _dptr(cu_vis_out), _stream(stream)),
           "lightkv_compact")


def lightkv_aggregate_compact(p: Problem, new_index, grp_offsets, grp_src, xi, X, K, V, pos, X_out, K_out, V_out,
                              pos_out, x_sqnorm_out=None, tail_rows=0, cu_vis_out=None, stream=None):
    _check(_lib.lightkv_aggregate_compact(p.ref(), _dptr(new_index), _dptr(grp_offsets), _dptr(grp_src), _dptr(xi),
                                          _dptr(X), _ld(X), _dptr(K), _ld(K), _dptr(V), _ld(V), _dptr(pos),
                                          _dptr(X_out), _dptr(K_out), _dptr(V_out), _dptr(pos_out),
                                          _dptr(x_sqnorm_out), _out_rows(X_out, K_out, V_out, pos_out),
                                          int(tail_rows), _dptr(cu_vis_out), _stream(stream)),
           "lightkv_aggregate_compact")


class StageArray:
    """A C array of `lightkv_stage` built from Problems and the stages' tensors; keeps everything it points to alive."""

    def __init__(self, stages):
        """stages: sequence of dicts with keys problem (Problem), w and the tensors named in lightkv_stage."""
        self.keep = list(stages)
        self.n = len(self.keep)
        self.c = (_CStage * self.n)()
        for i, st in enumerate(self.keep):
            c = self.c[i]
            C.memmove(C.byref(c.problem), C.byref(st["problem"].c), C.sizeof(_CProblem))
            c.w, c.reserved = int(st["w"]), 0
            for name in ("win_offsets", "win_tokens", "xi", "best_fd", "best_dst", "dst", "new_index", "grp_offsets",
                         "grp_src", "cu_vis_out", "X_out", "K_out", "V_out", "pos_out", "x_sqnorm_out", "cu_vis_target",
                         "win_remove", "status"):
                t = st.get(name)
                setattr(c, name, None if t is None else t.data_ptr())
            c.out_rows = _out_rows(st["X_out"], st["K_out"], st["V_out"], st["pos_out"])


def lightkv_compress_schedule(stages: StageArray, tiles, grid_h, grid_w, X, K, V, pos, Q, ws, *, softmax_scale=0.0,
                              stream=None):
    """All stages of a schedule in one call; X, K, V [sumN, d], Q [sumT, heads*head_dim] token-major."""
    hd = stages.keep[0]["problem"].c.head_dim
    _check(_lib.lightkv_compress_schedule(stages.c, stages.n, tiles, grid_h, grid_w, _dptr(X), _ld(X), _dptr(K), _ld(K),
                                          _dptr(V), _ld(V), _dptr(pos), _dptr(Q), int(Q.stride(0)), hd,
                                          float(softmax_scale), _dptr(ws), ws.numel() * ws.element_size(),
                                          _stream(stream)), "lightkv_compress_schedule")


def lightkv_compress_schedule_ratio(stages: StageArray, rho, tiles, grid_h, grid_w, X, K, V, pos, Q, ws, *,
                                    softmax_scale=0.0, stream=None) -> np.ndarray:
    """All stages of a schedule whose token counts depend on the data, in one call (it waits for the stream once per
    stage).  rho: one ratio per stage.  Returns the [n_stages, batch + 1] sequence offsets the stages left (host)."""
    prob = stages.keep[0]["problem"].c
    if len(rho) != stages.n:
        raise ValueError("one ratio per stage")
    rho_c = (C.c_double * stages.n)(*[float(r) for r in rho])
    h_out = np.zeros((stages.n, prob.batch + 1), dtype=np.int32)
    _check(_lib.lightkv_compress_schedule_ratio(stages.c, stages.n, rho_c, tiles, grid_h, grid_w, _dptr(X), _ld(X),
                                                _dptr(K), _ld(K), _dptr(V), _ld(V), _dptr(pos), _dptr(Q),
                                                int(Q.stride(0)), prob.head_dim, float(softmax_scale), _dptr(ws),
                                                ws.numel() * ws.element_size(), h_out.ctypes.data_as(C.c_void_p),
                                                _stream(stream)), "lightkv_compress_schedule_ratio")
    return h_out
