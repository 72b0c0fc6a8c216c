"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments before anything is launched (no GPU needed: validation happens on the host)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2605_00789_amd import binding
    return binding


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "lightkv.h")).read()
    declared = set(re.findall(r"^(?:const char \*|int |int32_t |lightkv_status )(lightkv_[a-z_]+)\(", header, re.M))
    assert declared == set(B.EXPORTS)
    lib = C.CDLL(B.lib_path())
    for name in declared:
        assert hasattr(lib, name), name
    assert B.lightkv_version() >= 100
    assert B.lightkv_status_string(0) == "ok"
    assert "half" not in B.lightkv_status_string(4) and "set A" in B.lightkv_status_string(4)
    assert B.lightkv_status_string(99) == "unknown status"


def _problem(B, **over):
    """A descriptor whose device pointers are fake but non-NULL: only host-side validation may touch it."""
    fake = 0x1000
    h_cu_vis = np.array([0, 8], dtype=np.int32)
    h_cu_txt = np.array([0, 4], dtype=np.int32)
    h_wo = np.array([0, 4, 8], dtype=np.int32)
    h_wr = np.array([1, 2], dtype=np.int32)
    p = B._CProblem()
    p.batch, p.d, p.heads, p.head_dim, p.dtype, p.n_windows, p.max_window_tokens = 1, 64, 2, 32, 1, 2, 0
    keep = dict(h_cu_vis=h_cu_vis, h_cu_txt=h_cu_txt, h_win_offsets=h_wo, h_win_remove=h_wr)
    for k, v in over.items():
        if isinstance(v, np.ndarray):
            keep[k] = v
    for k in ("h_cu_vis", "h_cu_txt", "h_win_offsets", "h_win_remove"):
        setattr(p, k, C.c_void_p(keep[k].ctypes.data))
    for k in ("cu_vis", "cu_txt", "win_offsets", "win_tokens", "win_remove"):
        setattr(p, k, C.c_void_p(fake))
    for k, v in over.items():
        if not isinstance(v, np.ndarray):
            setattr(p, k, v)
    p._keep = keep
    return p


def _ws_size(B, p):
    out = C.c_size_t(0)
    st = B._lib.lightkv_workspace_size(C.byref(p), C.byref(out))
    return st, out.value


def test_workspace_size_and_descriptor_validation(B):
    st, n = _ws_size(B, _problem(B))
    assert st == 0 and n > 0 and n % 256 == 0
    assert B._lib.lightkv_workspace_size(None, C.byref(C.c_size_t(0))) == 1
    assert B._lib.lightkv_workspace_size(C.byref(_problem(B)), None) == 1
    assert _ws_size(B, _problem(B, h_cu_vis=None))[0] == 1                      # NULL
    assert _ws_size(B, _problem(B, d=60))[0] == 5                               # 16-byte rows
    assert _ws_size(B, _problem(B, heads=3))[0] == 2                            # heads*head_dim != d
    assert _ws_size(B, _problem(B, d=96, heads=2, head_dim=48))[0] == 5         # head size
    assert _ws_size(B, _problem(B, dtype=7))[0] == 5
    assert _ws_size(B, _problem(B, metric=2))[0] == 0 and _ws_size(B, _problem(B, metric=3))[0] == 5   # lightkv_metric
    assert _ws_size(B, _problem(B, metric=-1))[0] == 5
    # lightkv_match: the k lowest edges need the host's counts, count pairs instead of A nodes, and bound the window
    assert _ws_size(B, _problem(B, match=3))[0] == 5 and _ws_size(B, _problem(B, match=-1))[0] == 5
    # full pairwise matching: bf16 rows of whole 64-element k-steps only
    assert _ws_size(B, _problem(B, match=2))[0] == 0
    assert _ws_size(B, _problem(B, match=2, dtype=0))[0] == 5
    assert _ws_size(B, _problem(B, match=2, d=96, heads=3))[0] == 5
    # lightkv_direction: the reverse direction exists for one proposal per node only
    assert _ws_size(B, _problem(B, direction=1))[0] == 0
    assert _ws_size(B, _problem(B, direction=2))[0] == 5 and _ws_size(B, _problem(B, direction=-1))[0] == 5
    assert _ws_size(B, _problem(B, direction=1, match=2))[0] == 5
    assert _ws_size(B, _problem(B, direction=1, match=1, h_win_remove=np.array([1, 1], dtype=np.int32)))[0] == 5
    st_e, n_e = _ws_size(B, _problem(B, match=1, h_win_remove=np.array([4, 3], dtype=np.int32)))   # 2 x 2 pairs per window
    assert st_e == 0 and n_e >= _ws_size(B, _problem(B))[1]
    assert _ws_size(B, _problem(B, match=0, h_win_remove=np.array([4, 3], dtype=np.int32)))[0] == 4   # more than |A| = 2
    assert _ws_size(B, _problem(B, match=1, h_win_remove=np.array([5, 0], dtype=np.int32)))[0] == 4   # more than 4 pairs
    p_nohost = _problem(B, match=1)                          # counts on the device only: one slot per token instead
    p_nohost.h_win_remove = None
    assert _ws_size(B, p_nohost)[0] == 0
    p_half = _problem(B, match=1, max_window_tokens=4)       # host counts cannot be validated without host window sizes
    p_half.h_win_offsets = None
    assert _ws_size(B, p_half)[0] == 1
    big = np.array([0, 300], dtype=np.int32)                 # a 300-token window: the keys of its 150 x 150 pairs are in the workspace
    st_b, n_b = _ws_size(B, _problem(B, match=1, n_windows=1, h_cu_vis=big, h_win_offsets=big, h_win_remove=np.array([1], dtype=np.int32)))
    assert st_b == 0 and n_b > 150 * 150 * 4
    assert _ws_size(B, _problem(B, batch=0))[0] == 2
    assert _ws_size(B, _problem(B, h_cu_vis=np.array([1, 8], dtype=np.int32)))[0] == 2
    assert _ws_size(B, _problem(B, h_cu_vis=np.array([0, 20000], dtype=np.int32),
                                h_win_offsets=np.array([0, 4, 20000], dtype=np.int32)))[0] == 5   # sequence limit
    assert _ws_size(B, _problem(B, h_win_offsets=np.array([0, 5, 7], dtype=np.int32)))[0] == 3    # not a partition
    assert _ws_size(B, _problem(B, h_win_offsets=np.array([0, 6, 4], dtype=np.int32)))[0] == 3
    assert _ws_size(B, _problem(B, h_win_offsets=np.array([1, 4, 8], dtype=np.int32)))[0] == 3
    assert _ws_size(B, _problem(B, max_window_tokens=3))[0] == 3                # bound below the real size
    assert _ws_size(B, _problem(B, h_win_remove=np.array([3, 0], dtype=np.int32)))[0] == 4        # r > |A|
    assert _ws_size(B, _problem(B, h_win_remove=np.array([-1, 0], dtype=np.int32)))[0] == 4
    assert _ws_size(B, _problem(B, h_win_remove=np.array([2, 2], dtype=np.int32)))[0] == 0        # r = |A| is the limit
    # no host mirror: the bound becomes mandatory
    assert _ws_size(B, _problem(B, h_win_offsets=None))[0] == 1
    assert _ws_size(B, _problem(B, h_win_offsets=None, max_window_tokens=4))[0] == 0
    assert _ws_size(B, _problem(B, h_win_offsets=None, max_window_tokens=5000))[0] == 5
    # a one-token window cannot give up its token
    assert _ws_size(B, _problem(B, h_win_offsets=np.array([0, 1, 8], dtype=np.int32),
                                h_win_remove=np.array([1, 0], dtype=np.int32)))[0] == 4


def test_entry_points_reject_bad_arguments_before_launch(B):
    lib = B._lib
    fake = C.c_void_p(0x1000)
    p = _problem(B)
    _, ws = _ws_size(B, p)
    # score: NULL outputs, misaligned X, short row stride, bad mode, missing workspace
    args = lambda **o: [o.get("p", C.byref(p)), o.get("X", fake), o.get("ldx", 64), o.get("sq", None), fake, 64, 32, fake, 64, 32,
                        o.get("mode", 0), o.get("lse", None), 0.0, o.get("xi", fake), fake, fake,
                        o.get("dump", None), o.get("dumpn", 0), o.get("ws", fake), o.get("wsb", ws), None]
    assert lib.lightkv_score(*args(xi=None)) == 1
    assert lib.lightkv_score(*args(X=C.c_void_p(0x1008))) == 5
    assert lib.lightkv_score(*args(ldx=32)) == 2
    assert lib.lightkv_score(*args(ldx=68)) == 5
    assert lib.lightkv_score(*args(sq=C.c_void_p(0x1002))) == 5                  # misaligned squared norms
    assert lib.lightkv_score(*args(mode=3)) == 5
    assert lib.lightkv_score(*args(mode=1)) == 1                                 # vision-query needs lse
    assert lib.lightkv_score(*args(ws=None)) == 6
    assert lib.lightkv_score(*args(wsb=ws - 1)) == 6
    assert lib.lightkv_score(*args(ws=C.c_void_p(0x1010))) == 6                  # workspace alignment
    assert lib.lightkv_score(*args(dump=fake, dumpn=-1)) == 2                    # FD dump: negative capacity
    assert lib.lightkv_score(*args(dump=C.c_void_p(0x1002), dumpn=64)) == 5     # ... misaligned
    assert lib.lightkv_score(*args(dump=fake, dumpn=64, X=None)) == 1           # ... needs the FD half
    # score_select: the union of both argument lists
    ss = lambda **o: [C.byref(p), o.get("X", fake), 64, None, fake, 64, 32, fake, 64, 32, 0, None, 0.0, fake, fake, fake,
                      o.get("dst", fake), fake, fake, fake, fake, o.get("ws", fake), o.get("wsb", ws), None]
    assert lib.lightkv_score_select(*ss(X=None)) == 1
    assert lib.lightkv_score_select(*ss(dst=None)) == 1
    assert lib.lightkv_score_select(*ss(wsb=8)) == 6
    # select
    assert lib.lightkv_select(C.byref(p), fake, fake, None, fake, fake, fake, fake, fake, ws, None) == 1
    assert lib.lightkv_select(C.byref(p), fake, fake, fake, fake, fake, fake, fake, fake, 16, None) == 6
    # the k lowest edges cannot be chosen from per-node scores: only lightkv_score_select takes that reading
    pe = _problem(B, match=1)
    assert lib.lightkv_select(C.byref(pe), fake, fake, fake, fake, fake, fake, fake, fake, ws, None) == 5
    # the schedule driver validates every stage before it enqueues anything
    sched = lib.lightkv_compress_schedule
    stage = B._CStage()
    C.memmove(C.byref(stage.problem), C.byref(p), C.sizeof(B._CProblem))
    for name in ("win_offsets", "win_tokens", "xi", "best_fd", "best_dst", "dst", "new_index", "grp_offsets", "grp_src",
                 "cu_vis_out", "X_out", "K_out", "V_out", "pos_out"):
        setattr(stage, name, 0x1000)
    stage.out_rows = 5

    def sc(stages=None, n=1, X=fake, Q=fake, wsb=1 << 30):
        arr = (B._CStage * 1)(stage) if stages is None else stages
        return sched(arr, n, 1, 2, 4, X, 64, fake, 64, fake, 64, fake, Q, 64, 32, 0.0, fake, wsb, None)

    assert sched(None, 1, 1, 2, 4, fake, 64, fake, 64, fake, 64, fake, fake, 64, 32, 0.0, fake, 1 << 30, None) == 1
    assert sc(n=0) == 2 and sc(X=None) == 1 and sc(Q=None) == 1
    assert sc(wsb=16) == 6
    stage.xi = None
    assert sc() == 1
    stage.xi = 0x1000
    stage.win_tokens = 0x2000                      # not the array the descriptor points to
    assert sc() == 2
    stage.win_tokens = 0x1000
    stage.problem.match = 1                        # data-dependent token counts: not in a fixed schedule
    assert sc() == 5
    stage.problem.match = 0
    stage.reserved = 3
    assert sc() == 5
    stage.reserved = 0
    # the ratio-driven schedule: same validation before anything is enqueued; counts and window sizes are the device's
    ratio = lib.lightkv_compress_schedule_ratio
    rho = (C.c_double * 1)(0.5)
    h_out = np.zeros(2, dtype=np.int32)
    h_out_p = C.c_void_p(h_out.ctypes.data)

    def sr(n=1, rho_=rho, X=fake, out=h_out_p):
        return ratio((B._CStage * 1)(stage), n, rho_, 1, 2, 4, X, 64, fake, 64, fake, 64, fake, fake, 64, 32, 0.0, fake,
                     1 << 30, out, None)

    stage.win_remove = 0x1000
    stage.problem.win_remove = 0x1000
    stage.problem.max_window_tokens = 4
    assert sr() == 5                               # host window sizes in the descriptor: not here
    stage.problem.h_win_offsets = None
    assert sr() == 5                               # ... nor host counts
    stage.problem.h_win_remove = None
    assert sr(n=0) == 2 and sr(X=None) == 1 and sr(rho_=None) == 1 and sr(out=None) == 1
    assert sr(rho_=(C.c_double * 1)(-0.1)) == 2 and sr(rho_=(C.c_double * 1)(float("nan"))) == 2
    stage.win_remove = None
    assert sr() == 1                               # the counts need a place
    stage.win_remove = 0x2000
    assert sr() == 2                               # ... the one the descriptor points to
    stage.win_remove = 0x1000
    stage.cu_vis_target = 0x1000
    assert sr() == 5                               # token budgets belong to lightkv_compress_schedule
    stage.cu_vis_target = None
    stage.problem.max_window_tokens = 0
    assert sr() == 2                               # the bound is mandatory
    # aggregate / compact
    assert lib.lightkv_aggregate(C.byref(p), None, fake, fake, fake, 64, fake, 64, fake, 64, None) == 1
    assert lib.lightkv_aggregate(C.byref(p), fake, fake, fake, fake, 8, fake, 64, fake, 64, None) == 2
    other = C.c_void_p(0x100000)
    assert lib.lightkv_compact(C.byref(p), fake, fake, 64, None, 0, None, 0, None, fake, None, None, None, None, 8, 0, None, None) == 2   # in == out
    assert lib.lightkv_compact(C.byref(p), fake, fake, 64, None, 0, None, 0, None, None, None, None, None, None, 8, 0, None, None) == 1   # out missing
    assert lib.lightkv_compact(C.byref(p), None, fake, 64, None, 0, None, 0, None, other, None, None, None, None, 8, 0, None, None) == 1
    assert lib.lightkv_compact(C.byref(p), fake, fake, 64, None, 0, None, 0, fake, other, None, None, None, None, 8, 0, None, None) == 1  # pos without pos_out
    assert lib.lightkv_compact(C.byref(p), fake, fake, 64, None, 0, None, 0, None, C.c_void_p(0x1100), None, None, None, None, 8, 0, None, None) == 2  # overlap
    assert lib.lightkv_compact(C.byref(p), fake, None, 0, fake, 64, None, 0, None, None, other, None, None, other, 8, 0, None, None) == 1  # norms of X without X
    assert lib.lightkv_compact(C.byref(p), fake, fake, 64, None, 0, None, 0, None, other, None, None, None, None, 8, 3, None, None) == 1   # trailing rows need cu_vis_out
    assert lib.lightkv_compact(C.byref(p), fake, fake, 64, None, 0, None, 0, None, other, None, None, None, None, 8, -1, fake, None) == 2
    # build_windows
    hcu = np.array([0, 8], dtype=np.int32)
    hp = C.c_void_p(hcu.ctypes.data)
    assert lib.lightkv_build_windows(1, hp, fake, None, 1, 4, 2, 2, fake, fake, None) == 1
    assert lib.lightkv_build_windows(1, hp, fake, fake, 0, 4, 2, 2, fake, fake, None) == 2
    assert lib.lightkv_build_windows(1, hp, fake, fake, 1, 4, 2, -1, fake, fake, None) == 2
    assert lib.lightkv_build_windows(1, hp, fake, fake, 1, 4, 2, 1000, fake, fake, None) == 5


def test_partition_helpers_agree_with_the_oracle():
    """Host arithmetic exported by the library (no device needed): windows per sequence, and the bound on a window's size."""
    from paper_2605_00789_amd.schedule import windows_per_sequence, max_window_cells
    from oracle import lightkv_oracle as O
    assert windows_per_sequence(5, 6) == 180 and windows_per_sequence(5, 0) == 1
    assert max_window_cells(1, 24, 24, 4) == 36 and max_window_cells(5, 24, 24, 0) == 2880
    # the bound really bounds every window the oracle builds, also on grids that do not divide
    for gh, gw, w in ((24, 24, 6), (5, 7, 2), (7, 9, 4), (3, 3, 3), (3, 3, 5), (64, 64, 32)):
        wo, _ = O.build_windows(np.arange(gh * gw), np.array([0, gh * gw]), 1, gh, gw, w)
        assert np.diff(wo).max() == max_window_cells(1, gh, gw, w)
    with pytest.raises(ValueError):
        windows_per_sequence(0, 2)
    with pytest.raises(ValueError):
        max_window_cells(1, 0, 4, 2)


def test_window_counts_rejects_bad_arguments_before_any_launch(B):
    lib = B._lib
    fake = C.c_void_p(0x1000)
    f = lib.lightkv_window_counts
    assert f(1, 4, None, 0, 0, 0.5, None, None, fake, None, None) == 1
    assert f(1, 4, fake, 0, 0, 0.5, None, None, None, None, None) == 1
    assert f(3, 4, fake, 0, 0, 0.5, None, None, fake, None, None) == 2          # windows do not divide over the sequences
    assert f(1, 4, fake, 7, 0, 0.5, None, None, fake, None, None) == 5          # unknown mode
    assert f(1, 4, fake, 0, 2, 0.5, None, None, fake, None, None) == 5          # unknown direction
    assert f(1, 4, fake, 1, 1, 0.5, None, None, fake, None, None) == 5          # edge counts have no direction
    assert f(1, 4, fake, 2, 0, 0.0, None, fake, fake, None, None) == 1          # target mode without the current offsets
    assert f(1, 4, fake, 0, 0, float("nan"), None, None, fake, None, None) == 2
    assert f(1, 4, fake, 1, 0, -0.1, None, None, fake, None, None) == 2
    assert f(2, 0, fake, 0, 0, 0.5, None, None, fake, None, None) == 0          # nothing to do


def test_probe_library_exports_what_its_header_declares():
    """The measurement library behind bench.py --pass ceilings (no method arithmetic) loads and exports its two calls."""
    header = open(os.path.join(ROOT, "include", "lightkv_probe.h")).read()
    declared = set(re.findall(r"^int (lightkv_probe_[a-z_]+)\(", header, re.M))
    assert declared == {"lightkv_probe_operand_delivery", "lightkv_probe_mfma"}
    lib = C.CDLL(os.path.join(ROOT, "paper_2605_00789_amd", "liblightkv_probe.so"))
    for name in declared:
        assert hasattr(lib, name), name
    # arguments are checked before anything is launched (no device needed)
    lib.lightkv_probe_mfma.restype = C.c_int
    assert lib.lightkv_probe_mfma(None, 4, 10, 1, None, None) != 0
