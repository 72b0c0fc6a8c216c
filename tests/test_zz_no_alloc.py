"""lightkv_select_static: the selection with its scratch in a static device array of the library (for callers that
cannot allocate) against lightkv_select with a caller workspace -- same inputs, every output bit for bit, on two calls
in a row, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _case(seed, batch, tiles, gh, gw, w, frac):
    """Windows of a (batch, tiles, gh, gw) grid cut w x w, random scores and proposals inside every window."""
    from oracle import lightkv_oracle as O
    rng = np.random.default_rng(seed)
    n_seq = tiles * gh * gw
    cu = (np.arange(batch + 1) * n_seq).astype(np.int32)
    pos = np.tile(np.arange(n_seq, dtype=np.int32), batch)
    wo, wt = O.build_windows(pos, cu, tiles, gh, gw, w)
    n = int(cu[-1])
    best_fd = np.full(n, np.inf, dtype=np.float32)
    best_dst = np.full(n, -1, dtype=np.int32)
    rem = np.zeros(len(wo) - 1, dtype=np.int32)
    for k in range(len(wo) - 1):
        toks = wt[wo[k]:wo[k + 1]]
        A, Bn = toks[0::2], toks[1::2]
        if len(Bn) == 0:
            continue
        best_fd[A] = rng.integers(0, 12, size=len(A)).astype(np.float32) / 8.0      # many equal scores: ties by position
        best_dst[A] = rng.choice(Bn, size=len(A))
        rem[k] = int(frac * len(A))
    return cu, wo.astype(np.int32), wt.astype(np.int32), rem, best_fd, best_dst


def _run(case, static):
    from paper_2605_00789_amd import binding as B
    cu, wo, wt, rem, best_fd, best_dst = case
    dev = "cuda:0"
    n = int(cu[-1])
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    prob = B.Problem(batch=len(cu) - 1, d=64, heads=2, head_dim=32, dtype="f32", h_cu_vis=cu, cu_vis=t(cu),
                     n_windows=len(wo) - 1, max_window_tokens=0, win_offsets=t(wo), win_tokens=t(wt), win_remove=t(rem),
                     h_win_offsets=wo, h_win_remove=rem)
    i32 = dict(dtype=torch.int32, device=dev)
    outs = [torch.full((n,), -9, **i32), torch.full((n,), -9, **i32), torch.full((n + 1,), -9, **i32),
            torch.full((max(int(rem.sum()), 1),), -9, **i32), torch.full((len(cu),), -9, **i32)]
    fd, bd = t(best_fd), t(best_dst)
    if static:
        B.lightkv_select_static(prob, fd, bd, *outs)
    else:
        ws = torch.empty(B.lightkv_workspace_size(prob), dtype=torch.uint8, device=dev)
        B.lightkv_select(prob, fd, bd, *outs, ws)
    torch.cuda.synchronize()
    return [o.cpu().numpy() for o in outs]


def test_select_static_equals_select_on_two_calls_in_a_row():
    big = _case(1, batch=3, tiles=2, gh=24, gw=24, w=2, frac=0.8)          # 3456 tokens, windows of 144 (selection by counting)
    small = _case(2, batch=1, tiles=1, gh=10, gw=7, w=3, frac=0.5)         # 70 tokens: reuses the front of the array
    huge = _case(3, batch=1, tiles=1, gh=40, gw=40, w=0, frac=0.6)         # one window of 1600 tokens (multi-workgroup ranking)
    for name, case in (("big", big), ("small", small), ("huge", huge), ("small again", small)):
        print("[select_static]", name, int(case[0][-1]), "tokens", flush=True)
        got = _run(case, static=True)
        want = _run(case, static=False)
        for g, w_, nm in zip(got, want, ("dst", "new_index", "grp_offsets", "grp_src", "cu_vis_out")):
            np.testing.assert_array_equal(g, w_, err_msg="%s: %s" % (name, nm))
        assert int((got[0] >= 0).sum()) == int(case[3].sum())


def test_select_static_refuses_more_tokens_than_the_array_holds():
    from paper_2605_00789_amd import binding as B
    import paper_2605_00789_amd as L
    dev = "cuda:0"
    n = B.SELECT_STATIC_MAX_TOKENS + 1
    cu = (np.arange(6) * 16384).astype(np.int32)[: n // 16384 + 2]
    cu[-1] = n
    z = torch.zeros(n + 1, dtype=torch.int32, device=dev)
    f = torch.zeros(n, dtype=torch.float32, device=dev)
    prob = B.Problem(batch=len(cu) - 1, d=64, heads=2, head_dim=32, dtype="f32", h_cu_vis=cu,
                     cu_vis=torch.from_numpy(cu).to(dev), n_windows=1, max_window_tokens=16, win_offsets=z, win_tokens=z,
                     win_remove=z)
    with pytest.raises(L.LightKVError) as e:
        B.lightkv_select_static(prob, f, z, z, z, z, z, z)
    assert e.value.status == 5
