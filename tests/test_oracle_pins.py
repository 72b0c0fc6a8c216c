"""Pins for the CPU oracle: values the paper prints, closed forms, invariants,
textbook special cases and brute force on tiny inputs.  No GPU involved."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import lightkv_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def _golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=")
                out[k.strip()] = [float(t) for t in v.split()]
    return out


# ---------------------------------------------------------------- Sec. 3.3 / appendix tables
def test_token_fraction_matches_printed_example():
    g = _golden()
    frac = O.token_fraction(40, [10, 20, 30], [0.5, 0.5, 0.5])
    assert frac == pytest.approx(0.46875, abs=1e-15)            # (10 + 5 + 2.5 + 1.25) / 40
    assert round(100 * frac, 1) == g["token_fraction_example_percent"][0]


def test_token_fraction_terms():
    # no compression at all; one stage; a ratio of zero changes nothing
    assert O.token_fraction(10, [10], [0.9]) == pytest.approx(1.0)
    assert O.token_fraction(10, [4], [0.5]) == pytest.approx((4 + 6 * 0.5) / 10)
    assert O.token_fraction(32, [12, 18, 24], [0.0, 0.0, 0.0]) == pytest.approx(1.0)
    # the schedules the paper's tables use, rho = .5 each: the "55 %" retention
    assert O.token_fraction(40, [15, 23, 31], [0.5] * 3) == pytest.approx(0.553125)
    assert O.token_fraction(32, [12, 18, 24], [0.5] * 3) == pytest.approx(0.546875)
    # stages are not interchangeable: order of ratios matters
    assert O.token_fraction(40, [10, 20, 30], [0.5, 0.0, 0.0]) != pytest.approx(
        O.token_fraction(40, [10, 20, 30], [0.0, 0.0, 0.5]))


def test_flops_convention_matches_appendix_table():
    g = _golden()
    for v, bi, full in zip(g["flops_tokens"], g["flops_bipartite"], g["flops_full"]):
        v = int(v)
        assert O.fd_flops(v, 1024, True) / 1e9 == pytest.approx(bi, rel=3e-3)
        assert O.fd_flops(v, 1024, False) / 1e9 == pytest.approx(full, rel=3e-3)
        assert O.fd_flops(v, 1024, False) == 4 * O.fd_flops(v, 1024, True)
    assert O.fd_flops(5, 3, True) == 2 * 3 * 2 * 3              # |A|=3, |B|=2


# ---------------------------------------------------------------- windows
def test_windows_equal_sized_and_spatial():
    gh = gw = 24
    pos = np.arange(gh * gw, dtype=np.int32)
    cu = np.array([0, gh * gw], dtype=np.int32)
    for w, per in ((4, 36), (6, 16), (2, 144), (1, 576)):
        offs, toks = O.build_windows(pos, cu, 1, gh, gw, w)
        assert len(offs) == w * w + 1
        assert np.all(np.diff(offs) == per)                     # "each containing an equal number of tokens"
        assert sorted(toks.tolist()) == list(range(gh * gw))    # a partition
        for k in range(w * w):
            t = toks[offs[k]:offs[k + 1]]
            assert np.all(np.diff(t) > 0)                       # ascending inside a window
            rows, cols = t // gw, t % gw
            side = gh // w
            assert np.all(rows // side == k // w) and np.all(cols // side == k % w)


def test_windows_tiles_sequences_and_holes():
    gh = gw = 4
    # two sequences, two tiles each; the second sequence lost some tokens at an earlier stage
    pos_full = np.arange(2 * gh * gw, dtype=np.int32)
    kept2 = np.array([0, 3, 5, 6, 9, 17, 18, 30, 31], dtype=np.int32)
    pos = np.concatenate([pos_full, kept2])
    cu = np.array([0, 32, 32 + len(kept2)], dtype=np.int32)
    offs, toks = O.build_windows(pos, cu, 2, gh, gw, 2)
    assert len(offs) - 1 == 2 * 2 * 4
    assert offs[-1] == len(pos)
    # windows never mix sequences or tiles
    for k in range(len(offs) - 1):
        t = toks[offs[k]:offs[k + 1]]
        seq = k // 8
        assert np.all((t >= cu[seq]) & (t < cu[seq + 1]))
        assert np.all(pos[t] // (gh * gw) == (k % 8) // 4)
    # token with original cell (tile 1, row 3, col 2) = pos 30 sits in window tile1/(1,1) of sequence 1
    k = 8 + 4 + 3
    assert 32 + 7 in toks[offs[k]:offs[k + 1]].tolist()
    # w = 0: one window per sequence
    offs0, toks0 = O.build_windows(pos, cu, 2, gh, gw, 0)
    assert offs0.tolist() == [0, 32, 41] and toks0.tolist() == list(range(41))


def test_windows_grid_not_divisible():
    gh, gw, w = 5, 7, 2
    pos = np.arange(gh * gw, dtype=np.int32)
    offs, toks = O.build_windows(pos, np.array([0, gh * gw], dtype=np.int32), 1, gh, gw, w)
    assert offs[-1] == gh * gw and len(offs) == 5
    for k in range(4):
        t = toks[offs[k]:offs[k + 1]]
        assert np.all((t // gw) * w // gh == k // w) and np.all((t % gw) * w // gw == k % w)


def test_split_first_token_goes_to_A():
    A, B = O.split_window(np.array([3, 4, 9, 11, 20]))
    assert A.tolist() == [3, 9, 20] and B.tolist() == [4, 11]    # near-equal halves, |A| = ceil(v/2)


# ---------------------------------------------------------------- FD
def test_fd_closed_forms():
    XA = np.array([[1.0, 0, 0], [2.0, 0, 0], [0, 3.0, 0], [-1.0, 0, 0], [1.0, 1.0, 0]])
    XB = np.array([[5.0, 0, 0], [0, 0, 7.0]])
    fd = O.feature_divergence(XA, XB)
    assert fd.shape == (5, 2)
    np.testing.assert_allclose(fd[:, 0], [0, 0, 1, 2, 1 - math.sqrt(0.5)], atol=1e-15)   # same, scaled, orthogonal, opposite, 45 deg
    np.testing.assert_allclose(fd[:, 1], [1, 1, 1, 1, 1], atol=1e-15)
    # zero vector: cosine taken as 0
    np.testing.assert_allclose(O.feature_divergence(np.zeros((1, 3)), XB), [[1, 1]])


def test_fd_against_library_and_scaling():
    rng = np.random.default_rng(0)
    XA, XB = rng.standard_normal((7, 33)), rng.standard_normal((5, 33))
    from scipy.spatial.distance import cdist
    ref = cdist(XA, XB, metric="cosine")                         # 1 - cos, independent implementation
    np.testing.assert_allclose(O.feature_divergence(XA, XB), ref, atol=1e-13)
    sa, sb = rng.uniform(0.1, 9, (7, 1)), rng.uniform(0.1, 9, (5, 1))
    np.testing.assert_allclose(O.feature_divergence(XA * sa, XB * sb), ref, atol=1e-13)
    # rows index A, columns index B (a transposed operand would change the shape or the values)
    np.testing.assert_allclose(O.feature_divergence(XB, XA), ref.T, atol=1e-13)


def test_distance_metrics_closed_forms_library_and_selection():
    """Euclidean and squared-L2 divergences of the similarity-metric ablation (appendix, "Influence of similarity
    metrics"): textbook values, scipy's cdist, and what the two share with / differ from the cosine score."""
    A = np.array([[0.0, 0.0], [1.0, 1.0], [3.0, 4.0]])
    Bm = np.array([[3.0, 4.0], [0.0, 0.0], [6.0, 8.0], [4.0, 5.0]])
    eu = O.feature_divergence(A, Bm, "euclidean")
    np.testing.assert_allclose(eu[0], [5.0, 0.0, 10.0, math.sqrt(41.0)], atol=1e-14)   # 3-4-5 triangle and its double
    np.testing.assert_allclose(eu[2], [0.0, 5.0, 5.0, math.sqrt(2.0)], atol=1e-14)
    np.testing.assert_allclose(O.feature_divergence(A, Bm, "l2sq")[1], [13.0, 2.0, 74.0, 25.0], atol=1e-13)
    rng = np.random.default_rng(3)
    XA, XB = rng.standard_normal((9, 21)), rng.standard_normal((6, 21))
    from scipy.spatial.distance import cdist
    np.testing.assert_allclose(O.feature_divergence(XA, XB, "euclidean"), cdist(XA, XB, "euclidean"), atol=1e-13)
    np.testing.assert_allclose(O.feature_divergence(XA, XB, "l2sq"), cdist(XA, XB, "sqeuclidean"), atol=1e-12)
    np.testing.assert_allclose(O.feature_divergence(XB, XA, "l2sq"), cdist(XA, XB, "sqeuclidean").T, atol=1e-12)
    # translation invariant, not scale invariant (the opposite of the cosine score)
    shift = rng.standard_normal((1, 21))
    np.testing.assert_allclose(O.feature_divergence(XA + shift, XB + shift, "euclidean"), cdist(XA, XB), atol=1e-12)
    np.testing.assert_allclose(O.feature_divergence(2 * XA, 2 * XB, "l2sq"), 4 * cdist(XA, XB, "sqeuclidean"), atol=1e-11)
    assert O.feature_divergence(XA[:1], 2 * XA[:1], "cosine")[0, 0] < 1e-15 < O.feature_divergence(XA[:1], 2 * XA[:1], "l2sq")[0, 0]
    # the square root is monotone: both distances select the same edges and the same merged set
    X = rng.standard_normal((40, 16))
    wo, wt = np.array([0, 17, 40], dtype=np.int32), np.arange(40, dtype=np.int32)
    rem = np.array([4, 7], dtype=np.int32)
    fe, de = O.best_edges(X, wo, wt, "euclidean")
    fs, ds = O.best_edges(X, wo, wt, "l2sq")
    np.testing.assert_array_equal(de, ds)
    np.testing.assert_allclose(fe[np.isfinite(fe)] ** 2, fs[np.isfinite(fs)], rtol=1e-13)
    np.testing.assert_array_equal(O.select(fe, de, wo, wt, rem), O.select(fs, ds, wo, wt, rem))
    # ... and on unit-norm rows they order pairs exactly as the cosine score does (|a-b|^2 = 2 - 2 cos)
    U = X / np.linalg.norm(X, axis=1, keepdims=True)
    fc, dc = O.best_edges(U, wo, wt, "cosine")
    fu, du = O.best_edges(U, wo, wt, "l2sq")
    np.testing.assert_array_equal(dc, du)
    np.testing.assert_allclose(fu[np.isfinite(fu)], 2.0 * fc[np.isfinite(fc)], atol=1e-13)
    with pytest.raises(ValueError):
        O.feature_divergence(XA, XB, "manhattan")


# ---------------------------------------------------------------- selection
def _explicit_fd(X, a, b):
    xa, xb = X[a], X[b]
    dot = sum(float(p) * float(q) for p, q in zip(xa, xb))
    return 1.0 - dot / (math.sqrt(sum(float(p) ** 2 for p in xa)) * math.sqrt(sum(float(q) ** 2 for q in xb)))


@pytest.mark.parametrize("seed", range(12))
def test_selection_is_the_brute_force_minimiser(seed):
    """Among all ways of choosing r nodes of A and one B partner for each, the
    selected edge set has the smallest total FD."""
    rng = np.random.default_rng(seed)
    v = int(rng.integers(4, 10))
    d = 6
    X = rng.standard_normal((v + 3, d))
    toks = np.sort(rng.choice(v + 3, size=v, replace=False)).astype(np.int32)
    offs = np.array([0, v], dtype=np.int32)
    A, B = toks[0::2], toks[1::2]
    r = int(rng.integers(1, min(3, len(A)) + 1))
    bf, bd = O.best_edges(X, offs, toks)
    dst = O.select(bf, bd, offs, toks, np.array([r]))
    got = sorted((int(a), int(dst[a])) for a in range(len(dst)) if dst[a] >= 0)
    assert len(got) == r
    best, best_cost = None, float("inf")
    for S in itertools.combinations(A.tolist(), r):
        for g in itertools.product(B.tolist(), repeat=r):
            cost = sum(_explicit_fd(X, a, b) for a, b in zip(S, g))
            if cost < best_cost - 1e-14:
                best, best_cost = sorted(zip(S, g)), cost
    assert got == best
    # every endpoint is in the right set, and only A tokens leave
    assert all(a in A.tolist() and b in B.tolist() for a, b in got)


@pytest.mark.parametrize("seed,n,k", [(5, 7, 3), (6, 6, 1), (7, 8, 5), (8, 5, 6), (9, 8, 16), (10, 7, 4), (11, 4, 2)])
def test_edge_topk_is_the_brute_force_minimiser_over_edge_sets(seed, n, k):
    """Step 2 read literally: among all k-subsets of the window's |A| x |B| edges the one with the lowest total FD
    (random rows: no ties, so the minimiser is unique), for several window sizes and k up to every edge."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, 4))
    toks = np.arange(n, dtype=np.int32)
    offs = np.array([0, n], dtype=np.int32)
    A, B = toks[0::2], toks[1::2]
    got = sorted(O.select_edge_topk(X, offs, toks, np.array([k])))
    all_edges = [(int(a), int(b)) for a in A for b in B]
    assert k <= len(all_edges)
    best = min(itertools.combinations(all_edges, k), key=lambda es: sum(_explicit_fd(X, a, b) for a, b in es))
    assert got == sorted(best) and len(set(got)) == k


def test_edge_topk_ties_go_to_the_lower_a_position_then_the_lower_b_position():
    """Worked by hand.  Unit basis rows, so every cosine is exactly 1 or 0: window tokens 0..5, A = {0, 2, 4} holds
    e1, e1, e2 and B = {1, 3, 5} holds e1, e1, e2.  FD is 0 on the five edges (0,1) (0,3) (2,1) (2,3) (4,5) and 1 on the
    other four.  The tied edges rank by A position, then B position; the FD-1 edges follow in the same order."""
    e1, e2 = [1.0, 0.0, 0.0], [0.0, 1.0, 0.0]
    X = np.array([e1, e1, e1, e1, e2, e2])
    toks = np.arange(6, dtype=np.int32)
    offs = np.array([0, 6], dtype=np.int32)
    order = [(0, 1), (0, 3), (2, 1), (2, 3), (4, 5),       # FD 0
             (0, 5), (2, 5), (4, 1), (4, 3)]               # FD 1
    for k in range(10):
        assert O.select_edge_topk(X, offs, toks, np.array([k])) == order[:k], k
    # with k = 3 token 0 owns two edges, token 2 one: both leave, token 4 stays; B token 1 receives 0 and 2, B token 3 receives 0
    edges = O.select_edge_topk(X, offs, toks, np.array([3]))
    assert O.removed_by_edges(6, edges).tolist() == [True, False, True, False, False, False]
    go, gs = O.edges_csr(6, edges)
    assert go.tolist() == [0, 0, 2, 2, 3, 3, 3] and gs.tolist() == [0, 2, 0]
    # the order is a property of positions in the window, not of token numbers: list the same rows under other token ids
    toks2 = np.array([10, 3, 11, 4, 12, 5], dtype=np.int32) - 3          # tokens 7,0,8,1,9,2: A = 7,8,9  B = 0,1,2
    X2 = np.zeros((10, 3))
    X2[toks2] = X
    got = O.select_edge_topk(X2, offs, toks2, np.array([3]))
    assert got == [(7, 0), (7, 1), (8, 0)]


def test_selection_ties_and_hub():
    # three identical A tokens, one B equal to them, one far B: all FD ties at 0 -> lowest positions win
    X = np.array([[1.0, 0], [1.0, 0], [1.0, 0], [0, 1.0], [1.0, 0], [0, -1.0]])
    toks = np.arange(6, dtype=np.int32)      # A = 0,2,4   B = 1,3,5
    offs = np.array([0, 6], dtype=np.int32)
    bf, bd = O.best_edges(X, offs, toks)
    assert bd[[0, 2, 4]].tolist() == [1, 1, 1]                  # several A share one B (hub)
    assert np.all(bf[[0, 2, 4]] == 0) and np.all(np.isinf(bf[[1, 3, 5]]))
    dst = O.select(bf, bd, offs, toks, np.array([2]))
    assert dst.tolist() == [1, -1, 1, -1, -1, -1]
    # two equal B candidates: the earlier one is taken
    X2 = np.array([[3.0, 4.0], [6.0, 8.0], [5.0, 0], [30.0, 40.0]])   # norms 5, 10, 50: exact in binary
    bf2, bd2 = O.best_edges(X2, np.array([0, 4], dtype=np.int32), np.arange(4, dtype=np.int32))
    assert bd2[0] == 1


def test_selection_counts_and_limits():
    rng = np.random.default_rng(3)
    n = 40
    X = rng.standard_normal((n, 8))
    offs = np.array([0, 13, 13, 14, 40], dtype=np.int32)        # sizes 13, 0, 1, 26
    toks = np.arange(n, dtype=np.int32)
    bf, bd = O.best_edges(X, offs, toks)
    rem = np.array([7, 0, 0, 5], dtype=np.int32)                 # 7 = |A| of the first window: all of A leaves
    dst = O.select(bf, bd, offs, toks, rem)
    assert int((dst >= 0).sum()) == 12
    kept = np.nonzero(dst < 0)[0]
    assert len(kept) + int((dst >= 0).sum()) == n               # kept + merged = N
    assert [i for i in kept if i < 13] == list(range(1, 13, 2))  # r = |A|  =>  exactly B stays
    assert dst[13] == -1                                         # single-token window untouched
    with pytest.raises(ValueError):
        O.select(bf, bd, offs, toks, np.array([8, 0, 0, 0]))    # more than half cannot leave
    ni = O.kept_index(dst)
    assert ni[kept].tolist() == list(range(len(kept))) and np.all(ni[dst >= 0] == -1)
    go, gs = O.groups_csr(dst)
    assert go[-1] == 12 and sorted(gs.tolist()) == sorted(np.nonzero(dst >= 0)[0].tolist())
    for b in range(n):
        s = gs[go[b]:go[b + 1]]
        assert np.all(dst[s] == b) and np.all(np.diff(s) > 0)
    # positive rescaling of the embeddings does not change the choice
    bf2, bd2 = O.best_edges(X * rng.uniform(0.5, 2, (n, 1)), offs, toks)
    np.testing.assert_array_equal(O.select(bf2, bd2, offs, toks, rem), dst)


def test_ratio_counts_reproduce_the_printed_halving():
    g = _golden()
    n_in, n_out = int(g["halving_stage1_in"][0]), int(g["halving_stage1_out"][0])
    pos = np.arange(n_in, dtype=np.int32)
    offs, toks = O.build_windows(pos, np.array([0, n_in], dtype=np.int32), 1, 24, 24, 4)
    rem = O.removal_counts_ratio(offs, 0.5)
    assert n_in - int(rem.sum()) == n_out
    assert np.all(rem == (np.diff(offs) + 1) // 2)               # = |A|: the 50 % ceiling of one step
    assert np.all(O.removal_counts_ratio(offs, 0.9) == rem)      # capped by that ceiling
    assert rem.sum() / n_in == g["max_step_removal_fraction"][0]
    ev = O.removal_counts_even(104, 16)
    assert ev.sum() == 104 and ev.tolist() == [7] * 8 + [6] * 8


# ---------------------------------------------------------------- xi
def test_xi_closed_form_softmax():
    H, dh, N, T = 3, 4, 6, 5
    # head h: q = e_0 (all text tokens), k_i = log(w_hi) * sqrt(dh) * e_0  ->  softmax_i = w_hi / sum_i w_hi
    w = np.array([[1, 2, 3, 4, 5, 6], [1, 1, 1, 1, 1, 1], [6, 1, 1, 1, 1, 10]], dtype=float)
    Q = np.zeros((T, H * dh)); K = np.zeros((N, H * dh))
    for h in range(H):
        Q[:, h * dh] = 1.0
        K[:, h * dh] = np.log(w[h]) * math.sqrt(dh)
        K[:, h * dh + 1] = 7.0                                   # orthogonal to q: must not matter
    xi = O.xi_text_query(Q, K, [0, N], [0, T], H, dh)
    expect = T * (w / w.sum(axis=1, keepdims=True)).sum(axis=0)
    np.testing.assert_allclose(xi, expect, rtol=1e-13)
    assert xi.sum() == pytest.approx(H * T)
    # explicit scale overrides 1/sqrt(dh)
    xi1 = O.xi_text_query(Q, K / math.sqrt(dh), [0, N], [0, T], H, dh, scale=1.0)
    np.testing.assert_allclose(xi1, expect, rtol=1e-13)


def test_xi_equal_keys_ragged_batch_and_given_lse():
    rng = np.random.default_rng(1)
    H, dh = 2, 8
    cu_vis, cu_txt = [0, 5, 12], [0, 3, 7]
    Q = rng.standard_normal((7, H * dh))
    K = np.tile(rng.standard_normal((1, H * dh)), (12, 1))
    xi = O.xi_text_query(Q, K, cu_vis, cu_txt, H, dh)
    np.testing.assert_allclose(xi[:5], H * 3 / 5, rtol=1e-13)
    np.testing.assert_allclose(xi[5:], H * 4 / 7, rtol=1e-13)
    # random keys: mass per sequence is H*T_b, and a handed-in lse gives the same result
    K = rng.standard_normal((12, H * dh))
    xi = O.xi_text_query(Q, K, cu_vis, cu_txt, H, dh)
    assert xi[:5].sum() == pytest.approx(H * 3) and xi[5:].sum() == pytest.approx(H * 4)
    lse = np.zeros((H, 7))
    for b in range(2):
        for h in range(H):
            l = Q[cu_txt[b]:cu_txt[b + 1], h * dh:(h + 1) * dh] @ K[cu_vis[b]:cu_vis[b + 1], h * dh:(h + 1) * dh].T
            l = l / math.sqrt(dh)
            lse[h, cu_txt[b]:cu_txt[b + 1]] = np.log(np.exp(l).sum(axis=1))
    np.testing.assert_allclose(O.xi_text_query(Q, K, cu_vis, cu_txt, H, dh, lse=lse), xi, rtol=1e-12)
    # a larger normaliser (keys outside the vision span took part of the mass) scales xi down
    np.testing.assert_allclose(O.xi_text_query(Q, K, cu_vis, cu_txt, H, dh, lse=lse + math.log(2)), xi / 2, rtol=1e-12)
    # matches scipy's softmax, head by head
    from scipy.special import softmax
    ref = np.zeros(12)
    for b in range(2):
        for h in range(H):
            l = Q[cu_txt[b]:cu_txt[b + 1], h * dh:(h + 1) * dh] @ K[cu_vis[b]:cu_vis[b + 1], h * dh:(h + 1) * dh].T
            ref[cu_vis[b]:cu_vis[b + 1]] += softmax(l / math.sqrt(dh), axis=1).sum(axis=0)
    np.testing.assert_allclose(xi, ref, rtol=1e-12)


def test_xi_vision_query_degenerate_and_direction():
    rng = np.random.default_rng(2)
    H, dh, N, T = 2, 4, 6, 3
    Qv, Kt = rng.standard_normal((N, H * dh)), rng.standard_normal((T, H * dh))
    lse = np.zeros((H, N))
    for h in range(H):
        l = Qv[:, h * dh:(h + 1) * dh] @ Kt[:, h * dh:(h + 1) * dh].T / math.sqrt(dh)
        lse[h] = np.log(np.exp(l).sum(axis=1))
    # row normalised over the prompt keys only: every vision query spends all its mass there
    np.testing.assert_allclose(O.xi_vision_query(Qv, Kt, lse, [0, N], [0, T], H, dh), H, rtol=1e-13)
    # one extra key of logit 0 in every row: mass on the prompt is S/(S+1)
    lse2 = np.log(np.exp(lse) + 1.0)
    expect = (np.exp(lse) / (np.exp(lse) + 1.0)).sum(axis=0)
    np.testing.assert_allclose(O.xi_vision_query(Qv, Kt, lse2, [0, N], [0, T], H, dh), expect, rtol=1e-13)


def test_xi_floor():
    Q = np.array([[100.0]]); K = np.array([[10.0], [-10.0]])
    xi = O.xi_text_query(Q, K, [0, 2], [0, 1], 1, 1)
    assert xi[0] == pytest.approx(1.0) and xi[1] == O.XI_FLOOR      # exp(-2000) underflows


# ---------------------------------------------------------------- message passing, compaction
def test_message_passing_worked_examples():
    Y = np.array([[0.0, 8.0], [4.0, 0.0], [1.0, 1.0], [2.0, 6.0], [9.0, 9.0]])
    xi = np.array([1.0, 3.0, 2.0, 1.0, 5.0])
    dst = np.array([1, -1, 3, -1, 3], dtype=np.int32)             # 0 -> 1 ; 2 and 4 -> 3 (hub)
    out = O.message_passing(Y, xi, dst)
    np.testing.assert_allclose(out[1], [(3 * 4 + 1 * 0) / 4, (3 * 0 + 1 * 8) / 4])
    np.testing.assert_allclose(out[3], [(1 * 2 + 2 * 1 + 5 * 9) / 8, (1 * 6 + 2 * 1 + 5 * 9) / 8])
    np.testing.assert_array_equal(out[[0, 2, 4]], Y[[0, 2, 4]])   # A rows are not written
    np.testing.assert_array_equal(O.compact(out, dst), out[[1, 3]])


def test_message_passing_invariants():
    rng = np.random.default_rng(4)
    n, d = 30, 5
    Y = rng.standard_normal((n, d)); xi = rng.uniform(0.01, 3, n)
    dst = np.full(n, -1, dtype=np.int32)
    for a in range(0, n, 2):
        if rng.random() < 0.7:
            dst[a] = int(rng.choice(np.arange(1, n, 2)))
    out = O.message_passing(Y, xi, dst)
    # scale invariance in xi
    np.testing.assert_allclose(O.message_passing(Y, 37.5 * xi, dst), out, rtol=1e-13)
    # uniform xi -> arithmetic mean of the group
    outu = O.message_passing(Y, np.ones(n), dst)
    go, gs = O.groups_csr(dst)
    for b in range(n):
        src = gs[go[b]:go[b + 1]]
        if len(src):
            np.testing.assert_allclose(outu[b], np.mean(np.vstack([Y[b:b + 1], Y[src]]), axis=0), rtol=1e-13)
            grp = np.vstack([Y[b:b + 1], Y[src]])
            assert np.all(out[b] <= grp.max(axis=0) + 1e-12) and np.all(out[b] >= grp.min(axis=0) - 1e-12)  # convex
        else:
            np.testing.assert_array_equal(out[b], Y[b])
    # xi-weighted mass is conserved by merge + delete
    xi_out = xi.copy()
    for a in np.nonzero(dst >= 0)[0]:
        xi_out[dst[a]] += xi[a]
    keep = dst < 0
    np.testing.assert_allclose((xi[:, None] * Y).sum(axis=0), (xi_out[keep, None] * out[keep]).sum(axis=0), rtol=1e-12)
    # identical tokens merge without loss
    Y2 = Y.copy(); Y2[dst >= 0] = Y2[dst[dst >= 0]]
    out2 = O.message_passing(Y2, xi, dst)
    np.testing.assert_allclose(out2[keep], Y2[keep], rtol=1e-15, atol=0)
    # r = 0: identity
    np.testing.assert_array_equal(O.message_passing(Y, xi, np.full(n, -1, dtype=np.int32)), Y)


def test_message_passing_with_several_edges_per_node():
    """Step 2 read literally lets an A node own several edges; the message-passing equation then adds it, with its
    full weight, to each of its B nodes."""
    # worked by hand: A = 0, 2 ; B = 1, 3.  Edges 0->1, 0->3, 2->3.
    Y = np.array([[2.0, 0.0], [0.0, 4.0], [6.0, 6.0], [1.0, 1.0]])
    xi = np.array([1.0, 3.0, 2.0, 1.0])
    edges = [(0, 1), (0, 3), (2, 3)]
    out = O.message_passing_edges(Y, xi, edges)
    np.testing.assert_allclose(out[1], [(3 * 0 + 1 * 2) / 4, (3 * 4 + 1 * 0) / 4])
    np.testing.assert_allclose(out[3], [(1 * 1 + 1 * 2 + 2 * 6) / 4, (1 * 1 + 1 * 0 + 2 * 6) / 4])
    np.testing.assert_array_equal(out[[0, 2]], Y[[0, 2]])
    assert O.removed_by_edges(4, edges).tolist() == [True, False, True, False]
    go, gs = O.edges_csr(4, edges)
    assert go.tolist() == [0, 0, 1, 1, 3] and gs.tolist() == [0, 0, 2]
    # the adjacency-matrix form of the equation, written with matrix products
    rng = np.random.default_rng(12)
    n, d = 12, 3
    Y = rng.standard_normal((n, d)); xi = rng.uniform(0.1, 2, n)
    A, B = np.arange(0, n, 2), np.arange(1, n, 2)
    M = (rng.random((len(A), len(B))) < 0.3).astype(np.float64)
    edges = [(int(A[i]), int(B[j])) for i in range(len(A)) for j in range(len(B)) if M[i, j]]
    XB = (Y[B] * xi[B, None] + M.T @ (Y[A] * xi[A, None])) / (xi[B] + M.T @ xi[A])[:, None]
    out = O.message_passing_edges(Y, xi, edges)
    np.testing.assert_allclose(out[B], XB, rtol=1e-13)
    # one edge per A node: the same result as the single-target form
    dst = np.full(n, -1, dtype=np.int32)
    for a in A[:4]:
        dst[a] = int(rng.choice(B))
    one = [(int(a), int(dst[a])) for a in A[:4]]
    np.testing.assert_array_equal(O.message_passing_edges(Y, xi, one), O.message_passing(Y, xi, dst))
    np.testing.assert_array_equal(O.edges_csr(n, one)[1], O.groups_csr(dst)[1])
    # convexity and scale invariance hold edge list or not
    np.testing.assert_allclose(O.message_passing_edges(Y, 7.0 * xi, edges), out, rtol=1e-13)
    for j, b in enumerate(B):
        grp = np.vstack([Y[b:b + 1]] + [Y[A[i]:A[i] + 1] for i in range(len(A)) if M[i, j]])
        assert np.all(out[b] <= grp.max(axis=0) + 1e-12) and np.all(out[b] >= grp.min(axis=0) - 1e-12)


def test_edge_stage_counts_depend_on_the_data():
    """With the k lowest edges, between ceil(k / |B|) and min(k, |A|) tokens leave a window."""
    rng = np.random.default_rng(8)
    n, d, H, dh = 24, 8, 2, 4
    X = rng.standard_normal((n, d)); K = rng.standard_normal((n, d)); V = rng.standard_normal((n, d))
    Q = rng.standard_normal((5, d))
    toks = np.arange(n, dtype=np.int32)
    offs = np.array([0, 12, 24], dtype=np.int32)
    pos = np.arange(n, dtype=np.int32)
    k = np.array([9, 4])
    res = O.compress_stage_edges(X, K, V, Q, pos, np.array([0, n]), np.array([0, 5]), H, dh, offs, toks, k)
    assert len(res.edges) == 13 and len(set(res.edges)) == 13
    for w in range(2):
        gone = int(res.gone[offs[w]:offs[w + 1]].sum())
        assert -(-int(k[w]) // 6) <= gone <= min(int(k[w]), 6)
    assert res.X.shape[0] == n - int(res.gone.sum()) == res.cu_vis[1]
    assert np.all(np.diff(res.pos) > 0)
    # k = |A| * |B|: every edge is selected, every A node leaves, and each B row is the mean over the whole window
    full = O.compress_stage_edges(X, K, V, Q, pos, np.array([0, n]), np.array([0, 5]), H, dh, offs, toks,
                                  np.array([36, 36]), xi=np.ones(n))
    assert full.gone[0::2].all() and not full.gone[1::2].any()
    np.testing.assert_allclose(full.X[0], (X[1] + X[0:12:2].sum(axis=0)) / 7, rtol=1e-13)


# ---------------------------------------------------------------- storage casts
def test_storage_roundtrip():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.5, 3.140625, 1e-3])
    b = O.round_to_storage(x, "bf16")
    back = O.widen(b, "bf16")
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.0 + 2 ** -6   # ties to even
    assert back[3] == -2.5 and back[4] == 3.140625
    assert abs(back[5] - 1e-3) <= 1e-3 * 2 ** -8
    torch = pytest.importorskip("torch")
    r = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    tb = torch.from_numpy(r).to(torch.bfloat16)
    np.testing.assert_array_equal(O.widen(O.round_to_storage(r, "bf16"), "bf16"), tb.to(torch.float64).numpy())


# ---------------------------------------------------------------- whole step on the tiny configuration
def test_whole_schedule_tiny_config():
    from workloads import make_workload
    wl = make_workload(1)
    res = O.compress_schedule(wl)
    assert len(res) == 1
    r = res[0]
    assert r.X.shape == (36, 128) and r.K.shape == (36, 128) and r.pos.shape == (36,)
    assert int((r.dst >= 0).sum()) == 28 and r.cu_vis.tolist() == [0, 36]
    assert np.all(np.diff(r.pos) > 0)
    assert r.xi.sum() == pytest.approx(4 * 16)
    # merged pairs come from the same window and opposite halves
    wo, wt = O.build_windows(wl.pos, wl.cu_vis, 1, 8, 8, 2)
    win_of = np.empty(64, dtype=int); half = np.empty(64, dtype=int)
    for k in range(4):
        t = wt[wo[k]:wo[k + 1]]
        win_of[t] = k; half[t] = np.arange(len(t)) % 2
    for a in np.nonzero(r.dst >= 0)[0]:
        assert win_of[a] == win_of[r.dst[a]] and half[a] == 0 and half[r.dst[a]] == 1
    # with mixture data the merged pairs overwhelmingly share a centre: their FD is far below the median FD
    assert np.median(r.best_fd[r.dst >= 0]) < 0.05


# ---------------------------------------------------------------------------------------------------------------
# per-window counts from a stage's token budget (reading R1: even spread, no window above its set A)
# ---------------------------------------------------------------------------------------------------------------
def test_budget_spread_is_the_even_rule_when_no_window_is_short():
    # 16 equal windows of 36 tokens, 104 to remove: 6 each and one more for the first 8 (104 = 6*16 + 8)
    offs = np.arange(17) * 36
    r, bad = O.removal_counts_target(offs, 1, [104])
    assert r.tolist() == [7] * 8 + [6] * 8 and not bad.any()
    np.testing.assert_array_equal(r, O.removal_counts_even(104, 16))
    # two sequences, each with its own budget
    offs = np.arange(9) * 10
    r, bad = O.removal_counts_target(offs, 2, [9, 2])
    assert r.tolist() == [3, 2, 2, 2, 1, 1, 0, 0] and not bad.any()


def test_budget_spread_by_hand_when_small_windows_bind():
    # window sizes 2, 9, 1, 6, 3 -> caps 1, 5, 0, 3, 2 (a one-token window has nothing to merge into); budget 9:
    # level 2 gives 1+2+0+2+2 = 7, level 3 would give 1+3+0+3+2 = 9 <= 9 -> q = 3, nothing missing
    offs = np.cumsum([0, 2, 9, 1, 6, 3])
    r, bad = O.removal_counts_target(offs, 1, [9])
    assert r.tolist() == [1, 3, 0, 3, 2] and not bad[0]
    # budget 8: q = 2 (7 tokens), one missing -> the first window that can give more than 2 is window 1
    r, _ = O.removal_counts_target(offs, 1, [8])
    assert r.tolist() == [1, 3, 0, 2, 2]
    # the whole of every A set is the most a step can take (limitations paragraph): 11 here; 12 is flagged
    r, bad = O.removal_counts_target(offs, 1, [11])
    assert r.tolist() == [1, 5, 0, 3, 2] and not bad[0]
    r, bad = O.removal_counts_target(offs, 1, [12])
    assert r.tolist() == [1, 5, 0, 3, 2] and bad[0]
    r, bad = O.removal_counts_target(offs, 1, [0])
    assert r.tolist() == [0] * 5 and not bad[0]


def test_budget_spread_invariants_on_random_windows():
    rng = np.random.default_rng(12)
    for _ in range(200):
        batch = int(rng.integers(1, 4))
        per = int(rng.integers(1, 9))
        sizes = rng.integers(0, 12, size=batch * per)
        offs = np.concatenate([[0], np.cumsum(sizes)])
        cap = np.where(sizes >= 2, (sizes + 1) // 2, 0).reshape(batch, per)
        budget = [int(rng.integers(0, cap[b].sum() + 2)) for b in range(batch)]
        r, bad = O.removal_counts_target(offs, batch, budget)
        r = r.reshape(batch, per)
        for b in range(batch):
            assert np.all(r[b] <= cap[b]) and np.all(r[b] >= 0)
            if budget[b] > cap[b].sum():
                assert bad[b] and np.all(r[b] == cap[b])
                continue
            assert not bad[b] and r[b].sum() == budget[b]                      # the budget is met exactly
            free = r[b] < cap[b]                                               # windows that could have given more
            if free.any():
                top = r[b][free].max()
                assert np.all(r[b][free] >= top - 1)                           # ... differ by at most one token
                assert np.all(r[b][~free] <= top + 1)                          # and a window at its cap gives no more than one above them
                hi = np.nonzero(free & (r[b] == top))[0]
                lo = np.nonzero(free & (r[b] == top - 1))[0]
                if len(hi) and len(lo) and r[b][free].min() != top:
                    assert hi.max() < lo.min()                                 # the extra tokens come from the first windows


def test_edge_counts_follow_step_2_as_printed():
    offs = np.cumsum([0, 36, 16, 1, 2, 97])
    assert O.edge_counts_ratio(offs, 0.5).tolist() == [9, 4, 0, 0, 24]
    assert O.edge_counts_ratio(offs, 1.0).tolist() == [18, 8, 0, 1, 48]
    assert O.edge_counts_ratio(np.array([0, 2]), 8.0).tolist() == [1]          # never more than the window has pairs
    offs = np.array([0, 36, 36, 37, 39, 183, 199], dtype=np.int32)             # windows of 36, 0, 1, 2, 144, 16 tokens
    assert O.edge_counts_ratio(offs, 0.5).tolist() == [9, 0, 0, 0, 36, 4]
    assert O.edge_counts_ratio(offs, 0.36).tolist() == [6, 0, 0, 0, 25, 2]
    assert O.edge_counts_ratio(offs, 1.0).tolist() == [18, 0, 0, 1, 72, 8]
    assert O.edge_counts_ratio(np.array([0, 2, 5], dtype=np.int32), 40.0).tolist() == [1, 2]
    assert O.edge_counts_ratio(offs, 0.0).tolist() == [0] * 6


# ---------------------------------------------------------------------------------------------------------------
# full pairwise matching (appendix ablation)
# ---------------------------------------------------------------------------------------------------------------
def test_nearest_neighbours_against_a_library_distance_matrix():
    from scipy.spatial.distance import cdist
    rng = np.random.default_rng(31)
    X = rng.standard_normal((23, 7))
    offs = np.array([0, 9, 10, 23], dtype=np.int32)                  # windows of 9, 1 and 13 tokens
    toks = rng.permutation(23).astype(np.int32)
    toks[0:9].sort(); toks[10:23].sort()
    fd, nb = O.nearest_neighbours(X, offs, toks)
    for lo, hi in ((0, 9), (10, 23)):
        t = toks[lo:hi]
        D = cdist(X[t], X[t], "cosine")
        np.fill_diagonal(D, np.inf)
        np.testing.assert_allclose(fd[t], D.min(axis=1), rtol=0, atol=1e-12)
        np.testing.assert_array_equal(nb[t], t[D.argmin(axis=1)])
    assert np.isinf(fd[toks[9]]) and nb[toks[9]] == -1               # a token alone in its window has no neighbour
    # the whole v x v matrix is what the appendix FLOPs table counts: exactly 4 x the bipartite block of an even window
    assert O.fd_flops(512, 1024, False) == 4 * O.fd_flops(512, 1024, True)
    # Euclidean: 3-4-5
    Y = np.array([[0.0, 0.0], [3.0, 4.0], [3.0, 0.0]])
    fd, nb = O.nearest_neighbours(Y, np.array([0, 3]), np.arange(3, dtype=np.int32), "euclidean")
    assert fd.tolist() == [3.0, 4.0, 3.0] and nb.tolist() == [2, 2, 0]


def test_full_pairwise_selection_by_hand():
    """Unit rows at chosen angles, so the FD order is known: tokens 0..5 at 0, 1, 10, 12, 40 and 41.5 degrees.
    Nearest neighbours: 0<->1 (1 degree), 2<->3 (2 degrees), 4<->5 (1.5 degrees).  Visit order by FD: 0, 1 (1 deg),
    4, 5 (1.5 deg), 2, 3 (2 deg).  r = 2: token 0 leaves into 1; token 1 has received a token and stays; token 4
    leaves into 5.  r = 3 adds 2 -> 3 (5 stays as a destination).  r = 6: only three can leave."""
    ang = np.deg2rad([0.0, 1.0, 10.0, 12.0, 40.0, 41.5])
    X = np.stack([np.cos(ang), np.sin(ang)], axis=1)
    offs, toks = np.array([0, 6], dtype=np.int32), np.arange(6, dtype=np.int32)
    fd, nb = O.nearest_neighbours(X, offs, toks)
    assert nb.tolist() == [1, 0, 3, 2, 5, 4]
    assert O.select_full_pairwise(fd, nb, offs, toks, [2]).tolist() == [1, -1, -1, -1, 5, -1]
    assert O.select_full_pairwise(fd, nb, offs, toks, [3]).tolist() == [1, -1, 3, -1, 5, -1]
    assert O.select_full_pairwise(fd, nb, offs, toks, [6]).tolist() == [1, -1, 3, -1, 5, -1]
    assert O.select_full_pairwise(fd, nb, offs, toks, [0]).tolist() == [-1] * 6
    # a chain: tokens at 0, 3, 5, 6 degrees -> nearest: 0->1, 1->2, 2->3, 3->2; order by FD: 2, 3 (1 deg), 1 (2 deg), 0 (3 deg)
    ang = np.deg2rad([0.0, 3.0, 5.0, 6.0])
    X = np.stack([np.cos(ang), np.sin(ang)], axis=1)
    offs, toks = np.array([0, 4], dtype=np.int32), np.arange(4, dtype=np.int32)
    fd, nb = O.nearest_neighbours(X, offs, toks)
    assert nb.tolist() == [1, 2, 3, 2]
    # 2 leaves into 3; 3 has received and stays; 1's neighbour (2) is gone, so 1 stays; 0 leaves into 1
    assert O.select_full_pairwise(fd, nb, offs, toks, [3]).tolist() == [1, -1, 3, -1]
    # a hub: three tokens whose nearest neighbour is token 3, which itself is nearest to token 2
    ang = np.deg2rad([0.0, 20.0, 11.0, 10.0])
    X = np.stack([np.cos(ang), np.sin(ang)], axis=1)
    fd, nb = O.nearest_neighbours(X, offs, toks)
    assert nb.tolist() == [3, 2, 3, 2]
    # order: 2, 3 (1 deg), 1 (9 deg), 0 (10 deg): 2 -> 3; 3 stays; 1's neighbour 2 is gone; 0 -> 3 (a second source)
    assert O.select_full_pairwise(fd, nb, offs, toks, [4]).tolist() == [3, -1, 3, -1]


def test_full_pairwise_selection_invariants_and_the_conflict_free_optimum():
    rng = np.random.default_rng(77)
    for trial in range(60):
        n = int(rng.integers(2, 40))
        X = rng.standard_normal((n, 5))
        offs, toks = np.array([0, n], dtype=np.int32), np.arange(n, dtype=np.int32)
        fd, nb = O.nearest_neighbours(X, offs, toks)
        r = int(rng.integers(0, n // 2 + 2))
        dst = O.select_full_pairwise(fd, nb, offs, toks, [r])
        gone = dst >= 0
        assert gone.sum() <= r
        assert np.all(dst[gone] == nb[gone])                         # every merge goes to the nearest neighbour
        assert not gone[dst[gone]].any()                             # a destination stays
        if gone.sum() < r:                                           # the visit ran out: every stayer is blocked
            for t in np.nonzero(~gone)[0]:
                assert (dst == t).any() or gone[nb[t]]
        elif r > 0:                                                  # ... else everything before the last merge was visited
            last = max((fd[t], t) for t in np.nonzero(gone)[0])
            for t in np.nonzero(~gone)[0]:
                if (fd[t], t) < last:
                    assert (dst == t).any() or gone[nb[t]]
    # well separated mutual pairs: no conflict ever arises, and the r merges are the r lowest-FD pairs -- the choice
    # that minimises the summed FD over all ways of merging r tokens into distinct partners (brute force)
    ang = np.deg2rad([0.0, 2.0, 30.0, 33.0, 60.0, 61.0, 90.0, 94.0])
    X = np.stack([np.cos(ang), np.sin(ang)], axis=1)
    offs, toks = np.array([0, 8], dtype=np.int32), np.arange(8, dtype=np.int32)
    fd, nb = O.nearest_neighbours(X, offs, toks)
    full = O.feature_divergence(X, X)
    for r in (1, 2, 3, 4):
        dst = O.select_full_pairwise(fd, nb, offs, toks, [r])
        got = sum(full[a, dst[a]] for a in range(8) if dst[a] >= 0)
        best = np.inf
        for S in itertools.combinations(range(8), r):
            rest = [t for t in range(8) if t not in S]
            cost = sum(min(full[a, b] for b in rest) for a in S)     # each leaver to its best staying partner
            best = min(best, cost)
        assert abs(got - best) < 1e-12 and (dst >= 0).sum() == r


# ---------------------------------------------------------------- reverse direction (Sec. 3.2.1, message-passing paragraph)
def test_reverse_direction_by_hand_on_an_odd_window():
    """Five tokens (A = 10, 12, 14 at local positions 0, 2, 4; B = 11, 13): in the reverse direction the two B nodes
    propose and the three A nodes receive, the last A node included."""
    X = np.zeros((16, 2))
    ang = {10: 0.0, 11: 80.0, 12: 40.0, 13: 5.0, 14: 90.0}           # degrees; FD = 1 - cos(difference)
    for t, a in ang.items():
        X[t] = [math.cos(math.radians(a)), math.sin(math.radians(a))]
    toks = np.array([10, 11, 12, 13, 14], dtype=np.int32)
    offs = np.array([0, 5], dtype=np.int32)
    P, R = O.split_window(toks, "b_to_a")
    assert P.tolist() == [11, 13] and R.tolist() == [10, 12, 14]
    bf, bd = O.best_edges(X, offs, toks, direction="b_to_a")
    assert bd[11] == 14 and bd[13] == 10                              # 80 -> 90 (10 degrees), 5 -> 0 (5 degrees)
    assert bf[11] == pytest.approx(1 - math.cos(math.radians(10)), abs=1e-15)
    assert bf[13] == pytest.approx(1 - math.cos(math.radians(5)), abs=1e-15)
    assert np.all(np.isinf(bf[[10, 12, 14]])) and np.all(bd[[10, 12, 14]] == -1)   # the receiving side offers nothing
    dst1 = O.select(bf, bd, offs, toks, np.array([1]), "b_to_a")
    assert {t: int(dst1[t]) for t in toks} == {10: -1, 11: -1, 12: -1, 13: 10, 14: -1}   # the closer pair goes first
    dst2 = O.select(bf, bd, offs, toks, np.array([2]), "b_to_a")
    assert {t: int(dst2[t]) for t in toks} == {10: -1, 11: 14, 12: -1, 13: 10, 14: -1}
    with pytest.raises(ValueError):
        O.select(bf, bd, offs, toks, np.array([3]), "b_to_a")        # |B| = 2 nodes can leave, not 3
    # the paper's direction on the same window: A proposes (three offers), B receives
    bf0, bd0 = O.best_edges(X, offs, toks)
    assert bd0[[10, 12, 14]].tolist() == [13, 13, 11] and np.all(bd0[[11, 13]] == -1)


@pytest.mark.parametrize("seed", range(8))
def test_reverse_direction_is_the_forward_step_with_the_labels_exchanged(seed):
    """Windows of even size: exchanging the two tokens of every (A, B) position pair in the window list and running the
    paper's direction is the reverse direction on the original list (same offers, same merges, token by token)."""
    rng = np.random.default_rng(100 + seed)
    sizes = rng.choice([2, 4, 6, 8, 12], size=4)
    n = int(sizes.sum())
    X = rng.standard_normal((n, 5))
    toks = rng.permutation(n).astype(np.int32)
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    for k in range(4):
        toks[offs[k]:offs[k + 1]].sort()
    swapped = toks.copy()
    swapped[0::2], swapped[1::2] = toks[1::2], toks[0::2]            # all windows start at even offsets
    rem = np.array([int(rng.integers(0, s // 2 + 1)) for s in sizes], dtype=np.int32)
    bf_r, bd_r = O.best_edges(X, offs, toks, direction="b_to_a")
    bf_f, bd_f = O.best_edges(X, offs, swapped)
    np.testing.assert_array_equal(bf_r, bf_f)
    np.testing.assert_array_equal(bd_r, bd_f)
    np.testing.assert_array_equal(O.select(bf_r, bd_r, offs, toks, rem, "b_to_a"), O.select(bf_f, bd_f, offs, swapped, rem))


@pytest.mark.parametrize("seed", range(6))
def test_reverse_direction_is_the_brute_force_minimiser(seed):
    """As for the paper's direction: among all ways of choosing r proposing nodes (now of B) and one receiving node (of
    A) for each, the selected edge set has the smallest total FD; windows of odd size included."""
    rng = np.random.default_rng(200 + seed)
    v = int(rng.integers(4, 10))
    X = rng.standard_normal((v + 2, 6))
    toks = np.sort(rng.choice(v + 2, size=v, replace=False)).astype(np.int32)
    offs = np.array([0, v], dtype=np.int32)
    A, B = toks[0::2], toks[1::2]
    r = int(rng.integers(1, min(3, len(B)) + 1))
    bf, bd = O.best_edges(X, offs, toks, direction="b_to_a")
    dst = O.select(bf, bd, offs, toks, np.array([r]), "b_to_a")
    got = sorted((int(t), int(dst[t])) for t in range(len(dst)) if dst[t] >= 0)
    best, best_cost = None, float("inf")
    for S in itertools.combinations(B.tolist(), r):
        for g in itertools.product(A.tolist(), repeat=r):
            cost = sum(_explicit_fd(X, b, a) for b, a in zip(S, g))
            if cost < best_cost - 1e-14:
                best, best_cost = sorted(zip(S, g)), cost
    assert got == best and all(b in B.tolist() and a in A.tolist() for b, a in got)


def test_reverse_direction_counts():
    offs = np.array([0, 5, 6, 6, 14, 17], dtype=np.int32)              # sizes 5, 1, 0, 8, 3
    assert O.removal_counts_ratio(offs, 0.5, "b_to_a").tolist() == [2, 0, 0, 4, 1]
    assert O.removal_counts_ratio(offs, 0.5).tolist() == [2, 0, 0, 4, 1]
    assert O.removal_counts_ratio(offs, 0.9, "b_to_a").tolist() == [2, 0, 0, 4, 1]   # |B| = floor(v/2) at most
    assert O.removal_counts_ratio(offs, 0.9).tolist() == [3, 0, 0, 4, 2]             # |A| = ceil(v/2) at most (v = 1: its A)
    rem, bad = O.removal_counts_target(offs, 1, [7], "b_to_a")
    assert rem.tolist() == [2, 0, 0, 4, 1] and not bad[0]              # caps 2, 0, 0, 4, 1: every one binds
    rem, bad = O.removal_counts_target(offs, 1, [8], "b_to_a")
    assert bad[0] and rem.tolist() == [2, 0, 0, 4, 1]
    rem, bad = O.removal_counts_target(offs, 1, [8])
    assert not bad[0] and rem.tolist() == [3, 0, 0, 3, 2]              # caps 3, 0, 0, 4, 2: level 3 meets the budget exactly


def test_whole_stage_by_hand_on_four_tokens():
    """One window of four tokens worked by hand (Sec. 3.2.1 Steps 1-5, Eq. similarity and message-passing):
    A = {t0, t2}, B = {t1, t3}; t0 is identical to t1 (FD 0) and t2 is closest to t3 (FD 1 - 1/sqrt 2); with r = 1 the
    one merge is t0 -> t1, weighted 1 : 3 by the given xi; the sequence is then t1', t2, t3 in the old order."""
    s = 1.0 / math.sqrt(2.0)
    X = np.array([[1.0, 0.0], [1.0, 0.0], [0.0, 1.0], [s, s]])
    K = np.array([[4.0, 0.0], [0.0, 4.0], [5.0, 6.0], [7.0, 8.0]])
    V = np.array([[8.0, 8.0], [0.0, 4.0], [1.0, 2.0], [3.0, 4.0]])
    xi = np.array([1.0, 3.0, 1.0, 1.0])
    pos = np.arange(4, dtype=np.int32)
    cu = np.array([0, 4], dtype=np.int32)
    wo, wt = np.array([0, 4]), np.arange(4)
    r = O.compress_stage(X, K, V, None, pos, cu, np.array([0, 0]), 1, 2, wo, wt, np.array([1]), xi=xi)
    np.testing.assert_allclose(r.best_fd[[0, 2]], [0.0, 1.0 - s], atol=1e-15)
    np.testing.assert_array_equal(r.best_dst[[0, 2]], [1, 3])
    np.testing.assert_array_equal(r.dst, [1, -1, -1, -1])
    np.testing.assert_array_equal(r.new_index, [-1, 0, 1, 2])
    np.testing.assert_array_equal(r.grp_offsets, [0, 0, 1, 1, 1])
    np.testing.assert_array_equal(r.grp_src, [0])
    np.testing.assert_allclose(r.X, [[1.0, 0.0], [0.0, 1.0], [s, s]], atol=1e-15)
    np.testing.assert_allclose(r.K, [[1.0, 3.0], [5.0, 6.0], [7.0, 8.0]], atol=1e-15)      # (1*K0 + 3*K1) / 4
    np.testing.assert_allclose(r.V, [[2.0, 5.0], [1.0, 2.0], [3.0, 4.0]], atol=1e-15)
    np.testing.assert_array_equal(r.pos, [1, 2, 3])
    np.testing.assert_array_equal(r.cu_vis, [0, 3])
    # r = 2: both A nodes leave, the sequence is t1', t3'
    r2 = O.compress_stage(X, K, V, None, pos, cu, np.array([0, 0]), 1, 2, wo, wt, np.array([2]), xi=xi)
    np.testing.assert_array_equal(r2.dst, [1, -1, 3, -1])
    np.testing.assert_allclose(r2.K, [[1.0, 3.0], [6.0, 7.0]], atol=1e-15)                  # (K2 + K3) / 2
    np.testing.assert_array_equal(r2.pos, [1, 3])
    # the full pairwise visit on the same tokens: t0 and t1 are each other's neighbours at FD 0 and t0 comes first, so
    # t0 -> t1; t1 has received and stays; next in order is t2 (its neighbour t3 is still there): t2 -> t3
    p1 = O.compress_stage_full_pairwise(X, K, V, None, pos, cu, np.array([0, 0]), 1, 2, wo, wt, np.array([1]), xi=xi)
    np.testing.assert_array_equal(p1.dst, [1, -1, -1, -1])
    np.testing.assert_allclose(p1.K, r.K, atol=1e-15)
    p2 = O.compress_stage_full_pairwise(X, K, V, None, pos, cu, np.array([0, 0]), 1, 2, wo, wt, np.array([2]), xi=xi)
    np.testing.assert_array_equal(p2.dst, [1, -1, 3, -1])
    np.testing.assert_allclose(p2.X[1], [s / 2, (1 + s) / 2], atol=1e-15)                   # (X2 + X3) / 2
    np.testing.assert_array_equal(p2.cu_vis, [0, 2])


def test_proposing_side_and_even_spread_closed_forms():
    """The proposing set of a window of v tokens has ceil(v/2) nodes (floor(v/2) in the reverse direction); equal windows
    that all lose the same budget give floor(R/W) each and one more from the first R mod W (Sec. 3.2.2)."""
    for v in range(0, 12):
        assert O.proposing_count(v) == (v + 1) // 2 and O.proposing_count(v, "b_to_a") == v // 2
    np.testing.assert_array_equal(O.stage_removals(2, 576, 472, 16), np.tile([7] * 8 + [6] * 8, 2))   # 104 = 16*6 + 8
    np.testing.assert_array_equal(O.stage_removals(1, 64, 36, 4), [7, 7, 7, 7])
