"""CPU oracle for one LightKV compression step  --  TEST INFRASTRUCTURE ONLY.

Plain numpy, float64, slow on purpose.  It shares no code with the HIP path and
must never be imported by the product package; only tests, the smoke check and
the benchmark's cpu_baseline leg call it.

What it computes follows the paper's Sec. 3.2.1 (Steps 1-5), Sec. 3.2.2
(windows, hierarchical schedule) and Sec. 3.3 (token-count formula):

  windows        Sec. 3.2 / 3.2.2 "Window partitioning": the token grid is cut
                 into w x w non-overlapping windows, every later step is per window.
  split          Step 1: tokens of a window alternate between the two node sets;
                 the first token of a window goes to A (the paper counts from 1,
                 "odd-indexed" -> A).
  FD             Eq. (similarity): FD(a,b) = 1 - <x_a,x_b> / (|x_a| |x_b|).
  T_rho / M      Step 2: lowest-FD edges; an A node with no selected edge (set R)
                 is left unchanged.  Reading used here: every A node proposes its
                 lowest-FD B node, and the r A nodes with the lowest proposals are
                 the ones merged (several A may share one B; exactly r tokens go).
                 The literal reading -- the k lowest-FD edges of the window's
                 complete bipartite graph, an A node owning as many of them as
                 rank that low -- is `select_edge_topk` with
                 `message_passing_edges` / `compress_stage_edges`: every A node
                 with at least one selected edge leaves, so the number of tokens
                 that go depends on the data.
                 Full pairwise matching (the appendix ablation): FD between every two
                 tokens of a window, `nearest_neighbours` / `select_full_pairwise`.
  xi             Step 3, Eq. (attention-factor): attention between a vision token
                 and the prompt tokens, summed over heads and prompt tokens.
  message pass   Eq. (message-passing): X_B <- (xi_B + M^T xi_A)^-1 (X_B*xi_B + M^T (X_A*xi_A)),
                 applied alike to the hidden states and to the layer's K and V rows.
  delete/reorder Steps 4-5: merged A nodes are dropped, R and B keep their order.

Pins (tests/test_oracle_*.py):  brute force over all merge choices on tiny
windows, FD special cases and a library GEMM, softmax identities for xi,
convexity / scale invariance / uniform-weight mean / mass conservation for the
message passing, count identities, the printed 46.9 % example of Sec. 3.3 and
the appendix FLOPs table (bipartite vs. full pairwise).

Parity unpinned by the paper (fixed by a stated reading only): which parity of
the alternation goes to A, which K/V are merged and their position ids, the
order-preserving output layout, the window of a token after earlier stages
removed some of its neighbours, and how xi of a merged token is obtained at
the next stage (recomputed).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

NORM_EPS = 1e-12      # floor on |x| in the cosine
XI_FLOOR = 1e-30      # floor on xi (keeps the weighted mean defined)


# ---------------------------------------------------------------------------
# storage <-> float64
# ---------------------------------------------------------------------------
def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """Stored values (fp32, or bf16 bit patterns as uint16) as float64, exactly."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        bits = np.asarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """float64 -> stored dtype with round-to-nearest-even (stage boundary)."""
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return x32
    if dtype == "bf16":
        u = x32.view(np.uint32)
        r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        return (r >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


# ---------------------------------------------------------------------------
# Sec. 3.3 token-count formula and the appendix FLOPs convention
# ---------------------------------------------------------------------------
def token_fraction(L: int, Lambda: Sequence[int], P: Sequence[float]) -> float:
    """Eq. (complexity): vision tokens processed over L layers with compression
    after layers Lambda at ratios P, as a fraction of v*L."""
    s = len(Lambda)
    assert s == len(P) and s >= 1
    total = float(Lambda[0])                                   # term (1)
    keep = 1.0
    for i in range(1, s):                                      # term (2)
        keep *= (1.0 - P[i - 1])
        total += (Lambda[i] - Lambda[i - 1]) * keep
    keep *= (1.0 - P[s - 1])
    total += (L - Lambda[s - 1]) * keep                        # term (3)
    return total / L


def fd_flops(v: int, d: int, bipartite: bool) -> float:
    """Multiply-add count (2 per pair element) of the FD contraction of one
    window of v tokens: |A| x |B| pairs for the bipartite graph, the whole v x v
    matrix for full pairwise matching (appendix FLOPs table)."""
    if bipartite:
        return 2.0 * ((v + 1) // 2) * (v // 2) * d
    return 2.0 * v * v * d


# ---------------------------------------------------------------------------
# windows (Sec. 3.2, Sec. 3.2.2) and per-window removal counts
# ---------------------------------------------------------------------------
def build_windows(pos: np.ndarray, cu_vis: np.ndarray, tiles: int, grid_h: int, grid_w: int,
                  w: int) -> Tuple[np.ndarray, np.ndarray]:
    """Window lists in CSR form.

    A token's window is decided by its cell in the ORIGINAL grid (pos = tile*Gh*Gw
    + row*Gw + col): (tile, floor(row*w/Gh), floor(col*w/Gw)).  Windows never
    cross tiles or sequences.  w == 0 means one window per sequence.  Inside a
    window tokens are listed in ascending sequence order.
    Returns (win_offsets[int32, n_windows+1], win_tokens[int32, sumN])."""
    pos = np.asarray(pos, dtype=np.int64)
    batch = len(cu_vis) - 1
    per_seq = 1 if w == 0 else tiles * w * w
    lists: List[List[int]] = [[] for _ in range(batch * per_seq)]
    for b in range(batch):
        for i in range(int(cu_vis[b]), int(cu_vis[b + 1])):
            if w == 0:
                wid = 0
            else:
                p = int(pos[i])
                tile, cell = divmod(p, grid_h * grid_w)
                row, col = divmod(cell, grid_w)
                wid = tile * w * w + (row * w // grid_h) * w + (col * w // grid_w)
            lists[b * per_seq + wid].append(i)
    offs = np.zeros(len(lists) + 1, dtype=np.int32)
    for k, l in enumerate(lists):
        offs[k + 1] = offs[k] + len(l)
    toks = np.array([i for l in lists for i in l], dtype=np.int32).reshape(-1)
    return offs, toks


def removal_counts_even(n_remove: int, n_windows: int) -> np.ndarray:
    """Spread a stage's removal budget over the windows of one sequence:
    floor(R/W) each, the first R mod W windows one more."""
    q, rem = divmod(int(n_remove), int(n_windows))
    return np.array([q + (1 if k < rem else 0) for k in range(n_windows)], dtype=np.int32)


def proposing_count(v, direction: str = "a_to_b"):
    """Tokens of a v-token window on the side that proposes: |A| = ceil(v/2) in the paper's direction, |B| =
    floor(v/2) in the reverse one (Sec. 3.2.1, message-passing paragraph)."""
    if direction not in ("a_to_b", "b_to_a"):
        raise ValueError("unknown direction %r" % (direction,))
    return (v + 1) // 2 if direction == "a_to_b" else v // 2


def removal_counts_ratio(win_offsets: np.ndarray, rho: float, direction: str = "a_to_b") -> np.ndarray:
    """Paper-style count: a fraction rho of every window's tokens leaves
    (Sec. 3.2.2: a fraction 1-rho remains), capped by the proposing set (|A|: the 50 % limit
    named in the limitations paragraph)."""
    v = np.diff(np.asarray(win_offsets, dtype=np.int64))
    return np.minimum(np.floor(rho * v + 1e-9).astype(np.int64), proposing_count(v, direction)).astype(np.int32)


def removal_counts_target(win_offsets: np.ndarray, batch: int, n_remove: Sequence[int],
                          direction: str = "a_to_b") -> Tuple[np.ndarray, np.ndarray]:
    """Removal counts that take n_remove[b] tokens out of sequence b, whatever sizes its windows have
    (later stages: the windows no longer hold equal numbers of tokens).  Reading of Step 2 / Sec. 3.2.2 when a stage
    is given a token budget instead of a ratio: the budget is spread as evenly as the windows allow.  A window of v
    tokens can give up at most its proposing set, cap = ceil(v/2) (floor(v/2) in the reverse direction; 0 if v < 2:
    nothing to merge into).  With q the largest
    level for which sum_w min(cap_w, q) does not exceed the budget, window w gives min(cap_w, q), and what is then
    still missing comes one token each from the first windows (in window order) that can give more than q.  Where no
    cap binds this is floor(R/W) per window and one more for the first R mod W windows.
    Returns (win_remove[int32, n_windows], infeasible[bool, batch]): a budget above sum_w cap_w cannot be met; then
    every window gives its cap and the sequence is flagged."""
    v = np.diff(np.asarray(win_offsets, dtype=np.int64))
    per_seq = len(v) // batch
    out = np.zeros(len(v), dtype=np.int32)
    bad = np.zeros(batch, dtype=bool)
    for b in range(batch):
        vs = v[b * per_seq:(b + 1) * per_seq]
        cap = [int(proposing_count(int(x), direction)) if x >= 2 else 0 for x in vs]
        R = int(n_remove[b])
        if R < 0:
            raise ValueError("a stage cannot add tokens")
        if R > sum(cap):
            out[b * per_seq:(b + 1) * per_seq] = cap
            bad[b] = True
            continue
        q = 0
        while sum(min(c, q + 1) for c in cap) <= R:
            q += 1
            if q > max(cap + [0]):
                break
        r = [min(c, q) for c in cap]
        missing = R - sum(r)
        for k in range(per_seq):
            if missing == 0:
                break
            if cap[k] > q:
                r[k] += 1
                missing -= 1
        assert missing == 0
        out[b * per_seq:(b + 1) * per_seq] = r
    return out, bad


def edge_counts_ratio(win_offsets: np.ndarray, rho: float) -> np.ndarray:
    """Step 2 as printed: floor(rho * v / 2) lowest-FD pairs in a window of v tokens, never more than the window has
    pairs (|A| * |B|)."""
    v = np.diff(np.asarray(win_offsets, dtype=np.int64))
    k = np.floor(rho * v / 2.0 + 1e-9).astype(np.int64)
    return np.minimum(k, ((v + 1) // 2) * (v // 2)).astype(np.int32)


def split_window(tokens: np.ndarray, direction: str = "a_to_b") -> Tuple[np.ndarray, np.ndarray]:
    """Step 1: local positions 0,2,4,.. -> A ; 1,3,5,.. -> B.  Returns (proposing set, receiving set): (A, B) in the
    paper's direction; in the reverse direction (Sec. 3.2.1, message-passing paragraph: defined analogously) the
    nodes of B propose and those of A receive, so (B, A)."""
    tokens = np.asarray(tokens)
    if direction == "a_to_b":
        return tokens[0::2], tokens[1::2]
    if direction == "b_to_a":
        return tokens[1::2], tokens[0::2]
    raise ValueError("unknown direction %r" % (direction,))


# ---------------------------------------------------------------------------
# Step 3: prompt-guidance weight xi
# ---------------------------------------------------------------------------
def _lse(l: np.ndarray, axis: int) -> np.ndarray:
    m = np.max(l, axis=axis, keepdims=True)
    return (m + np.log(np.sum(np.exp(l - m), axis=axis, keepdims=True))).squeeze(axis)


def xi_text_query(Q: np.ndarray, K: np.ndarray, cu_vis, cu_txt, heads: int, head_dim: int,
                  scale: Optional[float] = None, lse: Optional[np.ndarray] = None) -> np.ndarray:
    """xi_i = sum_h sum_{j in prompt} A[h, j, i] with the prompt token j as the
    query and the vision token i as the key; A is the softmax over the sequence's
    vision keys of q_j.k_i*scale, or exp(logit - lse[h, j]) when the layer's own
    log-sum-exp is handed in (lse: [heads, sumT]).  Q: [sumT, H*d_h], K: [sumN, H*d_h]."""
    scale = 1.0 / math.sqrt(head_dim) if scale is None else scale
    xi = np.zeros(K.shape[0])
    for b in range(len(cu_vis) - 1):
        v0, v1, t0, t1 = int(cu_vis[b]), int(cu_vis[b + 1]), int(cu_txt[b]), int(cu_txt[b + 1])
        if v1 == v0 or t1 == t0:
            continue
        for h in range(heads):
            q = Q[t0:t1, h * head_dim:(h + 1) * head_dim]
            k = K[v0:v1, h * head_dim:(h + 1) * head_dim]
            l = (q @ k.T) * scale                                # [T, N]
            z = _lse(l, axis=1) if lse is None else lse[h, t0:t1]
            xi[v0:v1] += np.exp(l - z[:, None]).sum(axis=0)
    return np.maximum(xi, XI_FLOOR)


def xi_vision_query(Qv: np.ndarray, Kt: np.ndarray, lse: np.ndarray, cu_vis, cu_txt, heads: int,
                    head_dim: int, scale: Optional[float] = None) -> np.ndarray:
    """Index order of Eq. (attention-factor) taken literally: vision token i is the
    query, prompt token j the key; lse[h, i] is the log-sum-exp of the whole
    attention row of vision query i (given by the caller, since that row also
    covers keys outside the prompt).  Qv: [sumN, H*d_h], Kt: [sumT, H*d_h]."""
    scale = 1.0 / math.sqrt(head_dim) if scale is None else scale
    xi = np.zeros(Qv.shape[0])
    for b in range(len(cu_vis) - 1):
        v0, v1, t0, t1 = int(cu_vis[b]), int(cu_vis[b + 1]), int(cu_txt[b]), int(cu_txt[b + 1])
        for h in range(heads):
            q = Qv[v0:v1, h * head_dim:(h + 1) * head_dim]
            k = Kt[t0:t1, h * head_dim:(h + 1) * head_dim]
            l = (q @ k.T) * scale                                # [N, T]
            xi[v0:v1] += np.exp(l - lse[h, v0:v1][:, None]).sum(axis=1)
    return np.maximum(xi, XI_FLOOR)


# ---------------------------------------------------------------------------
# Steps 1-2: FD, best edge per A node, the r merged nodes per window
# ---------------------------------------------------------------------------
METRICS = ("cosine", "euclidean", "l2sq")


def feature_divergence(XA: np.ndarray, XB: np.ndarray, metric: str = "cosine") -> np.ndarray:
    """Pairwise divergence of the rows of XA and XB.
    "cosine" (the method's choice): Eq. (similarity), 1 - <a,b>/(max(|a|,eps) max(|b|,eps)), clamped at 0.
    "euclidean" / "l2sq" (the similarity-metric ablation of the appendix): |a - b| and |a - b|^2,
    written out as the sum of squared coordinate differences."""
    if metric == "cosine":
        na = np.maximum(np.sqrt((XA * XA).sum(axis=1)), NORM_EPS)
        nb = np.maximum(np.sqrt((XB * XB).sum(axis=1)), NORM_EPS)
        cos = (XA @ XB.T) / (na[:, None] * nb[None, :])
        return np.maximum(1.0 - cos, 0.0)
    if metric not in METRICS:
        raise ValueError("unknown metric %r" % (metric,))
    d2 = np.empty((XA.shape[0], XB.shape[0]))
    for i in range(XA.shape[0]):
        diff = XB - XA[i][None, :]
        d2[i] = (diff * diff).sum(axis=1)
    return np.sqrt(d2) if metric == "euclidean" else d2


def best_edges(X: np.ndarray, win_offsets: np.ndarray, win_tokens: np.ndarray, metric: str = "cosine",
               direction: str = "a_to_b"):
    """For every A node its lowest-FD B node of the same window (direction "b_to_a": read A as the proposing set B and
    B as the receiving set A throughout).
    Returns best_fd[float64, N] (+inf on B rows and on A rows of windows without a
    B node) and best_dst[int32, N] (token index, -1 where there is none).
    Ties go to the B node that comes first in the window."""
    n = X.shape[0]
    best_fd = np.full(n, np.inf)
    best_dst = np.full(n, -1, dtype=np.int32)
    for wdx in range(len(win_offsets) - 1):
        toks = win_tokens[win_offsets[wdx]:win_offsets[wdx + 1]]
        A, B = split_window(toks, direction)
        if len(B) == 0 or len(A) == 0:
            continue
        fd = feature_divergence(X[A], X[B], metric)
        j = np.argmin(fd, axis=1)                # first minimum = lowest local B position
        best_fd[A] = fd[np.arange(len(A)), j]
        best_dst[A] = B[j]
    return best_fd, best_dst


def select(best_fd: np.ndarray, best_dst: np.ndarray, win_offsets: np.ndarray,
           win_tokens: np.ndarray, win_remove: np.ndarray, direction: str = "a_to_b"):
    """Step 2 under the one-edge-per-A-node reading: in every window the r A nodes
    with the lowest proposal (ties: earlier in the window first) are merged.
    Returns dst[int32, N]: the B token an A token is merged into, -1 for every
    token that stays (R and B)."""
    n = best_fd.shape[0]
    dst = np.full(n, -1, dtype=np.int32)
    for wdx in range(len(win_offsets) - 1):
        toks = win_tokens[win_offsets[wdx]:win_offsets[wdx + 1]]
        A, B = split_window(toks, direction)
        r = int(win_remove[wdx])
        if r == 0 or len(B) == 0:
            continue
        if r > len(A):
            raise ValueError("window %d: r=%d exceeds |A|=%d (at most half of a window can leave)"
                             % (wdx, r, len(A)))
        order = sorted(range(len(A)), key=lambda la: (best_fd[A[la]], la))
        for la in order[:r]:
            dst[A[la]] = best_dst[A[la]]
    return dst


def select_edge_topk(X: np.ndarray, win_offsets, win_tokens, win_edges: np.ndarray, metric: str = "cosine"):
    """Step 2 read literally: the k lowest-FD EDGES of the window's complete
    bipartite graph (ties: lower A position, then lower B position).  Returns a
    list of (a_token, b_token) edges; an A node may own several edges."""
    edges = []
    for wdx in range(len(win_offsets) - 1):
        toks = win_tokens[win_offsets[wdx]:win_offsets[wdx + 1]]
        A, B = split_window(toks)
        k = int(win_edges[wdx])
        if k == 0 or len(B) == 0:
            continue
        fd = feature_divergence(X[A], X[B], metric)
        cand = sorted(((fd[i, j], i, j) for i in range(len(A)) for j in range(len(B))))
        edges += [(int(A[i]), int(B[j])) for _, i, j in cand[:k]]
    return edges


def nearest_neighbours(X: np.ndarray, win_offsets, win_tokens, metric: str = "cosine"):
    """Full pairwise matching (appendix, "Bipartite vs. full pairwise matching"): FD between every two tokens of a
    window (the whole v x v matrix, diagonal excluded), and for every token its lowest-FD neighbour (ties: the
    neighbour that comes first in the window).  Returns near_fd[float64, N] (+inf for a token alone in its window)
    and near_dst[int32, N] (token index, -1 where there is none)."""
    n = X.shape[0]
    near_fd = np.full(n, np.inf)
    near_dst = np.full(n, -1, dtype=np.int32)
    for wdx in range(len(win_offsets) - 1):
        toks = np.asarray(win_tokens[win_offsets[wdx]:win_offsets[wdx + 1]])
        if len(toks) < 2:
            continue
        fd = feature_divergence(X[toks], X[toks], metric)
        np.fill_diagonal(fd, np.inf)
        j = np.argmin(fd, axis=1)
        near_fd[toks] = fd[np.arange(len(toks)), j]
        near_dst[toks] = toks[j]
    return near_fd, near_dst


def select_full_pairwise(near_fd: np.ndarray, near_dst: np.ndarray, win_offsets, win_tokens, win_remove):
    """Which tokens leave under full pairwise matching.  The appendix gives accuracy and cost of this variant but no
    merge rule; the reading taken here: the tokens of a window are visited in ascending order of their
    nearest-neighbour FD (ties: earlier in the window first), and a visited token is merged into its nearest
    neighbour unless (a) a token merged earlier was merged INTO it (a token that has received others stays), or
    (b) its nearest neighbour has itself been merged away already; the visit ends after r_w merges.  So a token
    that leaves is never a destination, every destination stays, and at most r_w tokens leave a window -- fewer if
    the visit runs out of tokens that may leave.  Returns dst[int32, N] (-1: stays)."""
    n = near_fd.shape[0]
    dst = np.full(n, -1, dtype=np.int32)
    for wdx in range(len(win_offsets) - 1):
        toks = np.asarray(win_tokens[win_offsets[wdx]:win_offsets[wdx + 1]])
        r = int(win_remove[wdx])
        if r == 0 or len(toks) < 2:
            continue
        order = sorted(range(len(toks)), key=lambda l: (near_fd[toks[l]], l))
        received = set()
        gone = set()
        done = 0
        for l in order:
            if done == r:
                break
            t = int(toks[l])
            b = int(near_dst[t])
            if b < 0 or t in received or b in gone:
                continue
            dst[t] = b
            gone.add(t)
            received.add(b)
            done += 1
    return dst


def kept_index(dst: np.ndarray) -> np.ndarray:
    """new_index[i]: row of token i in the compacted tensors (order preserved), -1 if merged away."""
    keep = dst < 0
    new_index = np.where(keep, np.cumsum(keep) - 1, -1).astype(np.int32)
    return new_index


def groups_csr(dst: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Inverse of dst: sources of token b are grp_src[grp_offsets[b]:grp_offsets[b+1]], ascending."""
    n = dst.shape[0]
    srcs: List[List[int]] = [[] for _ in range(n)]
    for a in range(n):
        if dst[a] >= 0:
            srcs[int(dst[a])].append(a)
    offs = np.zeros(n + 1, dtype=np.int32)
    for b in range(n):
        offs[b + 1] = offs[b] + len(srcs[b])
    flat = np.array([a for l in srcs for a in l], dtype=np.int32).reshape(-1)
    return offs, flat


# ---------------------------------------------------------------------------
# Steps 3-5: message passing, delete, reorder
# ---------------------------------------------------------------------------
def message_passing(Y: np.ndarray, xi: np.ndarray, dst: np.ndarray) -> np.ndarray:
    """Eq. (message-passing) with M[a, dst[a]] = 1: every B row becomes the
    xi-weighted mean of itself and the A rows attached to it.  All reads are of
    the values before the update; rows without incoming edges are returned as is."""
    num = Y * xi[:, None]
    den = xi.copy()
    has = np.zeros(Y.shape[0], dtype=bool)
    for a in np.nonzero(dst >= 0)[0]:
        b = int(dst[a])
        num[b] += xi[a] * Y[a]
        den[b] += xi[a]
        has[b] = True
    out = Y.copy()
    out[has] = num[has] / den[has][:, None]
    return out


def message_passing_edges(Y: np.ndarray, xi: np.ndarray, edges) -> np.ndarray:
    """Eq. (message-passing) for an adjacency matrix M with any number of ones per
    row: row b becomes (xi_b Y_b + sum_{a: M[a,b]=1} xi_a Y_a) / (xi_b + sum_{a: M[a,b]=1} xi_a).
    An A node with several selected edges contributes to each of its B nodes with
    its full weight.  All reads are of the values before the update."""
    num = Y * xi[:, None]
    den = xi.copy()
    has = np.zeros(Y.shape[0], dtype=bool)
    for a, b in edges:
        num[b] += xi[a] * Y[a]
        den[b] += xi[a]
        has[b] = True
    out = Y.copy()
    out[has] = num[has] / den[has][:, None]
    return out


def edges_csr(n: int, edges) -> Tuple[np.ndarray, np.ndarray]:
    """Sources of token b under an edge list: grp_src[grp_offsets[b]:grp_offsets[b+1]], ascending."""
    srcs: List[List[int]] = [[] for _ in range(n)]
    for a, b in edges:
        srcs[b].append(a)
    offs = np.zeros(n + 1, dtype=np.int32)
    for b in range(n):
        srcs[b].sort()
        offs[b + 1] = offs[b] + len(srcs[b])
    flat = np.array([a for l in srcs for a in l], dtype=np.int32).reshape(-1)
    return offs, flat


def removed_by_edges(n: int, edges) -> np.ndarray:
    """Steps 4-5 under an edge list: True for every A node with at least one selected edge."""
    gone = np.zeros(n, dtype=bool)
    for a, _ in edges:
        gone[a] = True
    return gone


def compact(Y: np.ndarray, dst: np.ndarray) -> np.ndarray:
    """Steps 4-5: drop merged A rows; R and B rows keep their relative order."""
    return Y[dst < 0]


@dataclass
class StageResult:
    xi: np.ndarray
    best_fd: np.ndarray
    best_dst: np.ndarray
    dst: np.ndarray
    new_index: np.ndarray
    grp_offsets: np.ndarray
    grp_src: np.ndarray
    X: np.ndarray       # float64, compacted, not yet rounded to storage
    K: np.ndarray
    V: np.ndarray
    pos: np.ndarray
    cu_vis: np.ndarray


def compress_stage(X, K, V, Q, pos, cu_vis, cu_txt, heads, head_dim, win_offsets, win_tokens,
                   win_remove, scale=None, lse=None, xi=None, metric: str = "cosine",
                   direction: str = "a_to_b") -> StageResult:
    """One whole compression step on float64 inputs (already widened from storage)."""
    if xi is None:
        xi = xi_text_query(Q, K, cu_vis, cu_txt, heads, head_dim, scale=scale, lse=lse)
    best_fd, best_dst = best_edges(X, win_offsets, win_tokens, metric, direction)
    dst = select(best_fd, best_dst, win_offsets, win_tokens, win_remove, direction)
    new_index = kept_index(dst)
    go, gs = groups_csr(dst)
    Xo = compact(message_passing(X, xi, dst), dst)
    Ko = compact(message_passing(K, xi, dst), dst)
    Vo = compact(message_passing(V, xi, dst), dst)
    keep = dst < 0
    cu_out = np.zeros_like(np.asarray(cu_vis, dtype=np.int32))
    for b in range(len(cu_vis) - 1):
        cu_out[b + 1] = cu_out[b] + int(keep[int(cu_vis[b]):int(cu_vis[b + 1])].sum())
    return StageResult(xi, best_fd, best_dst, dst, new_index, go, gs, Xo, Ko, Vo,
                       np.asarray(pos)[keep].astype(np.int32), cu_out)


@dataclass
class EdgeStageResult:
    xi: np.ndarray
    edges: list          # (a_token, b_token) pairs
    gone: np.ndarray     # bool per token
    new_index: np.ndarray
    grp_offsets: np.ndarray
    grp_src: np.ndarray
    X: np.ndarray
    K: np.ndarray
    V: np.ndarray
    pos: np.ndarray
    cu_vis: np.ndarray


def compress_stage_edges(X, K, V, Q, pos, cu_vis, cu_txt, heads, head_dim, win_offsets, win_tokens,
                         win_edges, scale=None, lse=None, xi=None, metric: str = "cosine") -> EdgeStageResult:
    """One whole compression step with Step 2 read literally (k lowest edges per window)."""
    if xi is None:
        xi = xi_text_query(Q, K, cu_vis, cu_txt, heads, head_dim, scale=scale, lse=lse)
    edges = select_edge_topk(X, win_offsets, win_tokens, win_edges, metric)
    n = X.shape[0]
    gone = removed_by_edges(n, edges)
    keep = ~gone
    new_index = np.where(keep, np.cumsum(keep) - 1, -1).astype(np.int32)
    go, gs = edges_csr(n, edges)
    Xo, Ko, Vo = (message_passing_edges(Y, xi, edges)[keep] for Y in (X, K, V))
    cu_out = np.zeros_like(np.asarray(cu_vis, dtype=np.int32))
    for b in range(len(cu_vis) - 1):
        cu_out[b + 1] = cu_out[b] + int(keep[int(cu_vis[b]):int(cu_vis[b + 1])].sum())
    return EdgeStageResult(xi, edges, gone, new_index, go, gs, Xo, Ko, Vo,
                           np.asarray(pos)[keep].astype(np.int32), cu_out)


def compress_stage_full_pairwise(X, K, V, Q, pos, cu_vis, cu_txt, heads, head_dim, win_offsets, win_tokens,
                                 win_remove, scale=None, lse=None, xi=None, metric: str = "cosine") -> StageResult:
    """One whole compression step with full pairwise matching inside every window (appendix ablation)."""
    if xi is None:
        xi = xi_text_query(Q, K, cu_vis, cu_txt, heads, head_dim, scale=scale, lse=lse)
    near_fd, near_dst = nearest_neighbours(X, win_offsets, win_tokens, metric)
    dst = select_full_pairwise(near_fd, near_dst, win_offsets, win_tokens, win_remove)
    new_index = kept_index(dst)
    go, gs = groups_csr(dst)
    Xo, Ko, Vo = (compact(message_passing(Y, xi, dst), dst) for Y in (X, K, V))
    keep = dst < 0
    cu_out = np.zeros_like(np.asarray(cu_vis, dtype=np.int32))
    for b in range(len(cu_vis) - 1):
        cu_out[b + 1] = cu_out[b] + int(keep[int(cu_vis[b]):int(cu_vis[b + 1])].sum())
    return StageResult(xi, near_fd, near_dst, dst, new_index, go, gs, Xo, Ko, Vo,
                       np.asarray(pos)[keep].astype(np.int32), cu_out)


def stage_removals(batch: int, n_in: int, n_out: int, windows_per_seq: int) -> np.ndarray:
    """Removal counts for all windows of a batch whose sequences all go n_in -> n_out, when no window's cap binds
    (equal windows of the first stage): the even spread."""
    one = removal_counts_even(n_in - n_out, windows_per_seq)
    return np.tile(one, batch)


def compress_schedule(wl, stages: Optional[int] = None, metric: str = "cosine",
                      direction: str = "a_to_b") -> List[StageResult]:
    """Runs the hierarchical schedule (Sec. 3.2.2) of a workload: after every stage the
    outputs are rounded to the storage dtype, as a KV cache would hold them."""
    X, K, V = wl.X, wl.K, wl.V
    pos, cu_vis = wl.pos, wl.cu_vis
    Q = widen(wl.Q, wl.dtype)
    out = []
    n_in = wl.n_per_seq
    for s in range(wl.stages if stages is None else stages):
        w = wl.windows_per_axis[s]
        wo, wt = build_windows(pos, cu_vis, wl.tiles, wl.grid_h, wl.grid_w, w)
        n_seq = np.diff(np.asarray(cu_vis, dtype=np.int64))
        rem, bad = removal_counts_target(wo, wl.batch, n_seq - wl.targets[s], direction)
        if bad.any():
            raise ValueError("stage %d: the windows cannot give up %s tokens" % (s, (n_seq - wl.targets[s]).tolist()))
        res = compress_stage(widen(X, wl.dtype), widen(K, wl.dtype), widen(V, wl.dtype), Q, pos, cu_vis,
                             wl.cu_txt, wl.heads, wl.head_dim, wo, wt, rem, metric=metric, direction=direction)
        out.append(res)
        X, K, V = (round_to_storage(t, wl.dtype) for t in (res.X, res.K, res.V))
        pos, cu_vis, n_in = res.pos, res.cu_vis, wl.targets[s]
    return out
