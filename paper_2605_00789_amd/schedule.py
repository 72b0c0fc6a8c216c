"""Host-side schedule helpers of the hierarchical compression (paper Sec. 3.2.2):
how many windows a stage has and how many tokens each window gives up."""
from __future__ import annotations

import numpy as np


def windows_per_sequence(tiles: int, w: int) -> int:
    """w x w windows per image tile; w == 0 stands for one window over the whole sequence."""
    return 1 if w == 0 else tiles * w * w


def max_window_cells(tiles: int, grid_h: int, grid_w: int, w: int) -> int:
    """Upper bound on the tokens of any window: the grid cells it covers."""
    if w == 0:
        return tiles * grid_h * grid_w
    rows = max(len([r for r in range(grid_h) if r * w // grid_h == k]) for k in range(w))
    cols = max(len([c for c in range(grid_w) if c * w // grid_w == k]) for k in range(w))
    return rows * cols


def removal_counts(batch: int, n_in: int, n_out: int, win_per_seq: int) -> np.ndarray:
    """Tokens each window removes when every sequence goes from n_in to n_out tokens:
    the budget n_in - n_out is spread evenly, the first windows take the remainder."""
    total = n_in - n_out
    if total < 0:
        raise ValueError("a stage cannot add tokens")
    base, extra = divmod(total, win_per_seq)
    one = np.full(win_per_seq, base, dtype=np.int32)
    one[:extra] += 1
    return np.tile(one, batch)


def edge_counts(h_win_offsets: np.ndarray, rho: float) -> np.ndarray:
    """Edges taken per window when Step 2 is read literally (Sec. 3.2.1): floor(rho * v / 2) pairs for a window of v
    tokens, never more than the window has pairs."""
    v = np.diff(np.asarray(h_win_offsets, dtype=np.int64))
    k = np.floor(rho * v / 2.0 + 1e-9).astype(np.int64)
    return np.minimum(k, ((v + 1) // 2) * (v // 2)).astype(np.int32)
