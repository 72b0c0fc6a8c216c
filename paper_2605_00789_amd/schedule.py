"""Host-side names for the partition arithmetic of the hierarchical compression (paper Sec. 3.2.2): thin wrappers over
the library's own functions (the counts per window are computed on the device by lightkv_window_counts)."""
from __future__ import annotations

from . import binding as B


def windows_per_sequence(tiles: int, w: int) -> int:
    """w x w windows per image tile; w == 0 stands for one window over the whole sequence."""
    return B.lightkv_windows_per_sequence(tiles, w)


def max_window_cells(tiles: int, grid_h: int, grid_w: int, w: int) -> int:
    """Upper bound on the tokens of any window: the grid cells it covers."""
    return B.lightkv_max_window_cells(tiles, grid_h, grid_w, w)
