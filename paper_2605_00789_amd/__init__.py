"""LightKV compression step for AMD MI355X: thin Python binding over liblightkv.so.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/lightkv.h; this package only marshals arguments and owns buffers.
There is no CPU fallback: importing `binding` without the built library raises.
"""
from .binding import (  # noqa: F401
    LightKVError,
    Problem,
    lib_path,
    lightkv_aggregate,
    lightkv_aggregate_compact,
    lightkv_build_windows,
    lightkv_build_windows_next,
    lightkv_compact,
    lightkv_score,
    lightkv_score_select,
    lightkv_select,
    lightkv_select_static,
    lightkv_status_string,
    lightkv_version,
    lightkv_workspace_size,
    lightkv_window_counts,
    lightkv_windows_per_sequence,
    lightkv_max_window_cells,
    XI_TEXT_QUERY,
    XI_VISION_QUERY,
    XI_GIVEN,
)
from .schedule import windows_per_sequence, max_window_cells  # noqa: F401
from .pipeline import CompressionPipeline, EdgeTopKSchedule, from_device, to_device  # noqa: F401
