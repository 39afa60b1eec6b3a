"""MI355X-native frame-parallel GCN aggregation (PiPAD's parallel GNN hot path), HIP + C ABI.

The compute lives in ``libpipad.so`` (sources under ``csrc/``, contract in ``include/pipad.h``);
this package is the thin binding.  There is no CPU fallback.
"""
from .binding import (Frame, PipadError, frame_aggregate, frame_aggregate_subset, frame_aggregate_update,
                      frame_build_overlap, frame_transpose, get_option, load_library,
                      set_option)


def coalescent_row_bytes(snapshots: int, feat: int) -> int:
    """Bytes of one row of the coalescent feature operand: the feature rows of all snapshots of a
    group side by side, 4-byte floats (Section 4.2; sizes quoted in Section 5.3)."""
    return snapshots * feat * 4


def padded_row_stride(feat: int) -> int:
    """pipad_recommended_row_stride: the row stride, in floats, that a feature matrix whose rows are
    gathered should have (the smallest odd number of 128-byte lines that holds ``feat`` floats; the
    reason is in include/pipad.h)."""
    stride = int(load_library().pipad_recommended_row_stride(int(feat)))
    if stride < 0:
        raise ValueError("feat must be at least 1")
    return stride


__all__ = ["Frame", "PipadError", "frame_aggregate", "frame_aggregate_subset", "frame_aggregate_update", "frame_build_overlap", "frame_transpose", "get_option",
           "set_option", "load_library", "coalescent_row_bytes", "padded_row_stride"]
