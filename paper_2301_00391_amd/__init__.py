"""MI355X-native frame-parallel GCN aggregation (PiPAD's parallel GNN hot path), HIP + C ABI.

The compute lives in ``libpipad.so`` (sources under ``csrc/``, contract in ``include/pipad.h``);
this package is the thin binding.  There is no CPU fallback.
"""
from .binding import (Frame, PipadError, frame_aggregate, frame_aggregate_update,
                      frame_build_overlap, frame_transpose, get_option, load_library,
                      set_option)


def coalescent_row_bytes(snapshots: int, feat: int) -> int:
    """Bytes of one row of the coalescent feature operand: the feature rows of all snapshots of a
    group side by side, 4-byte floats (Section 4.2; sizes quoted in Section 5.3)."""
    return snapshots * feat * 4


def padded_row_stride(feat: int) -> int:
    """Row stride, in floats, for a feature matrix whose rows are gathered: the smallest odd
    multiple of 128 bytes that holds ``feat`` floats.  A power-of-two stride ties a row's memory
    channel to a few bits of the node id; when popular nodes share those bits (R-MAT ids do) their
    rows crowd onto a few channels.  An odd number of 128-byte lines per row spreads them evenly;
    the padding is never read."""
    lines = (feat * 4 + 127) // 128
    if lines % 2 == 0:
        lines += 1
    return lines * 32


__all__ = ["Frame", "PipadError", "frame_aggregate", "frame_aggregate_update", "frame_build_overlap", "frame_transpose", "get_option",
           "set_option", "load_library", "coalescent_row_bytes", "padded_row_stride"]
