"""MI355X-native frame-parallel GCN aggregation (PiPAD's parallel GNN hot path), HIP + C ABI.

The compute lives in ``libpipad.so`` (sources under ``csrc/``, contract in ``include/pipad.h``);
this package is the thin binding.  There is no CPU fallback.
"""
from .binding import (Frame, PipadError, frame_aggregate, frame_build_overlap, get_option,
                      load_library, set_option)


def coalescent_row_bytes(snapshots: int, feat: int) -> int:
    """Bytes of one row of the coalescent feature operand: the feature rows of all snapshots of a
    group side by side, 4-byte floats (Section 4.2; sizes quoted in Section 5.3)."""
    return snapshots * feat * 4


__all__ = ["Frame", "PipadError", "frame_aggregate", "frame_build_overlap", "get_option",
           "set_option", "load_library", "coalescent_row_bytes"]
